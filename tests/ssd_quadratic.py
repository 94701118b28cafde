"""Independent numpy evaluators used only to pin the CPU oracle.

They follow different formulas than the oracle's token-by-token loop:
  * the router/mix is written with a stable sort and dense one-hot weights;
  * the SSM is evaluated in its quadratic "Y = M X" form (SSD background
    section: M is the semiseparable matrix masked by the decay), which comes
    from unrolling the recurrence, h_t = sum_i A^{t-i} U_i (proof of the
    stability theorem).
Only suitable for tiny inputs (O(L^2) memory per head).
"""
import numpy as np


def dense_router_weights(logits, top_k):
    """(…,E) logits -> (…,E) weights: softmax over all experts, zeroed outside
    the top_k set, not renormalised.  Ties go to the lower index."""
    g = np.asarray(logits, dtype=np.float64)
    E = g.shape[-1]
    z = np.exp(g - g.max(axis=-1, keepdims=True))
    pi = z / z.sum(axis=-1, keepdims=True)
    # stable argsort of -g: equal logits keep ascending index order
    order = np.argsort(-g, axis=-1, kind="stable")
    keep = np.zeros(g.shape, dtype=bool)
    np.put_along_axis(keep, order[..., :top_k], True, axis=-1)
    return np.where(keep, pi, 0.0), order[..., :top_k]


def mix_streams(S_experts, weights):
    """S_experts (B,L,E,G,N), weights (B,L,E) -> (B,L,G,N)."""
    return np.einsum("blegn,ble->blgn", np.asarray(S_experts, dtype=np.float64), weights)


def ssd_quadratic(x, dt, A, D, Bm, Cm):
    """Plain selective SSM with premixed streams, zero initial state.
    x (B,L,H,P), dt (B,L,H), A (H), D (H), Bm/Cm (B,L,G,N) -> y (B,L,H,P)."""
    x = np.asarray(x, dtype=np.float64)
    dt = np.asarray(dt, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    B_, L, H, P = x.shape
    G = Bm.shape[2]
    y = np.zeros_like(x)
    for b in range(B_):
        for h in range(H):
            q = (h * G) // H
            a = dt[b, :, h] * A[h]
            # Lambda[t, s] = exp(sum_{r=s+1..t} a_r) for t >= s, else 0
            lam = np.zeros((L, L))
            for t in range(L):
                for s in range(t + 1):
                    lam[t, s] = np.exp(a[s + 1:t + 1].sum())
            M = lam * (Cm[b, :, q, :] @ Bm[b, :, q, :].T)
            y[b, :, h, :] = M @ (dt[b, :, h, None] * x[b, :, h, :])
            if D is not None:
                y[b, :, h, :] += D[h] * x[b, :, h, :]
    return y


def swimba_quadratic(x, dt, A, D, Be, Ce, logits, top_k):
    wts, order = dense_router_weights(logits, top_k)
    return ssd_quadratic(x, dt, A, D, mix_streams(Be, wts), mix_streams(Ce, wts)), order


def swimba_quadratic_xe(x_experts, dt, A, D, Be, Ce, logits, top_k):
    """Expert-specific input streams, x_experts (B,L,E,H,P), quadratic form:
    y_t = sum_{s<=t} Lambda[t,s] dt_s sum_e w_{s,e} (Cmix_t . B_s^(e)) x_s^(e)  +  D xbar_t,
    xbar = sum_e w_e x^(e): the k outer products of a token enter as k separate columns
    of the masked matrix product (one term per expert, dense over all E with zero weights)."""
    xe = np.asarray(x_experts, dtype=np.float64)
    dt = np.asarray(dt, dtype=np.float64)
    A = np.asarray(A, dtype=np.float64)
    Be = np.asarray(Be, dtype=np.float64)
    wts, order = dense_router_weights(logits, top_k)
    Cm = mix_streams(Ce, wts)
    B_, L, E, H, P = xe.shape
    G = Be.shape[3]
    y = np.zeros((B_, L, H, P))
    for b in range(B_):
        for h in range(H):
            q = (h * G) // H
            a = dt[b, :, h] * A[h]
            cum = np.concatenate([[0.0], np.cumsum(a)])
            lam = np.tril(np.exp(np.subtract.outer(cum[1:], cum[1:])))   # exp(sum_{s+1..t} a)
            for e in range(E):
                M = lam * (Cm[b, :, q, :] @ Be[b, :, e, q, :].T)
                y[b, :, h, :] += M @ ((dt[b, :, h] * wts[b, :, e])[:, None] * xe[b, :, e, h, :])
            if D is not None:
                y[b, :, h, :] += D[h] * np.einsum("le,lep->lp", wts[b], xe[b, :, :, h, :])
    return y, order
