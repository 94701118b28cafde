"""ctypes front end of the CPU oracle (swimba_oracle.c).  TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's cpu_baseline leg may
import this module; the product path never does.  It shares nothing with the
HIP library: it loads its own shared object, built from the one C file beside
it with gcc.

All tensor arguments are numpy arrays holding the exact stored values
(float32, or bf16 widened to float32).  Results are float64.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "swimba_oracle.c")
_LIB = os.path.join(_HERE, "libswimba_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


class _Dims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in
                ("batch", "seqlen", "nheads", "headdim", "dstate", "ngroups", "nexperts", "top_k")]


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.swimba_oracle_num_threads.restype = ctypes.c_int
    return _lib


def num_threads() -> int:
    return int(_load().swimba_oracle_num_threads())


def _f32(a) -> np.ndarray:
    a = np.asarray(a)
    out = np.ascontiguousarray(a, dtype=np.float32)
    if a.dtype != np.float32 and not np.array_equal(out.astype(np.float64), a.astype(np.float64),
                                                    equal_nan=True):
        raise ValueError("oracle inputs must be exactly representable in float32")
    return out


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def router(router_logits, top_k: int):
    """logits (..., E) -> (idx (..., k) int32, w (..., k) float64)."""
    g = _f32(router_logits)
    E = g.shape[-1]
    T = g.size // E if E else 0
    idx = np.zeros(g.shape[:-1] + (top_k,), dtype=np.int32)
    w = np.zeros(g.shape[:-1] + (top_k,), dtype=np.float64)
    rc = _load().swimba_oracle_router(_p(g), ctypes.c_int64(T), ctypes.c_int64(E),
                                      ctypes.c_int64(top_k), _p(idx), _p(w))
    if rc:
        raise ValueError("oracle router: bad arguments")
    return idx, w


def _dims_of(x, B_experts, top_k):
    B, L, H, P = x.shape
    Bb, Lb, E, G, N = B_experts.shape
    assert (Bb, Lb) == (B, L)
    return _Dims(B, L, H, P, N, G, E, top_k), (B, L, H, P, N, G, E)


def mixer_fwd(x, dt, A, D, B_experts, C_experts, router_logits, top_k: int,
              h0=None, snap_every: int = 0) -> Dict[str, np.ndarray]:
    """Mixed single-trajectory forward.  Shapes:
    x (B,L,H,P), dt (B,L,H), A (H), D (H) or None, B/C_experts (B,L,E,G,N),
    router_logits (B,L,E), h0 (B,H,P,N) or None.
    Returns y (B,L,H,P), h_final (B,H,P,N), topk_idx, topk_w (B,L,k) and, when
    snap_every > 0, snaps (B, ceil(L/snap_every), H, P, N): the state carried
    into each block of snap_every tokens.
    """
    x = _f32(x); dt = _f32(dt); A = _f32(A)
    D = None if D is None else _f32(D)
    Be = _f32(B_experts); Ce = _f32(C_experts); g = _f32(router_logits)
    dims, (B, L, H, P, N, G, E) = _dims_of(x, Be, top_k)
    assert dt.shape == (B, L, H) and A.shape == (H,) and Ce.shape == Be.shape and g.shape == (B, L, E)
    h0d = None if h0 is None else np.ascontiguousarray(h0, dtype=np.float64)
    if h0d is not None:
        assert h0d.shape == (B, H, P, N)
    y = np.zeros((B, L, H, P), dtype=np.float64)
    hf = np.zeros((B, H, P, N), dtype=np.float64)
    idx = np.zeros((B, L, top_k), dtype=np.int32)
    w = np.zeros((B, L, top_k), dtype=np.float64)
    snaps = None
    if snap_every > 0:
        snaps = np.zeros((B, (L + snap_every - 1) // snap_every, H, P, N), dtype=np.float64)
    rc = _load().swimba_oracle_mixer_fwd(ctypes.byref(dims), _p(x), _p(dt), _p(A), _p(D), _p(Be),
                                         _p(Ce), _p(g), _p(h0d), _p(y), _p(hf), _p(idx), _p(w),
                                         ctypes.c_int64(snap_every), _p(snaps))
    if rc:
        raise ValueError("oracle mixer_fwd: bad arguments")
    out = {"y": y, "h_final": hf, "topk_idx": idx, "topk_w": w}
    if snaps is not None:
        out["snaps"] = snaps
    return out


def mixer_fwd_xe(x_experts, dt, A, D, B_experts, C_experts, router_logits, top_k: int,
                 h0=None) -> Dict[str, np.ndarray]:
    """Mixed forward with one input stream per expert, x_experts (B,L,E,H,P): the injection
    is sum_e pi_e x^(e) (x) B^(e); the skip term sees sum_e pi_e x^(e).
    Returns y (B,L,H,P), h_final (B,H,P,N), topk_idx, topk_w."""
    xe = _f32(x_experts); dt = _f32(dt); A = _f32(A)
    D = None if D is None else _f32(D)
    Be = _f32(B_experts); Ce = _f32(C_experts); g = _f32(router_logits)
    B, L, E, H, P = xe.shape
    dims, (B, L, H, P, N, G, E) = _dims_of(np.empty((B, L, H, P), dtype=np.float32), Be, top_k)
    assert xe.shape == (B, L, E, H, P)
    h0 = None if h0 is None else np.ascontiguousarray(h0, dtype=np.float64)
    y = np.zeros((B, L, H, P), dtype=np.float64)
    hf = np.zeros((B, H, P, N), dtype=np.float64)
    idx = np.zeros((B, L, top_k), dtype=np.int32)
    w = np.zeros((B, L, top_k), dtype=np.float64)
    rc = _load().swimba_oracle_mixer_fwd_xe(ctypes.byref(dims), _p(xe), _p(dt), _p(A), _p(D), _p(Be), _p(Ce),
                                            _p(g), _p(h0), _p(y), _p(hf), _p(idx), _p(w))
    if rc:
        raise ValueError("oracle mixer_fwd_xe: bad arguments")
    return {"y": y, "h_final": hf, "topk_idx": idx, "topk_w": w}


def expert_proj(u, W_B, W_C, router_logits, top_k: int, fill=np.nan):
    """Routed expert in-projection.  u (B,L,Dm), W_B/W_C (E,G,N,Dm), router_logits (B,L,E)
    -> B_experts, C_experts (B,L,E,G,N) float64 with the rows of the active experts computed and
    every other row equal to `fill`; topk_idx, topk_w."""
    u = _f32(u); WB = _f32(W_B); WC = _f32(W_C); g = _f32(router_logits)
    B, L, Dm = u.shape
    E, G, N, Dm2 = WB.shape
    assert Dm2 == Dm and WC.shape == WB.shape and g.shape == (B, L, E)
    Be = np.full((B, L, E, G, N), fill, dtype=np.float64)
    Ce = np.full((B, L, E, G, N), fill, dtype=np.float64)
    idx = np.zeros((B, L, top_k), dtype=np.int32)
    w = np.zeros((B, L, top_k), dtype=np.float64)
    i64 = ctypes.c_int64
    rc = _load().swimba_oracle_expert_proj(i64(B * L), i64(Dm), i64(E), i64(top_k), i64(G * N), _p(u), _p(WB),
                                           _p(WC), _p(g), _p(Be), _p(Ce), _p(idx), _p(w))
    if rc:
        raise ValueError("oracle expert_proj: bad arguments")
    return {"B_experts": Be, "C_experts": Ce, "topk_idx": idx, "topk_w": w}


def expert_proj_x(u, W_X, router_logits, top_k: int):
    """Routed in-projection of the input streams.  u (B,L,Dm), W_X (E,H,P,Dm), router_logits (B,L,E)
    -> x_sel (B,L,k,H,P) float64, row r = the token's r-th active expert; topk_idx, topk_w."""
    u = _f32(u); WX = _f32(W_X); g = _f32(router_logits)
    B, L, Dm = u.shape
    E, H, P, Dm2 = WX.shape
    assert Dm2 == Dm and g.shape == (B, L, E)
    xs = np.zeros((B, L, top_k, H, P), dtype=np.float64)
    idx = np.zeros((B, L, top_k), dtype=np.int32)
    w = np.zeros((B, L, top_k), dtype=np.float64)
    i64 = ctypes.c_int64
    rc = _load().swimba_oracle_expert_proj_x(i64(B * L), i64(Dm), i64(E), i64(top_k), i64(H * P), _p(u), _p(WX),
                                             _p(g), _p(xs), _p(idx), _p(w))
    if rc:
        raise ValueError("oracle expert_proj_x: bad arguments")
    return {"x_sel": xs, "topk_idx": idx, "topk_w": w}


def router_linear(u, W_g) -> np.ndarray:
    """Routing logits g = W_g u for every token: u (B,L,Dm), W_g (E,Dm) -> (B,L,E) float64."""
    u = _f32(u); Wg = _f32(W_g)
    B, L, Dm = u.shape
    E, Dm2 = Wg.shape
    assert Dm2 == Dm
    g = np.zeros((B, L, E), dtype=np.float64)
    i64 = ctypes.c_int64
    rc = _load().swimba_oracle_router_linear(i64(B * L), i64(Dm), i64(E), _p(u), _p(Wg), _p(g))
    if rc:
        raise ValueError("oracle router_linear: bad arguments")
    return g


def separated_fwd(x, dt, A, D, B_experts, C_experts, router_logits, top_k: int) -> Dict[str, np.ndarray]:
    """MoE of separated SSMs (one trajectory per expert, zero initial states).
    Returns y (B,L,H,P), h_final (B,E,H,P,N), topk_idx, topk_w."""
    x = _f32(x); dt = _f32(dt); A = _f32(A)
    D = None if D is None else _f32(D)
    Be = _f32(B_experts); Ce = _f32(C_experts); g = _f32(router_logits)
    dims, (B, L, H, P, N, G, E) = _dims_of(x, Be, top_k)
    y = np.zeros((B, L, H, P), dtype=np.float64)
    hf = np.zeros((B, E, H, P, N), dtype=np.float64)
    idx = np.zeros((B, L, top_k), dtype=np.int32)
    w = np.zeros((B, L, top_k), dtype=np.float64)
    rc = _load().swimba_oracle_separated_fwd(ctypes.byref(dims), _p(x), _p(dt), _p(A), _p(D), _p(Be),
                                             _p(Ce), _p(g), _p(y), _p(hf), _p(idx), _p(w))
    if rc:
        raise ValueError("oracle separated_fwd: bad arguments")
    return {"y": y, "h_final": hf, "topk_idx": idx, "topk_w": w}


def step(state, x, dt, A, D, B_experts, C_experts, router_logits, top_k: int):
    """One decode token = one iteration of the recurrence.
    state (B,H,P,N) float64, x (B,H,P), dt (B,H), B/C_experts (B,E,G,N),
    router_logits (B,E).  Returns (y (B,H,P), state' (B,H,P,N), idx (B,k))."""
    x = np.asarray(x); dt = np.asarray(dt)
    r = mixer_fwd(x[:, None], dt[:, None], A, D, np.asarray(B_experts)[:, None],
                  np.asarray(C_experts)[:, None], np.asarray(router_logits)[:, None], top_k, h0=state)
    return r["y"][:, 0], r["h_final"], r["topk_idx"][:, 0]
