/*
 * CPU oracle for the Swimba token mixer.  TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, sequential evaluation of the method in double precision,
 * written from the paper's definitions.  It shares no code with the HIP
 * library and must never be called from the product path: only the tests,
 * the smoke check and the benchmark's cpu_baseline leg may use it.
 *
 * What it evaluates (paper sections "Mixture of Experts and Switching
 * Dynamics", "Selective SSM and SSD", "MoE-parameterized SSM" and
 * "Alternative: MoE of separated SSMs"):
 *
 *   router      pi_t = softmax(g_t) over all E experts (router softmax
 *               equation); K_t = the top_k largest logits; the softmax values
 *               are kept on K_t and NOT renormalised.
 *   mixing      Bmix_t = sum_{e in K_t} pi_{t,e} B_t^(e),
 *               Cmix_t = sum_{e in K_t} pi_{t,e} C_t^(e)       (Theorem 1)
 *   recurrence  h_t = exp(dt_t A_h) h_{t-1} + dt_t Bmix_t x_t^T (mixed state
 *               update equation, with the scalar-identity transition of SSD
 *               and Mamba-2's dt-scaled injection)
 *   readout     y_t = Cmix_t . h_t + D_h x_t     (mixed readout equation; the
 *               state is read AFTER its update, as in the selective SSM
 *               equation y_t = C_t^T h_t)
 *   separated   h_t^(e) = exp(dt_t A_h) h_{t-1}^(e) + dt_t B_t^(e) x_t^T for
 *               every expert e, y_t = sum_{e in K_t} pi_{t,e} C_t^(e) . h_t^(e)
 *               + D_h x_t                       (separated-SSM equation)
 *   projection  B_t^(e), C_t^(e) for the active experts only, as expert-specific
 *               linear maps of the token features (swimba_oracle_expert_proj), and the
 *               input streams x_t^(e) of the active experts the same way, stored per
 *               selected slot (swimba_oracle_expert_proj_x)
 *   router map  g_t = W_g u_t, the routing logits as a linear function of the
 *               token features (swimba_oracle_router_linear)
 *   expert x    the mixed state update in its full form, with one input stream
 *               per expert: h_t = exp(dt_t A_h) h_{t-1}
 *               + dt_t sum_{e in K_t} pi_{t,e} x_t^(e) (x) B_t^(e); same readout
 *               (swimba_oracle_mixer_fwd_xe)
 *
 * Readings where the paper is silent (kept in step with the design notes):
 *   - ties between equal logits go to the lower expert index, and the active
 *     set is reported in (logit descending, index ascending) order;
 *   - the transition is one negative scalar A_h per head, time variation comes
 *     only from dt; dt is a single positive stream, not routed;
 *   - x is shared by the experts (the API has one x), so the mixed injection
 *     is the rank-1 term dt Bmix x^T; the expert-x function takes the paper's
 *     per-expert input streams instead, and its skip term D_h multiplies the
 *     mixed input sum_{e in K_t} pi_{t,e} x_t^(e) (the paper has no skip term);
 *   - B/C streams come per group, head h reads group floor(h*G/H);
 *   - D is a per-head skip coefficient (NULL means 0);
 *   - the state starts at h0 (NULL means zeros).
 *
 * Inputs are float arrays holding the exact stored values (fp32, or bf16
 * widened to fp32); every product and sum is done in double.
 *
 * Pins (tests/test_oracle_pins.py): the sigmoid worked example of the
 * expressivity theorem's proof, the geometric-series closed form, the
 * quadratic masked form Y = M X on tiny inputs, the E=1 / one-hot / identical
 * expert reductions to a plain selective SSM, linearity in x, the
 * separated-vs-mixed equality regime, the BIBO bound, brute-force top-k; the
 * two linear maps against an independent library contraction and hand values.
 * Nothing here is "parity unpinned".
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int64_t batch, seqlen, nheads, headdim, dstate, ngroups, nexperts, top_k;
} oracle_dims;

int swimba_oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Router for one token: g[E] -> idx[k], w[k]. */
static void route_token(const float *g, int64_t E, int64_t k, int32_t *idx, double *w)
{
    double m = -INFINITY, Z = 0.0;
    for (int64_t e = 0; e < E; ++e)
        if ((double)g[e] > m) m = (double)g[e];
    for (int64_t e = 0; e < E; ++e)
        Z += exp((double)g[e] - m);
    /* k rounds of "largest logit not yet taken"; strict > keeps the lowest
       index among equal logits (and treats +0 and -0 as equal). */
    for (int64_t r = 0; r < k; ++r) {
        int64_t best = -1;
        for (int64_t e = 0; e < E; ++e) {
            int taken = 0;
            for (int64_t s = 0; s < r; ++s)
                if (idx[s] == (int32_t)e) taken = 1;
            if (taken) continue;
            if (best < 0 || g[e] > g[best]) best = e;
        }
        idx[r] = (int32_t)best;
        w[r] = exp((double)g[best] - m) / Z;
    }
}

/* logits (T,E) -> idx (T,k), w (T,k) */
int swimba_oracle_router(const float *logits, int64_t T, int64_t E, int64_t k,
                         int32_t *idx, double *w)
{
    if (!logits || !idx || !w || E < 1 || k < 1 || k > E || T < 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        route_token(logits + t * E, E, k, idx + t * k, w + t * k);
    return 0;
}

/*
 * Mixed (single-trajectory) forward.
 *   x (B,L,H,P)  dt (B,L,H)  A (H)  D (H)|NULL  Be,Ce (B,L,E,G,N)  logits (B,L,E)
 *   h0 (B,H,P,N)|NULL
 *   y (B,L,H,P)  h_final (B,H,P,N)|NULL  idx (B,L,k)  w (B,L,k)
 *   snaps: if snap_every > 0, (B, ceil(L/snap_every), H, P, N): the state
 *          BEFORE token c*snap_every is consumed (the state carried into
 *          block c).
 */
int swimba_oracle_mixer_fwd(const oracle_dims *d, const float *x, const float *dt,
                            const float *A, const float *D, const float *Be, const float *Ce,
                            const float *logits, const double *h0, double *y, double *h_final,
                            int32_t *idx, double *w, int64_t snap_every, double *snaps)
{
    const int64_t B = d->batch, L = d->seqlen, H = d->nheads, P = d->headdim, N = d->dstate,
                  G = d->ngroups, E = d->nexperts, k = d->top_k;
    if (B < 0 || L < 0 || H < 1 || P < 1 || N < 1 || G < 1 || E < 1 || k < 1 || k > E || H % G)
        return 1;
    if (swimba_oracle_router(logits, B * L, E, k, idx, w)) return 1;
    const int64_t nsnap = snap_every > 0 ? (L + snap_every - 1) / snap_every : 0;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < B * H; ++bh) {
        const int64_t b = bh / H, h = bh % H, q = (h * G) / H;
        double *st = (double *)malloc(sizeof(double) * P * N);
        double *Bm = (double *)malloc(sizeof(double) * N);
        double *Cm = (double *)malloc(sizeof(double) * N);
        for (int64_t i = 0; i < P * N; ++i) st[i] = h0 ? h0[(b * H + h) * P * N + i] : 0.0;

        for (int64_t t = 0; t < L; ++t) {
            const int64_t bt = b * L + t;
            if (snap_every > 0 && t % snap_every == 0)
                memcpy(snaps + (((b * nsnap + t / snap_every) * H + h) * P * N), st,
                       sizeof(double) * P * N);
            /* parameter-space mixing of the injection and readout streams */
            for (int64_t n = 0; n < N; ++n) { Bm[n] = 0.0; Cm[n] = 0.0; }
            for (int64_t r = 0; r < k; ++r) {
                const int64_t e = idx[bt * k + r];
                const double pi = w[bt * k + r];
                const float *be = Be + ((bt * E + e) * G + q) * N;
                const float *ce = Ce + ((bt * E + e) * G + q) * N;
                for (int64_t n = 0; n < N; ++n) {
                    Bm[n] += pi * (double)be[n];
                    Cm[n] += pi * (double)ce[n];
                }
            }
            /* one step of the single recurrence, then the readout */
            const double dtt = (double)dt[bt * H + h];
            const double a = exp(dtt * (double)A[h]);
            for (int64_t p = 0; p < P; ++p) {
                const double xv = (double)x[(bt * H + h) * P + p];
                const double u = dtt * xv;
                double *sp = st + p * N;
                double acc = 0.0;
                for (int64_t n = 0; n < N; ++n) {
                    sp[n] = a * sp[n] + u * Bm[n];
                    acc += Cm[n] * sp[n];
                }
                y[(bt * H + h) * P + p] = acc + (D ? (double)D[h] * xv : 0.0);
            }
        }
        if (h_final) memcpy(h_final + (b * H + h) * P * N, st, sizeof(double) * P * N);
        free(st); free(Bm); free(Cm);
    }
    return 0;
}

/*
 * Mixed forward with expert-specific input streams (paper: mixed state update
 * equation in its full form, every expert brings its own X stream):
 *   h_t = exp(dt_t A_h) h_{t-1} + dt_t sum_{e in K_t} pi_{t,e} x_t^(e) (x) B_t^(e)
 *   y_t = (sum_{e in K_t} pi_{t,e} C_t^(e)) . h_t + D_h xbar_t,
 *   xbar_t = sum_{e in K_t} pi_{t,e} x_t^(e)    (the skip term sees the mixed input)
 * The injection is a sum of k outer products per token (rank k), the state is one.
 *   xe (B,L,E,H,P); everything else as in swimba_oracle_mixer_fwd.
 */
int swimba_oracle_mixer_fwd_xe(const oracle_dims *d, const float *xe, const float *dt,
                               const float *A, const float *D, const float *Be, const float *Ce,
                               const float *logits, const double *h0, double *y, double *h_final,
                               int32_t *idx, double *w)
{
    const int64_t B = d->batch, L = d->seqlen, H = d->nheads, P = d->headdim, N = d->dstate,
                  G = d->ngroups, E = d->nexperts, k = d->top_k;
    if (B < 0 || L < 0 || H < 1 || P < 1 || N < 1 || G < 1 || E < 1 || k < 1 || k > E || H % G)
        return 1;
    if (swimba_oracle_router(logits, B * L, E, k, idx, w)) return 1;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < B * H; ++bh) {
        const int64_t b = bh / H, h = bh % H, q = (h * G) / H;
        double *st = (double *)malloc(sizeof(double) * P * N);
        double *Cm = (double *)malloc(sizeof(double) * N);
        for (int64_t i = 0; i < P * N; ++i) st[i] = h0 ? h0[(b * H + h) * P * N + i] : 0.0;

        for (int64_t t = 0; t < L; ++t) {
            const int64_t bt = b * L + t;
            const double dtt = (double)dt[bt * H + h];
            const double a = exp(dtt * (double)A[h]);
            /* decay, then the k weighted outer products of the active experts */
            for (int64_t i = 0; i < P * N; ++i) st[i] *= a;
            for (int64_t n = 0; n < N; ++n) Cm[n] = 0.0;
            for (int64_t r = 0; r < k; ++r) {
                const int64_t e = idx[bt * k + r];
                const double pi = w[bt * k + r];
                const float *be = Be + ((bt * E + e) * G + q) * N;
                const float *ce = Ce + ((bt * E + e) * G + q) * N;
                const float *xr = xe + ((bt * E + e) * H + h) * P;
                for (int64_t n = 0; n < N; ++n) Cm[n] += pi * (double)ce[n];
                for (int64_t p = 0; p < P; ++p) {
                    const double u = dtt * pi * (double)xr[p];
                    double *sp = st + p * N;
                    for (int64_t n = 0; n < N; ++n) sp[n] += u * (double)be[n];
                }
            }
            for (int64_t p = 0; p < P; ++p) {
                const double *sp = st + p * N;
                double acc = 0.0, xbar = 0.0;
                for (int64_t n = 0; n < N; ++n) acc += Cm[n] * sp[n];
                for (int64_t r = 0; r < k; ++r)
                    xbar += w[bt * k + r] * (double)xe[((bt * E + idx[bt * k + r]) * H + h) * P + p];
                y[(bt * H + h) * P + p] = acc + (D ? (double)D[h] * xbar : 0.0);
            }
        }
        if (h_final) memcpy(h_final + (b * H + h) * P * N, st, sizeof(double) * P * N);
        free(st); free(Cm);
    }
    return 0;
}

/*
 * Routed expert in-projection (paper, MoE-parameterized SSM: the expert streams are
 * expert-specific linear projections of the same token features; only the experts of the
 * active set K_t enter the mix, so only their rows are needed):
 *   for every token t and every e in K_t:
 *     B_t^(e)[c] = sum_d WB[e][c][d] u_t[d],   C_t^(e)[c] = sum_d WC[e][c][d] u_t[d]
 *   u (T,Dm)  WB, WC (E, GN, Dm)  logits (T,E)  ->  Be, Ce (T,E,GN): rows of the active
 *   experts are written (double), all other rows are left as they are.
 */
int swimba_oracle_expert_proj(int64_t T, int64_t Dm, int64_t E, int64_t k, int64_t GN,
                              const float *u, const float *WB, const float *WC,
                              const float *logits, double *Be, double *Ce, int32_t *idx, double *w)
{
    if (T < 0 || Dm < 1 || GN < 1 || E < 1 || k < 1 || k > E) return 1;
    if (swimba_oracle_router(logits, T, E, k, idx, w)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t r = 0; r < k; ++r) {
            const int64_t e = idx[t * k + r];
            for (int64_t c = 0; c < GN; ++c) {
                const float *wb = WB + (e * GN + c) * Dm;
                const float *wc = WC + (e * GN + c) * Dm;
                double sb = 0.0, sc = 0.0;
                for (int64_t d = 0; d < Dm; ++d) {
                    sb += (double)wb[d] * (double)u[t * Dm + d];
                    sc += (double)wc[d] * (double)u[t * Dm + d];
                }
                Be[(t * E + e) * GN + c] = sb;
                Ce[(t * E + e) * GN + c] = sc;
            }
        }
    }
    return 0;
}

/*
 * Routed in-projection of the input streams (paper, MoE-parameterized SSM: the experts also emit
 * X^(e), an expert-specific linear map of the token features, and the mixed state update injects
 * the products B^(e) X^(e) of the active set):
 *   x_t^(e_r)[c] = sum_d WX[e_r][c][d] u_t[d]     for the token's r-th active expert e_r
 *   u (T,Dm)  WX (E, HP, Dm)  logits (T,E)  ->  Xsel (T, k, HP) double, row r of a token belongs
 *   to its r-th active expert in router order (no array with an expert axis is formed).
 */
int swimba_oracle_expert_proj_x(int64_t T, int64_t Dm, int64_t E, int64_t k, int64_t HP,
                                const float *u, const float *WX, const float *logits,
                                double *Xsel, int32_t *idx, double *w)
{
    if (T < 0 || Dm < 1 || HP < 1 || E < 1 || k < 1 || k > E) return 1;
    if (swimba_oracle_router(logits, T, E, k, idx, w)) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t r = 0; r < k; ++r) {
            const int64_t e = idx[t * k + r];
            for (int64_t c = 0; c < HP; ++c) {
                const float *wx = WX + (e * HP + c) * Dm;
                double sx = 0.0;
                for (int64_t d = 0; d < Dm; ++d) sx += (double)wx[d] * (double)u[t * Dm + d];
                Xsel[(t * k + r) * HP + c] = sx;
            }
        }
    }
    return 0;
}

/*
 * Routing logits as a linear function of the token features (paper: the expressivity
 * theorem assumes g a linear function of the features; the Swimba layer's router selects
 * among the in-projection experts from the token's hidden state):
 *   g_t[e] = sum_d Wg[e][d] u_t[d]        u (T,Dm)  Wg (E,Dm)  ->  g (T,E) double
 * No bias, no temperature.
 */
int swimba_oracle_router_linear(int64_t T, int64_t Dm, int64_t E, const float *u, const float *Wg, double *g)
{
    if (T < 0 || Dm < 1 || E < 1) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t) {
        for (int64_t e = 0; e < E; ++e) {
            double sum = 0.0;
            for (int64_t d = 0; d < Dm; ++d) sum += (double)Wg[e * Dm + d] * (double)u[t * Dm + d];
            g[t * E + e] = sum;
        }
    }
    return 0;
}

/*
 * MoE of separated SSMs: one state per expert, every expert advances on every
 * token with its own B stream; the readout sums the active experts only.
 *   h_final (B,E,H,P,N)|NULL
 */
int swimba_oracle_separated_fwd(const oracle_dims *d, const float *x, const float *dt,
                                const float *A, const float *D, const float *Be, const float *Ce,
                                const float *logits, double *y, double *h_final,
                                int32_t *idx, double *w)
{
    const int64_t B = d->batch, L = d->seqlen, H = d->nheads, P = d->headdim, N = d->dstate,
                  G = d->ngroups, E = d->nexperts, k = d->top_k;
    if (B < 0 || L < 0 || H < 1 || P < 1 || N < 1 || G < 1 || E < 1 || k < 1 || k > E || H % G)
        return 1;
    if (swimba_oracle_router(logits, B * L, E, k, idx, w)) return 1;

#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t bh = 0; bh < B * H; ++bh) {
        const int64_t b = bh / H, h = bh % H, q = (h * G) / H;
        double *st = (double *)calloc((size_t)(E * P * N), sizeof(double));
        for (int64_t t = 0; t < L; ++t) {
            const int64_t bt = b * L + t;
            const double dtt = (double)dt[bt * H + h];
            const double a = exp(dtt * (double)A[h]);
            for (int64_t e = 0; e < E; ++e) {
                const float *be = Be + ((bt * E + e) * G + q) * N;
                for (int64_t p = 0; p < P; ++p) {
                    const double u = dtt * (double)x[(bt * H + h) * P + p];
                    double *sp = st + (e * P + p) * N;
                    for (int64_t n = 0; n < N; ++n) sp[n] = a * sp[n] + u * (double)be[n];
                }
            }
            for (int64_t p = 0; p < P; ++p) {
                const double xv = (double)x[(bt * H + h) * P + p];
                double acc = 0.0;
                for (int64_t r = 0; r < k; ++r) {
                    const int64_t e = idx[bt * k + r];
                    const double pi = w[bt * k + r];
                    const float *ce = Ce + ((bt * E + e) * G + q) * N;
                    const double *sp = st + (e * P + p) * N;
                    double dot = 0.0;
                    for (int64_t n = 0; n < N; ++n) dot += (double)ce[n] * sp[n];
                    acc += pi * dot;
                }
                y[(bt * H + h) * P + p] = acc + (D ? (double)D[h] * xv : 0.0);
            }
        }
        if (h_final)
            for (int64_t e = 0; e < E; ++e)
                memcpy(h_final + (((b * E + e) * H + h) * P * N), st + e * P * N,
                       sizeof(double) * P * N);
        free(st);
    }
    return 0;
}
