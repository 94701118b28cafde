// Internal declarations shared by the HIP translation units of libswimba.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "swimba.h"

namespace swimba {

// ---- storage types -------------------------------------------------------
struct bf16 {
    uint16_t bits;
};

__device__ __forceinline__ float to_float(float v) { return v; }
__device__ __forceinline__ float to_float(bf16 v) { return __uint_as_float((uint32_t)v.bits << 16); }

// fp32 -> bf16, round to nearest even (NaN stays NaN)
__device__ __forceinline__ uint16_t bf16_bits_rne(float f)
{
    uint32_t u = __float_as_uint(f);
    if ((u & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((u >> 16) | 0x0040u);
    u += 0x7fffu + ((u >> 16) & 1u);
    return (uint16_t)(u >> 16);
}

template <typename T> __device__ __forceinline__ T from_float(float v);
template <> __device__ __forceinline__ float from_float<float>(float v) { return v; }
template <> __device__ __forceinline__ bf16 from_float<bf16>(float v) { return bf16{bf16_bits_rne(v)}; }

// ---- problem description passed to kernels ------------------------------------
struct Shape {
    int B, L, H, P, N, G, E, K, Q, nc;
};

inline Shape make_shape(const swimba_dims *d)
{
    Shape s;
    s.B = d->batch; s.L = d->seqlen; s.H = d->nheads; s.P = d->headdim; s.N = d->dstate;
    s.G = d->ngroups; s.E = d->nexperts; s.K = d->top_k; s.Q = d->chunk;
    s.nc = (d->chunk > 0) ? (d->seqlen + d->chunk - 1) / d->chunk : 0;
    return s;
}

// true when the bf16 MFMA kernels cover this problem
inline bool use_mfma_path(const swimba_dims *d)
{
    // head dimensions below 64 and state sizes below 128 (multiples of 8) run on the same kernels:
    // x is staged with zero channels, the mixed rows and the states are zero-padded to 64 x 128
    return d->io_dtype == SWIMBA_BF16 && d->headdim <= 64 && d->headdim % 8 == 0 && d->dstate <= 128 &&
           d->dstate % 8 == 0 &&
           (d->chunk == 64 || d->chunk == 128 || d->chunk == 256);
}

void set_last_hip_error(int e);

#define SWIMBA_CHECK_LAUNCH()                                  \
    do {                                                       \
        hipError_t e__ = hipGetLastError();                    \
        if (e__ != hipSuccess) {                               \
            ::swimba::set_last_hip_error((int)e__);            \
            return SWIMBA_ERR_HIP;                             \
        }                                                      \
    } while (0)

// ---- kernel launchers (one per translation unit) ----------------------------------
swimba_status launch_router(int64_t tokens, int E, int K, int io_dtype, const void *logits,
                            int32_t *idx, float *w, hipStream_t st);
swimba_status launch_router_linear(int64_t tokens, int Dm, int E, int io_dtype, const void *u, const void *Wg,
                                   void *logits, hipStream_t st);
swimba_status launch_cumsum(const Shape &s, int io_dtype, const void *dt, const float *A, float *cs,
                            hipStream_t st);
swimba_status launch_state_scan(const Shape &s, const float *h0, float *h_final, float *states,
                                void *states_lp, const float *cs, hipStream_t st);
swimba_status launch_chunk_state_generic(const Shape &s, int io_dtype, const void *x, const void *dt,
                                         const void *Be, const int32_t *idx, const float *w,
                                         const float *cs, float *states, hipStream_t st);
swimba_status launch_output_generic(const Shape &s, int io_dtype, const void *x, const void *dt,
                                    const float *D, const void *Be, const void *Ce,
                                    const int32_t *idx, const float *w, const float *wc,
                                    const float *cs, const float *states, void *y, const float *skip_w,
                                    int skip_stride, int accumulate, hipStream_t st);
swimba_status launch_mix_rows_mfma(const Shape &s, const void *Be, const void *Ce, const void *logits,
                                   int32_t *idx, float *w, void *cmix, void *bfrag, void *bmix_t8,
                                   int sep_e, int slot, const float *w_sel, hipStream_t st);
// routed expert in-projection (expert_proj.hip)
swimba_status launch_expert_proj(int64_t tokens, int E, int K, int GN, int Dm, int io_dtype, const void *u,
                                 const void *WB, const void *WC, const void *logits, void *Be, void *Ce,
                                 int32_t *idx, float *w, int32_t *counts, int32_t *lists, int compact,
                                 hipStream_t st, const void *WX = nullptr, void *Xo = nullptr, int HP = 0);
bool expert_proj_on_mfma(int io_dtype, int GN, int HP, int Dm);
swimba_status launch_slot_ids(int32_t *idx, int64_t tokens, int K, hipStream_t st);
// expert-specific input streams (xe.hip)
swimba_status launch_xe_gather(const Shape &s, int io_dtype, int slot, const void *x_experts,
                               const int32_t *idx, void *xg, hipStream_t st);
swimba_status launch_xe_slot_weights(const Shape &s, int slot, const float *w, float *wslot, hipStream_t st);
swimba_status launch_sep_prepare(const Shape &s, int e, const int32_t *idx, const float *w,
                                 int32_t *idx1, float *wb1, float *wc1, hipStream_t st);
swimba_status launch_sep_accumulate(int io_dtype, int64_t n, const void *y_e, float *acc, int first,
                                    hipStream_t st);
swimba_status launch_chunk_state_mfma(const Shape &s, const void *x, const void *dt, const float *A,
                                      const void *bmix_t8, float *cs, void *states_lp, hipStream_t st,
                                      int nslots = 1, const void *cmix = nullptr, const void *bfrag = nullptr,
                                      void *cb = nullptr, int nseg = 1, const float *cs2 = nullptr);
swimba_status launch_scan_cb_mfma(const Shape &s, const float *h0, float *h_final, void *states_lp,
                                  const float *cs, const void *cmix, const void *bfrag, void *cb,
                                  hipStream_t st, int nslots = 1);
constexpr int OUTPUT_LOOKBACK_MAX_CHUNKS = 8;   // most chunks launch_output_lookback_mfma takes
swimba_status launch_output_lookback_mfma(const Shape &s, const void *x, const void *dt, const float *D,
                                          const void *cmix, const void *cb, const float *cs, const void *states_lp,
                                          void *y, const float *h0, float *h_final, hipStream_t st);
swimba_status launch_output_slots_mfma(const Shape &s, const void *x, const void *dt, const float *D,
                                       const void *cmix, const void *cb, const float *cs,
                                       const void *states_lp, void *y, const float *w, int nslots,
                                       hipStream_t st);
// launch_mix_rows_mfma, slot argument: every slot's weighted B rows as images of their own
constexpr int MIX_ALL_SLOTS = -2;
constexpr int MIX_ALL_SLOTS_MAX = 4;   // most slots the slot-image kernels take
swimba_status launch_output_mfma(const Shape &s, const void *x, const void *dt, const float *D,
                                 const void *cmix, const void *cb, const float *cs,
                                 const void *states_lp, void *y, const float *skip_w, int skip_stride,
                                 int accumulate, hipStream_t st);
// single pass with all 64 channels of a head per workgroup (fused_pass64.hip); same arguments as launch_pass_mfma
swimba_status launch_pass64_mfma(const Shape &s, const void *x, const void *dt, const float *D, const void *cmix,
                                 const void *bt8, const void *cb, const float *cs2, const float *fdec,
                                 const float *cdec, const float *h0, float *h_final, void *y, hipStream_t st,
                                 int nseg = 1, const float *hmid = nullptr);
// split pass: the sequences as nseg equal segments of whole chunks, each a chain of its own; the states at
// the nseg - 1 boundaries (hmid, (B, nseg-1, H, P, N) fp32) come from this launch pair in front of the pass
constexpr int PASS_SPLIT_MAX_SEGMENTS = 4;
constexpr int PASS_SPLIT_MAX_CHUNKS = 1024;      // chunks per segment (the boundary kernel keeps their totals in LDS)
// A chunk state counts at the boundary behind it when the sum of the chunk totals in between (log2 units)
// is at least this: below it the factor is under 2^-150 and rounds to zero in fp32.
constexpr float SPLIT_KEEP_LOG2 = -150.f;
swimba_status launch_boundary_states_mfma(const Shape &s, int nseg, const void *x, const void *dt, const float *A,
                                          const void *bt8, const float *cs2, void *states_lp, const float *h0,
                                          float *hmid, hipStream_t st);
// router + mixing + G^T tiles of whole chunks in one persistent kernel (mix_chunk.hip)
bool mix_chunk_covers(const Shape &s, bool selected);
swimba_status launch_mix_chunk_mfma(const Shape &s, const void *Be, const void *Ce, const void *logits, int32_t *idx,
                                    float *w, void *cmix, void *bmix_t8, void *cb, const float *w_sel, int ncu,
                                    hipStream_t st);
// single-pass forward (fused_pass.hip)
swimba_status launch_prep_mfma(const Shape &s, const void *dt, const float *A, const void *cmix, const void *bfrag,
                               void *cb, float *cs2, float *fdec, float *cdec, hipStream_t st, bool tiles = true);
swimba_status launch_pass_mfma(const Shape &s, const void *x, const void *dt, const float *D, const void *cmix,
                               const void *bt8, const void *cb, const float *cs2, const float *fdec,
                               const float *cdec, const float *h0, float *h_final, void *y, hipStream_t st);
swimba_status launch_step(const Shape &s, int io_dtype, const float *state_in, float *state_out,
                          const void *x, const void *dt, const float *A, const float *D,
                          const void *Be, const void *Ce, const void *logits, void *y, int32_t *idx,
                          float *bc, hipStream_t st);
swimba_status launch_step_static(const Shape &s, int io_dtype, const float *state_in, float *state_out,
                                 const void *x, const void *dt, const float *A, const float *D,
                                 const void *Be, const void *Ce, const void *logits, void *y, int32_t *idx,
                                 hipStream_t st);
swimba_status launch_step_multi(const Shape &s, int io_dtype, const float *state_in, float *state_out,
                                const void *x, const void *dt, const float *A, const float *D,
                                const void *Be, const void *Ce, const void *logits, void *y, int32_t *idx,
                                float *bc, hipStream_t st);

// Workgroup barrier that orders LDS traffic only.  __syncthreads() also waits for every
// outstanding global load and store of the wave, which would drain the prefetches and
// the result stores these kernels deliberately keep in flight across barriers.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// ---- device helper shared by the router kernel and the decode kernel -----------------
// Top-k over E logits read through `load(e)`, in (logit descending, index
// ascending) order; softmax over all E, no renormalisation.
// exp(v) for v <= 0 through the hardware exp2 (about 1 ulp; the product v * log2(e) adds a
// relative error of |v| * 2^-24, far inside the 1e-5 the routing weights are held to)
__device__ __forceinline__ float route_exp(float v) { return __builtin_amdgcn_exp2f(v * 1.4426950408889634f); }

template <typename Load>
__device__ __forceinline__ void route_token(Load load, int E, int K, int32_t *idx, float *w)
{
    float m = -INFINITY;
    for (int e = 0; e < E; ++e) m = fmaxf(m, load(e));
    float Z = 0.f;
    for (int e = 0; e < E; ++e) Z += route_exp(load(e) - m);
    const float invZ = 1.0f / Z;
    float pv = 0.f;
    int pi = -1;
    for (int r = 0; r < K; ++r) {
        int best = -1;
        float bv = 0.f;
        for (int e = 0; e < E; ++e) {
            const float v = load(e);
            // candidates are the experts that come after the previous pick in the order
            const bool after = (r == 0) || (v < pv) || (v == pv && e > pi);
            if (after && (best < 0 || v > bv)) { best = e; bv = v; }
        }
        // Only logits outside the contract (NaN, +inf, all -inf) leave no candidate.  The result is
        // undefined then, but the index stays a valid one: it addresses the expert rows.
        if (best < 0) { best = (pi + 1) % E; bv = -INFINITY; }
        idx[r] = best;
        w[r] = route_exp(bv - m) * invZ;
        pv = bv;
        pi = best;
    }
}

}  // namespace swimba
