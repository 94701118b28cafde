// Router kernel: softmax over all experts, top-k on the raw logits, no
// renormalisation (paper: router softmax equation and the top-k rule).
#include "common.hpp"

namespace swimba {

template <typename T>
__global__ void __launch_bounds__(256)
router_kernel(const T *__restrict__ logits, int64_t tokens, int E, int K,
              int32_t *__restrict__ idx, float *__restrict__ w)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= tokens) return;
    const T *g = logits + t * E;
    int32_t li[SWIMBA_MAX_TOPK];
    float lw[SWIMBA_MAX_TOPK];
    route_token([&](int e) { return to_float(g[e]); }, E, K, li, lw);
#pragma unroll
    for (int r = 0; r < SWIMBA_MAX_TOPK; ++r)
        if (r < K) {
            idx[t * K + r] = li[r];
            w[t * K + r] = lw[r];
        }
}

swimba_status launch_router(int64_t tokens, int E, int K, int io_dtype, const void *logits,
                            int32_t *idx, float *w, hipStream_t st)
{
    if (tokens == 0) return SWIMBA_OK;
    const unsigned grid = (unsigned)((tokens + 255) / 256);
    if (io_dtype == SWIMBA_BF16)
        hipLaunchKernelGGL(router_kernel<bf16>, dim3(grid), dim3(256), 0, st,
                           (const bf16 *)logits, tokens, E, K, idx, w);
    else
        hipLaunchKernelGGL(router_kernel<float>, dim3(grid), dim3(256), 0, st,
                           (const float *)logits, tokens, E, K, idx, w);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

// Routing logits as a linear function of the token features (paper: the expressivity theorem
// takes g a linear function of the features):  g_t[e] = sum_d Wg[e][d] u_t[d].
// HBM-bound (u is read once, E outputs per token): a wave takes 4 tokens at a time and the
// experts in groups of 8; its lanes split the feature index (16-byte pieces when the rows allow
// it; rows of up to 2048 features stay in registers over the expert groups), the rows of Wg come
// from L1/L2.  The 32 partial sums of a group (4 tokens x 8 experts) are reduced over the 64
// lanes together: each butterfly step halves the number of sums a lane carries (16 + 8 + 4 + 2
// + 1 + 1 shuffles instead of 6 per sum), and lane 2i ends up with sum i, which makes the store
// of a token's 8 logits one contiguous piece.  fp32 accumulation.
// (First version: one expert at a time, token rows re-read per expert, 6 shuffles per sum:
// 27 us on the 130M-shaped layer against a 4.5 us floor; rows in registers: 21 us.)
constexpr int RL_TOK = 4;
constexpr int RL_EXP = 8;

__device__ __forceinline__ void unpack_bf16x8(float (&f)[8], const uint4 v)
{
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        f[2 * i] = __uint_as_float(w[i] << 16);
        f[2 * i + 1] = __uint_as_float(w[i] & 0xffff0000u);
    }
}

// one butterfly step: lanes with bit `off` clear keep the lower N sums and receive the partner's
// contribution to them, the others the upper N
template <int N>
__device__ __forceinline__ void rl_halve(float (&v)[RL_TOK * RL_EXP], int lane, int off)
{
    const bool hi = (lane & off) != 0;
#pragma unroll
    for (int j = 0; j < N; ++j) {
        const float keep = hi ? v[N + j] : v[j];
        const float send = hi ? v[j] : v[N + j];
        v[j] = keep + __shfl_xor(send, off);
    }
}

template <typename T, bool VEC, bool REG>
__global__ void __launch_bounds__(256)
router_linear_kernel(const T *__restrict__ u, const T *__restrict__ Wg, T *__restrict__ logits, int64_t tokens,
                     int Dm, int E)
{
    const int lane = threadIdx.x & 63;
    const int64_t wave = ((int64_t)blockIdx.x * blockDim.x + threadIdx.x) >> 6;
    const int64_t t0 = wave * RL_TOK;
    if (t0 >= tokens) return;                                  // whole wave
    const T *ur[RL_TOK];
#pragma unroll
    for (int q = 0; q < RL_TOK; ++q) ur[q] = u + min(t0 + q, tokens - 1) * Dm;
    uint4 ureg[REG ? 4 : 1][RL_TOK];
    if constexpr (VEC && REG) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const int d = min(lane * 8 + 512 * c, Dm - 8);         // clamped: unused past the row end
#pragma unroll
            for (int q = 0; q < RL_TOK; ++q) ureg[c][q] = *reinterpret_cast<const uint4 *>(ur[q] + d);
        }
    }
    for (int e0 = 0; e0 < E; e0 += RL_EXP) {
        float v[RL_TOK * RL_EXP];                              // sum of token q, expert e0 + el at q * 8 + el
#pragma unroll
        for (int i = 0; i < RL_TOK * RL_EXP; ++i) v[i] = 0.f;
        const T *wr[RL_EXP];
#pragma unroll
        for (int el = 0; el < RL_EXP; ++el) wr[el] = Wg + (int64_t)min(e0 + el, E - 1) * Dm;
        if constexpr (VEC) {
            // bf16 rows of a multiple of 8 features: a lane owns 8 consecutive features per 512
            auto chunk = [&](int d, const uint4 (&up)[RL_TOK]) __attribute__((always_inline)) {
                float uf[RL_TOK][8];
#pragma unroll
                for (int q = 0; q < RL_TOK; ++q) unpack_bf16x8(uf[q], up[q]);
#pragma unroll
                for (int el = 0; el < RL_EXP; ++el) {
                    float wf[8];
                    unpack_bf16x8(wf, *reinterpret_cast<const uint4 *>(wr[el] + d));
#pragma unroll
                    for (int q = 0; q < RL_TOK; ++q)
#pragma unroll
                        for (int i = 0; i < 8; ++i) v[q * RL_EXP + el] += wf[i] * uf[q][i];
                }
            };
            if constexpr (REG) {
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    const int d = lane * 8 + 512 * c;
                    if (d < Dm) chunk(d, ureg[c]);
                }
            } else {
                for (int d = lane * 8; d < Dm; d += 512) {
                    uint4 up[RL_TOK];
#pragma unroll
                    for (int q = 0; q < RL_TOK; ++q) up[q] = *reinterpret_cast<const uint4 *>(ur[q] + d);
                    chunk(d, up);
                }
            }
        } else {
            for (int d = lane; d < Dm; d += 64) {
                float uq[RL_TOK];
#pragma unroll
                for (int q = 0; q < RL_TOK; ++q) uq[q] = to_float(ur[q][d]);
#pragma unroll
                for (int el = 0; el < RL_EXP; ++el) {
                    const float wv = to_float(wr[el][d]);
#pragma unroll
                    for (int q = 0; q < RL_TOK; ++q) v[q * RL_EXP + el] += wv * uq[q];
                }
            }
        }
        rl_halve<16>(v, lane, 32);
        rl_halve<8>(v, lane, 16);
        rl_halve<4>(v, lane, 8);
        rl_halve<2>(v, lane, 4);
        rl_halve<1>(v, lane, 2);
        const float total = v[0] + __shfl_xor(v[0], 1);        // lanes 2i and 2i + 1 both hold sum i
        const int i = lane >> 1, q = i / RL_EXP, el = i % RL_EXP;
        if ((lane & 1) == 0 && t0 + q < tokens && e0 + el < E)
            logits[(t0 + q) * E + e0 + el] = from_float<T>(total);
    }
}

swimba_status launch_router_linear(int64_t tokens, int Dm, int E, int io_dtype, const void *u, const void *Wg,
                                   void *logits, hipStream_t st)
{
    if (tokens == 0) return SWIMBA_OK;
    const int64_t waves = (tokens + RL_TOK - 1) / RL_TOK;
    const unsigned grid = (unsigned)((waves + 3) / 4);
    if (io_dtype == SWIMBA_BF16) {
        if (Dm % 8 == 0 && Dm <= 2048)
            hipLaunchKernelGGL((router_linear_kernel<bf16, true, true>), dim3(grid), dim3(256), 0, st,
                               (const bf16 *)u, (const bf16 *)Wg, (bf16 *)logits, tokens, Dm, E);
        else if (Dm % 8 == 0)
            hipLaunchKernelGGL((router_linear_kernel<bf16, true, false>), dim3(grid), dim3(256), 0, st,
                               (const bf16 *)u, (const bf16 *)Wg, (bf16 *)logits, tokens, Dm, E);
        else
            hipLaunchKernelGGL((router_linear_kernel<bf16, false, false>), dim3(grid), dim3(256), 0, st,
                               (const bf16 *)u, (const bf16 *)Wg, (bf16 *)logits, tokens, Dm, E);
    } else {
        hipLaunchKernelGGL((router_linear_kernel<float, false, false>), dim3(grid), dim3(256), 0, st,
                           (const float *)u, (const float *)Wg, (float *)logits, tokens, Dm, E);
    }
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

}  // namespace swimba
