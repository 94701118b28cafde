// Helpers of the mixed forward with one input stream per expert (paper: mixed state update
// equation in its full form, the injection sum_{e in K_t} pi_{t,e} x_t^(e) (x) B_t^(e)).
// The state is linear in the injection, so the rank-k update is evaluated as k rank-1 passes
// through the mixer's own kernels: pass r uses x = x^(e_r) (gathered here, e_r = the token's
// r-th active expert), Bmix = pi_{e_r} B^(e_r) and the full Cmix; outputs and final states
// are summed in fp32.  The skip term multiplies xbar = sum_r pi_{e_r} x^(e_r).
#include "common.hpp"

namespace swimba {

// xg[t][hp] = x_experts[t][idx[t][slot]][hp];  xbar[t][hp] (+)= w[t][slot] * xg[t][hp]
template <typename T, int VEC>
__global__ void __launch_bounds__(256)
xe_gather_kernel(const T *__restrict__ xe, const int32_t *__restrict__ idx, const float *__restrict__ w,
                 T *__restrict__ xg, float *__restrict__ xbar, int64_t tokens, int E, int K, int HP,
                 int slot, int first)
{
    const int per_tok = HP / VEC;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= tokens * per_tok) return;
    const int64_t t = i / per_tok;
    const int hp = (int)(i % per_tok) * VEC;
    const int e = idx[t * K + slot];
    const float wt = w[t * K + slot];
    const T *src = xe + ((t * E + e) * HP + hp);
    T v[VEC];
#pragma unroll
    for (int q = 0; q < VEC; ++q) v[q] = src[q];
#pragma unroll
    for (int q = 0; q < VEC; ++q) xg[t * HP + hp + q] = v[q];
    if (xbar) {
#pragma unroll
        for (int q = 0; q < VEC; ++q) {
            const float prev = first ? 0.f : xbar[t * HP + hp + q];
            xbar[t * HP + hp + q] = prev + wt * to_float(v[q]);
        }
    }
}

__global__ void __launch_bounds__(256)
xe_slot_weights_kernel(const float *__restrict__ w, float *__restrict__ wslot, int64_t n, int K, int slot)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    wslot[i] = ((int)(i % K) == slot) ? w[i] : 0.f;
}

template <typename T>
__global__ void __launch_bounds__(256)
xe_finish_kernel(const float *__restrict__ acc, const float *__restrict__ xbar, const float *__restrict__ D,
                 T *__restrict__ y, int64_t n, int H, int P)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const int h = (int)((i / P) % H);
    y[i] = from_float<T>(acc[i] + (D ? D[h] * xbar[i] : 0.f));
}

swimba_status launch_xe_gather(const Shape &s, int io_dtype, int slot, int first, const void *x_experts,
                               const int32_t *idx, const float *w, void *xg, float *xbar, hipStream_t st)
{
    const int64_t T = (int64_t)s.B * s.L;
    const int HP = s.H * s.P;
    if (T == 0) return SWIMBA_OK;
    const int vec = (HP % 8 == 0) ? 8 : 1;
    const dim3 grid((unsigned)((T * (HP / vec) + 255) / 256));
    if (io_dtype == SWIMBA_BF16) {
        if (vec == 8)
            hipLaunchKernelGGL((xe_gather_kernel<bf16, 8>), grid, dim3(256), 0, st, (const bf16 *)x_experts, idx, w,
                               (bf16 *)xg, xbar, T, s.E, s.K, HP, slot, first);
        else
            hipLaunchKernelGGL((xe_gather_kernel<bf16, 1>), grid, dim3(256), 0, st, (const bf16 *)x_experts, idx, w,
                               (bf16 *)xg, xbar, T, s.E, s.K, HP, slot, first);
    } else {
        if (vec == 8)
            hipLaunchKernelGGL((xe_gather_kernel<float, 8>), grid, dim3(256), 0, st, (const float *)x_experts, idx,
                               w, (float *)xg, xbar, T, s.E, s.K, HP, slot, first);
        else
            hipLaunchKernelGGL((xe_gather_kernel<float, 1>), grid, dim3(256), 0, st, (const float *)x_experts, idx,
                               w, (float *)xg, xbar, T, s.E, s.K, HP, slot, first);
    }
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_xe_slot_weights(const Shape &s, int slot, const float *w, float *wslot, hipStream_t st)
{
    const int64_t n = (int64_t)s.B * s.L * s.K;
    if (n == 0) return SWIMBA_OK;
    hipLaunchKernelGGL(xe_slot_weights_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, w, wslot, n,
                       s.K, slot);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_xe_finish(const Shape &s, int io_dtype, const float *acc, const float *xbar,
                               const float *D, void *y, hipStream_t st)
{
    const int64_t n = (int64_t)s.B * s.L * s.H * s.P;
    if (n == 0) return SWIMBA_OK;
    const dim3 grid((unsigned)((n + 255) / 256));
    if (io_dtype == SWIMBA_BF16)
        hipLaunchKernelGGL(xe_finish_kernel<bf16>, grid, dim3(256), 0, st, acc, xbar, D, (bf16 *)y, n, s.H, s.P);
    else
        hipLaunchKernelGGL(xe_finish_kernel<float>, grid, dim3(256), 0, st, acc, xbar, D, (float *)y, n, s.H, s.P);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

}  // namespace swimba
