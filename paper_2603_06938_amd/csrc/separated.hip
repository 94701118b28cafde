// Helpers of the separated-SSM contrast (paper: "Alternative: MoE of separated SSMs"):
//   h_t^(e) = exp(dt_t A) h_{t-1}^(e) + dt_t B_t^(e) x_t^T  for every expert e,
//   y_t = sum_{e in K_t} pi_{t,e} C_t^(e) . h_t^(e) + D x_t.
// Each expert is one plain SSM pass through the mixer's own kernels with the streams
// Bmix = B^(e), Cmix = gate_e * C^(e), whose output kernel adds to y; these kernels build the
// per-expert routing tables of the fp32 kernels and add fp32 buffers (final states of the
// passes of the forward with per-expert inputs).
#include "common.hpp"

namespace swimba {

// per token: idx1 = e, wb1 = 1, wc1 = pi_{t,e} if e is in the token's active set else 0
__global__ void __launch_bounds__(256)
sep_prepare_kernel(const int32_t *__restrict__ idx, const float *__restrict__ w, int64_t tokens, int K,
                   int e, int32_t *__restrict__ idx1, float *__restrict__ wb1, float *__restrict__ wc1)
{
    const int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= tokens) return;
    float gate = 0.f;
    for (int r = 0; r < K; ++r)
        if (idx[t * K + r] == e) gate += w[t * K + r];
    idx1[t] = e;
    wb1[t] = 1.f;
    wc1[t] = gate;
}

template <typename T>
__global__ void __launch_bounds__(256)
sep_accumulate_kernel(const T *__restrict__ y_e, float *__restrict__ acc, int64_t n, int first)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    const float v = to_float(y_e[i]);
    acc[i] = first ? v : acc[i] + v;
}

swimba_status launch_sep_prepare(const Shape &s, int e, const int32_t *idx, const float *w,
                                 int32_t *idx1, float *wb1, float *wc1, hipStream_t st)
{
    const int64_t T = (int64_t)s.B * s.L;
    if (T == 0) return SWIMBA_OK;
    hipLaunchKernelGGL(sep_prepare_kernel, dim3((unsigned)((T + 255) / 256)), dim3(256), 0, st, idx, w, T,
                       s.K, e, idx1, wb1, wc1);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_sep_accumulate(int io_dtype, int64_t n, const void *y_e, float *acc, int first,
                                    hipStream_t st)
{
    if (n == 0) return SWIMBA_OK;
    const dim3 grid((unsigned)((n + 255) / 256));
    if (io_dtype == SWIMBA_BF16)
        hipLaunchKernelGGL(sep_accumulate_kernel<bf16>, grid, dim3(256), 0, st, (const bf16 *)y_e, acc, n, first);
    else
        hipLaunchKernelGGL(sep_accumulate_kernel<float>, grid, dim3(256), 0, st, (const float *)y_e, acc, n, first);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

}  // namespace swimba
