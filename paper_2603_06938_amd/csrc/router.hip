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

}  // namespace swimba
