// Measurement helpers: a streaming copy and a register-resident MFMA loop.
#include "common.hpp"

namespace swimba {

__global__ void __launch_bounds__(256)
copy_kernel(uint4 *__restrict__ dst, const uint4 *__restrict__ src, size_t n)
{
    size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    const size_t stride = (size_t)gridDim.x * blockDim.x;
    for (; i < n; i += stride) dst[i] = src[i];
}

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

__global__ void __launch_bounds__(256)
mfma_loop_kernel(float *__restrict__ sink, int iters)
{
    bf16x8_t a, b;
    for (int i = 0; i < 8; ++i) {
        a[i] = (__bf16)(float)((threadIdx.x + i) & 3);
        b[i] = (__bf16)(float)((threadIdx.x * 3 + i) & 1);
    }
    f32x16_t c0 = {0}, c1 = {0}, c2 = {0}, c3 = {0};
    for (int i = 0; i < iters; i += 4) {
        c0 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c0, 0, 0, 0);
        c1 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c1, 0, 0, 0);
        c2 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c2, 0, 0, 0);
        c3 = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c3, 0, 0, 0);
    }
    float r = 0.f;
    for (int i = 0; i < 16; ++i) r += c0[i] + c1[i] + c2[i] + c3[i];
    sink[(size_t)blockIdx.x * blockDim.x + threadIdx.x] = r;
}

}  // namespace swimba

using namespace swimba;

extern "C" {

swimba_status swimba_probe_copy(void *dst, const void *src, size_t bytes, void *hip_stream)
{
    if (!dst || !src) return SWIMBA_ERR_NULL;
    if (bytes % 16 || ((uintptr_t)dst & 15u) || ((uintptr_t)src & 15u)) return SWIMBA_ERR_SHAPE;
    if (bytes == 0) return SWIMBA_OK;
    const size_t n = bytes / 16;
    size_t blocks = (n + 255) / 256;
    if (blocks > 256 * 64) blocks = 256 * 64;
    hipLaunchKernelGGL(copy_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                       (uint4 *)dst, (const uint4 *)src, n);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status swimba_probe_mfma(float *sink, int32_t blocks, int32_t iters, void *hip_stream)
{
    if (!sink) return SWIMBA_ERR_NULL;
    if (blocks < 1 || iters < 4 || iters % 4 || blocks > (1 << 20)) return SWIMBA_ERR_SHAPE;
    hipLaunchKernelGGL(mfma_loop_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)hip_stream,
                       sink, iters);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

}  // extern "C"
