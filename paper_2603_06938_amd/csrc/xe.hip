// Helpers of the mixed forward with one input stream per expert (paper: mixed state update
// equation in its full form, the injection sum_{e in K_t} pi_{t,e} x_t^(e) (x) B_t^(e)).
// The state is linear in the injection, so the rank-k update is evaluated as k rank-1 passes
// through the mixer's own kernels: pass r uses x = x^(e_r) (gathered here, e_r = the token's
// r-th active expert), Bmix = pi_{e_r} B^(e_r) and the full Cmix.  The output kernel of pass r
// adds its result (and its share pi_{e_r} D x^(e_r) of the skip term) to y; the final states
// are summed in fp32.
#include "common.hpp"

namespace swimba {

// xg[t][:] = x_experts[t][idx[t][slot]][:], 16 bytes per lane when the row length allows;
// with slot < 0 every slot: xg[t][r][:] = x_experts[t][idx[t][r]][:]
template <int BYTES>
__global__ void __launch_bounds__(256)
xe_gather_kernel(const unsigned char *__restrict__ xe, const int32_t *__restrict__ idx,
                 unsigned char *__restrict__ xg, int64_t tokens, int E, int K, int64_t row_bytes, int slot)
{
    const int64_t per_tok = row_bytes / BYTES;
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t rows = (slot < 0) ? tokens * K : tokens;
    if (i >= rows * per_tok) return;
    const int64_t row = i / per_tok, o = (i % per_tok) * BYTES;
    const int64_t t = (slot < 0) ? row / K : row;
    const int e = idx[(slot < 0) ? row : t * K + slot];
    const unsigned char *src = xe + (t * E + e) * row_bytes + o;
    unsigned char *dst = xg + row * row_bytes + o;
    if (BYTES == 16)
        *reinterpret_cast<uint4 *>(dst) = *reinterpret_cast<const uint4 *>(src);
    else if (BYTES == 4)
        *reinterpret_cast<uint32_t *>(dst) = *reinterpret_cast<const uint32_t *>(src);
    else
        *reinterpret_cast<uint16_t *>(dst) = *reinterpret_cast<const uint16_t *>(src);
}

__global__ void __launch_bounds__(256)
xe_slot_weights_kernel(const float *__restrict__ w, float *__restrict__ wslot, int64_t n, int K, int slot)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n) return;
    wslot[i] = ((int)(i % K) == slot) ? w[i] : 0.f;
}

swimba_status launch_xe_gather(const Shape &s, int io_dtype, int slot, const void *x_experts,
                               const int32_t *idx, void *xg, hipStream_t st)
{
    const int64_t T = (int64_t)s.B * s.L;
    const int64_t row_bytes = (int64_t)s.H * s.P * (io_dtype == SWIMBA_BF16 ? 2 : 4);
    if (T == 0) return SWIMBA_OK;
    // rows start at multiples of row_bytes from 16-byte aligned bases
    const int bytes = (row_bytes % 16 == 0) ? 16 : (row_bytes % 4 == 0) ? 4 : 2;
    const int64_t rows = (slot < 0) ? T * s.K : T;
    const dim3 grid((unsigned)((rows * (row_bytes / bytes) + 255) / 256));
    const unsigned char *src = (const unsigned char *)x_experts;
    unsigned char *dst = (unsigned char *)xg;
    if (bytes == 16)
        hipLaunchKernelGGL(xe_gather_kernel<16>, grid, dim3(256), 0, st, src, idx, dst, T, s.E, s.K, row_bytes, slot);
    else if (bytes == 4)
        hipLaunchKernelGGL(xe_gather_kernel<4>, grid, dim3(256), 0, st, src, idx, dst, T, s.E, s.K, row_bytes, slot);
    else
        hipLaunchKernelGGL(xe_gather_kernel<2>, grid, dim3(256), 0, st, src, idx, dst, T, s.E, s.K, row_bytes, slot);
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

}  // namespace swimba
