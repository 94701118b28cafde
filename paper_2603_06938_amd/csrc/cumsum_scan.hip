// Per-chunk cumulative sum of dt*A, and the inter-chunk state-passing scan
// (paper, background section on SSD: matrix work inside chunks, a linear
// recurrence between chunks).
#include "common.hpp"

namespace swimba {

// ---- cs[b,c,h,q] = sum_{j<=q} dt[b, c*Q+j, h] * A[h]  (tokens past L add 0) ---------
constexpr int CS_HEAD_TILE = 16;

template <typename T>
__global__ void __launch_bounds__(256)
cumsum_kernel(const T *__restrict__ dt, const float *__restrict__ A, float *__restrict__ cs, Shape s)
{
    __shared__ float sa[CS_HEAD_TILE][SWIMBA_MAX_CHUNK + 1];
    const int b = blockIdx.x / s.nc, c = blockIdx.x % s.nc;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int Q = s.Q, H = s.H;
    const int epl = (Q + 63) / 64;  // elements per lane
    for (int h0 = 0; h0 < H; h0 += CS_HEAD_TILE) {
        for (int i = tid; i < Q * CS_HEAD_TILE; i += 256) {
            const int q = i / CS_HEAD_TILE, hh = i % CS_HEAD_TILE;
            const int h = h0 + hh, t = c * Q + q;
            float a = 0.f;
            if (h < H && t < s.L) a = to_float(dt[((int64_t)b * s.L + t) * H + h]) * A[h];
            sa[hh][q] = a;
        }
        __syncthreads();
        for (int hh = wave; hh < CS_HEAD_TILE && h0 + hh < H; hh += 4) {
            const int base = lane * epl;
            float run = 0.f;
            for (int e = 0; e < epl; ++e)
                if (base + e < Q) run += sa[hh][base + e];
            float incl = run;
            for (int off = 1; off < 64; off <<= 1) {
                const float v = __shfl_up(incl, off);
                if (lane >= off) incl += v;
            }
            float acc = __shfl_up(incl, 1);
            if (lane == 0) acc = 0.f;
            float *out = cs + (((int64_t)b * s.nc + c) * H + (h0 + hh)) * Q;
            for (int e = 0; e < epl; ++e)
                if (base + e < Q) {
                    acc += sa[hh][base + e];
                    out[base + e] = acc;
                }
        }
        __syncthreads();
    }
}

swimba_status launch_cumsum(const Shape &s, int io_dtype, const void *dt, const float *A, float *cs,
                            hipStream_t st)
{
    if (s.B * s.nc == 0) return SWIMBA_OK;
    dim3 grid((unsigned)(s.B * s.nc));
    if (io_dtype == SWIMBA_BF16)
        hipLaunchKernelGGL(cumsum_kernel<bf16>, grid, dim3(256), 0, st, (const bf16 *)dt, A, cs, s);
    else
        hipLaunchKernelGGL(cumsum_kernel<float>, grid, dim3(256), 0, st, (const float *)dt, A, cs, s);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

// ---- H_0 = h0, H_{c+1} = exp(cs_c[Q-1]) H_c + S_c ; states[c] <- H_c in place -------------
// One lane owns VEC consecutive state elements of one (b,h) and walks the chunks.
template <int VEC>
__global__ void __launch_bounds__(256)
state_scan_kernel(float *__restrict__ states, uint16_t *__restrict__ lp,
                  const float *__restrict__ h0, float *__restrict__ h_final,
                  const float *__restrict__ cs, Shape s)
{
    const int64_t per_bh = (int64_t)s.P * s.N / VEC;
    const int64_t gid = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (gid >= per_bh * s.B * s.H) return;
    const int64_t bh = gid / per_bh;
    const int64_t pn = (gid % per_bh) * VEC;
    const int b = (int)(bh / s.H), h = (int)(bh % s.H);
    const int64_t PN = (int64_t)s.P * s.N;

    float run[VEC];
#pragma unroll
    for (int v = 0; v < VEC; ++v) run[v] = h0 ? h0[bh * PN + pn + v] : 0.f;

    constexpr int UN = 4;  // chunks whose loads are issued together
    for (int c0 = 0; c0 < s.nc; c0 += UN) {
        float S[UN][VEC];
        float decay[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int c = c0 + u;
            if (c < s.nc) {
                const float *p = states + (((int64_t)b * s.nc + c) * s.H + h) * PN + pn;
                if constexpr (VEC == 4) {
                    const float4 t = *reinterpret_cast<const float4 *>(p);
                    S[u][0] = t.x; S[u][1] = t.y; S[u][2] = t.z; S[u][3] = t.w;
                } else {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) S[u][v] = p[v];
                }
                decay[u] = expf(cs[(((int64_t)b * s.nc + c) * s.H + h) * s.Q + s.Q - 1]);
            }
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int c = c0 + u;
            if (c < s.nc) {
                const int64_t off = (((int64_t)b * s.nc + c) * s.H + h) * PN + pn;
                if constexpr (VEC == 4) {
                    *reinterpret_cast<float4 *>(states + off) = make_float4(run[0], run[1], run[2], run[3]);
                    if (lp) {
                        uint2 pk;
                        pk.x = (uint32_t)bf16_bits_rne(run[0]) | ((uint32_t)bf16_bits_rne(run[1]) << 16);
                        pk.y = (uint32_t)bf16_bits_rne(run[2]) | ((uint32_t)bf16_bits_rne(run[3]) << 16);
                        *reinterpret_cast<uint2 *>(lp + off) = pk;
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < VEC; ++v) {
                        states[off + v] = run[v];
                        if (lp) lp[off + v] = bf16_bits_rne(run[v]);
                    }
                }
#pragma unroll
                for (int v = 0; v < VEC; ++v) run[v] = decay[u] * run[v] + S[u][v];
            }
        }
    }
    if (h_final) {
#pragma unroll
        for (int v = 0; v < VEC; ++v) h_final[bh * PN + pn + v] = run[v];
    }
}

swimba_status launch_state_scan(const Shape &s, const float *h0, float *h_final, float *states,
                                void *states_lp, const float *cs, hipStream_t st)
{
    const int64_t elems = (int64_t)s.B * s.H * s.P * s.N;
    if (elems == 0) return SWIMBA_OK;
    if (s.N % 4 == 0) {
        const unsigned grid = (unsigned)((elems / 4 + 255) / 256);
        hipLaunchKernelGGL(state_scan_kernel<4>, dim3(grid), dim3(256), 0, st, states,
                           (uint16_t *)states_lp, h0, h_final, cs, s);
    } else {
        const unsigned grid = (unsigned)((elems + 255) / 256);
        hipLaunchKernelGGL(state_scan_kernel<1>, dim3(grid), dim3(256), 0, st, states,
                           (uint16_t *)states_lp, h0, h_final, cs, s);
    }
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

}  // namespace swimba
