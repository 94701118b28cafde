// fp32 SSD chunk kernels for any (P, N, Q, io type) within the library limits.
// These are the kernels of the fp32 workloads and of bf16 shapes the MFMA
// kernels do not cover.  The expert mixing is done while the chunk's B/C rows
// are staged into LDS; mixed streams never go to HBM.
#include "common.hpp"

namespace swimba {

constexpr int GEN_THREADS = 256;
constexpr int GEN_TB = 16;          // tokens staged per step in the chunk-state kernel
constexpr int GEN_MAX_OUT = 32;     // outputs per lane (P*N <= 256*32)
constexpr int GEN_TI = 16;          // tokens per block / per step in the output kernel

// mixed row: dst[n] = sum_r w[r] * src[(e_r*G + g)*N + n], for one token
template <typename T>
__device__ __forceinline__ float mix_elem(const T *__restrict__ tok_base, const int32_t *idx,
                                          const float *w, int K, int G, int N, int g, int n)
{
    float acc = 0.f;
    for (int r = 0; r < K; ++r)
        acc += w[r] * to_float(tok_base[((int64_t)idx[r] * G + g) * N + n]);
    return acc;
}

// ---- S_c[p][n] = sum_j exp(cs_last - cs_j) dt_j x[j][p] Bmix[j][n] ----------------------
template <typename T>
__global__ void __launch_bounds__(GEN_THREADS)
chunk_state_generic_kernel(const T *__restrict__ x, const T *__restrict__ dt,
                           const T *__restrict__ Be, const int32_t *__restrict__ idx,
                           const float *__restrict__ w, const float *__restrict__ cs,
                           float *__restrict__ states, Shape s)
{
    extern __shared__ float smem[];
    float *sx = smem;                       // [GEN_TB][P]  coefficient-weighted x
    float *sb = smem + GEN_TB * s.P;        // [GEN_TB][N]  mixed B
    const int h = blockIdx.x % s.H;
    const int c = (blockIdx.x / s.H) % s.nc;
    const int b = blockIdx.x / (s.H * s.nc);
    const int g = (h * s.G) / s.H;
    const int tid = threadIdx.x;
    const int PN = s.P * s.N;
    const int cnt = (PN + GEN_THREADS - 1) / GEN_THREADS;
    const float *csr = cs + (((int64_t)b * s.nc + c) * s.H + h) * s.Q;
    const float cs_last = csr[s.Q - 1];

    float acc[GEN_MAX_OUT];
#pragma unroll
    for (int i = 0; i < GEN_MAX_OUT; ++i) acc[i] = 0.f;

    for (int j0 = 0; j0 < s.Q; j0 += GEN_TB) {
        for (int i = tid; i < GEN_TB * s.P; i += GEN_THREADS) {
            const int jj = i / s.P, p = i % s.P, j = j0 + jj, t = c * s.Q + j;
            float v = 0.f;
            if (j < s.Q && t < s.L) {
                const int64_t bt = (int64_t)b * s.L + t;
                v = to_float(x[(bt * s.H + h) * s.P + p]) * to_float(dt[bt * s.H + h]) *
                    expf(cs_last - csr[j]);
            }
            sx[jj * s.P + p] = v;
        }
        for (int i = tid; i < GEN_TB * s.N; i += GEN_THREADS) {
            const int jj = i / s.N, n = i % s.N, j = j0 + jj, t = c * s.Q + j;
            float v = 0.f;
            if (j < s.Q && t < s.L) {
                const int64_t bt = (int64_t)b * s.L + t;
                v = mix_elem(Be + bt * s.E * s.G * s.N, idx + bt * s.K, w + bt * s.K, s.K, s.G, s.N, g, n);
            }
            sb[jj * s.N + n] = v;
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < GEN_MAX_OUT; ++i) {
            if (i < cnt) {
                const int o = tid + i * GEN_THREADS;
                if (o < PN) {
                    const int p = o / s.N, n = o % s.N;
                    float a = acc[i];
                    for (int jj = 0; jj < GEN_TB; ++jj) a += sx[jj * s.P + p] * sb[jj * s.N + n];
                    acc[i] = a;
                }
            }
        }
        __syncthreads();
    }
    float *out = states + (((int64_t)b * s.nc + c) * s.H + h) * PN;
#pragma unroll
    for (int i = 0; i < GEN_MAX_OUT; ++i) {
        if (i < cnt) {
            const int o = tid + i * GEN_THREADS;
            if (o < PN) out[o] = acc[i];
        }
    }
}

swimba_status launch_chunk_state_generic(const Shape &s, int io_dtype, const void *x, const void *dt,
                                         const void *Be, const int32_t *idx, const float *w,
                                         const float *cs, float *states, hipStream_t st)
{
    const int64_t blocks = (int64_t)s.B * s.nc * s.H;
    if (blocks == 0) return SWIMBA_OK;
    const size_t shm = sizeof(float) * GEN_TB * (size_t)(s.P + s.N);
    if (io_dtype == SWIMBA_BF16)
        hipLaunchKernelGGL(chunk_state_generic_kernel<bf16>, dim3((unsigned)blocks), dim3(GEN_THREADS),
                           shm, st, (const bf16 *)x, (const bf16 *)dt, (const bf16 *)Be, idx, w, cs,
                           states, s);
    else
        hipLaunchKernelGGL(chunk_state_generic_kernel<float>, dim3((unsigned)blocks), dim3(GEN_THREADS),
                           shm, st, (const float *)x, (const float *)dt, (const float *)Be, idx, w, cs,
                           states, s);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

// ---- y_i = sum_{j<=i} (Cmix_i.Bmix_j) exp(cs_i-cs_j) dt_j x_j + exp(cs_i) Cmix_i.H_c + D x_i --
// One block owns GEN_TI consecutive tokens of one (b, chunk, head).  `w` weighs the B rows,
// `wc` the C rows (the same array for the mixed model; they differ for the separated contrast).
// skip_w (optional): per-token factor of the skip term, skip_w[token * skip_stride];
// accumulate: add to what y already holds (passes of the forward with per-expert inputs).
constexpr int GEN_MAX_YPT = (GEN_TI * SWIMBA_MAX_HEADDIM) / GEN_THREADS;  // (i,p) pairs per lane

template <typename T>
__global__ void __launch_bounds__(GEN_THREADS)
output_generic_kernel(const T *__restrict__ x, const T *__restrict__ dt, const float *__restrict__ D,
                      const T *__restrict__ Be, const T *__restrict__ Ce,
                      const int32_t *__restrict__ idx, const float *__restrict__ w,
                      const float *__restrict__ wc, const float *__restrict__ cs,
                      const float *__restrict__ states, T *__restrict__ y, Shape s,
                      const float *__restrict__ skip_w, int skip_stride, int accumulate)
{
    extern __shared__ float smem[];
    // rows of the two mixed tiles are padded by one float: the (i, j) dot products below read
    // row ii of one and row jj of the other with the same n in every lane, and an unpadded
    // power-of-two row length puts all those reads on one LDS bank (16-way conflicts: the kernel
    // spent almost all of its time there)
    const int NS = s.N + 1;
    float *sc = smem;                         // [GEN_TI][NS] mixed C of the block's tokens
    float *sb = sc + GEN_TI * NS;             // [GEN_TI][NS] mixed B of the current j tile
    float *sx = sb + GEN_TI * NS;             // [GEN_TI][P] dt_j * x_j of the current j tile
    float *sm = sx + GEN_TI * s.P;            // [GEN_TI][GEN_TI] decay-masked C.B^T tile
    const int nib = (s.Q + GEN_TI - 1) / GEN_TI;
    const int ib = blockIdx.x % nib;
    const int h = (blockIdx.x / nib) % s.H;
    const int c = (blockIdx.x / (nib * s.H)) % s.nc;
    const int b = blockIdx.x / (nib * s.H * s.nc);
    const int g = (h * s.G) / s.H;
    const int tid = threadIdx.x;
    const int i0 = ib * GEN_TI;
    if (c * s.Q + i0 >= s.L) return;          // whole block past the end of the sequence
    const float *csr = cs + (((int64_t)b * s.nc + c) * s.H + h) * s.Q;
    const float *Hc = states + (((int64_t)b * s.nc + c) * s.H + h) * s.P * s.N;
    const int npair = GEN_TI * s.P;
    const int cnt = (npair + GEN_THREADS - 1) / GEN_THREADS;

    for (int i = tid; i < GEN_TI * s.N; i += GEN_THREADS) {
        const int ii = i / s.N, n = i % s.N, q = i0 + ii, t = c * s.Q + q;
        float v = 0.f;
        if (q < s.Q && t < s.L) {
            const int64_t bt = (int64_t)b * s.L + t;
            v = mix_elem(Ce + bt * s.E * s.G * s.N, idx + bt * s.K, wc + bt * s.K, s.K, s.G, s.N, g, n);
        }
        sc[ii * NS + n] = v;
    }
    __syncthreads();

    // contribution of the carried state
    float acc[GEN_MAX_YPT];
#pragma unroll
    for (int r = 0; r < GEN_MAX_YPT; ++r) {
        acc[r] = 0.f;
        if (r < cnt) {
            const int o = tid + r * GEN_THREADS;
            if (o < npair) {
                const int ii = o / s.P, p = o % s.P, q = i0 + ii;
                if (q < s.Q) {
                    float a = 0.f;
                    for (int n = 0; n < s.N; ++n) a += sc[ii * NS + n] * Hc[p * s.N + n];
                    acc[r] = a * expf(csr[q]);
                }
            }
        }
    }

    // intra-chunk part, j tiles up to and including the block's own tile
    for (int j0 = 0; j0 <= i0; j0 += GEN_TI) {
        __syncthreads();
        for (int i = tid; i < GEN_TI * s.N; i += GEN_THREADS) {
            const int jj = i / s.N, n = i % s.N, q = j0 + jj, t = c * s.Q + q;
            float v = 0.f;
            if (q < s.Q && t < s.L) {
                const int64_t bt = (int64_t)b * s.L + t;
                v = mix_elem(Be + bt * s.E * s.G * s.N, idx + bt * s.K, w + bt * s.K, s.K, s.G, s.N, g, n);
            }
            sb[jj * NS + n] = v;
        }
        for (int i = tid; i < GEN_TI * s.P; i += GEN_THREADS) {
            const int jj = i / s.P, p = i % s.P, q = j0 + jj, t = c * s.Q + q;
            float v = 0.f;
            if (q < s.Q && t < s.L) {
                const int64_t bt = (int64_t)b * s.L + t;
                v = to_float(x[(bt * s.H + h) * s.P + p]) * to_float(dt[bt * s.H + h]);
            }
            sx[i] = v;
        }
        __syncthreads();
        {
            const int ii = tid / GEN_TI, jj = tid % GEN_TI;   // GEN_THREADS == GEN_TI*GEN_TI
            const int qi = i0 + ii, qj = j0 + jj;
            float m = 0.f;
            if (qi < s.Q && qj <= qi) {
                float dot = 0.f;
                for (int n = 0; n < s.N; ++n) dot += sc[ii * NS + n] * sb[jj * NS + n];
                m = dot * expf(csr[qi] - csr[qj]);
            }
            sm[ii * GEN_TI + jj] = m;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < GEN_MAX_YPT; ++r) {
            if (r < cnt) {
                const int o = tid + r * GEN_THREADS;
                if (o < npair) {
                    const int ii = o / s.P, p = o % s.P;
                    float a = acc[r];
                    for (int jj = 0; jj < GEN_TI; ++jj) a += sm[ii * GEN_TI + jj] * sx[jj * s.P + p];
                    acc[r] = a;
                }
            }
        }
    }

#pragma unroll
    for (int r = 0; r < GEN_MAX_YPT; ++r) {
        if (r < cnt) {
            const int o = tid + r * GEN_THREADS;
            if (o < npair) {
                const int ii = o / s.P, p = o % s.P, q = i0 + ii, t = c * s.Q + q;
                if (q < s.Q && t < s.L) {
                    const int64_t off = (((int64_t)b * s.L + t) * s.H + h) * s.P + p;
                    float skip = D ? D[h] * to_float(x[off]) : 0.f;
                    if (skip_w) skip *= skip_w[((int64_t)b * s.L + t) * skip_stride];
                    const float prev = accumulate ? to_float(y[off]) : 0.f;
                    y[off] = from_float<T>(acc[r] + skip + prev);
                }
            }
        }
    }
}

swimba_status launch_output_generic(const Shape &s, int io_dtype, const void *x, const void *dt,
                                    const float *D, const void *Be, const void *Ce,
                                    const int32_t *idx, const float *w, const float *wc,
                                    const float *cs, const float *states, void *y, const float *skip_w,
                                    int skip_stride, int accumulate, hipStream_t st)
{
    static_assert(GEN_THREADS == GEN_TI * GEN_TI, "one lane per (i,j) pair of a tile");
    const int nib = (s.Q + GEN_TI - 1) / GEN_TI;
    const int64_t blocks = (int64_t)s.B * s.nc * s.H * nib;
    if (blocks == 0) return SWIMBA_OK;
    const size_t shm = sizeof(float) * (size_t)(2 * GEN_TI * (s.N + 1) + GEN_TI * s.P + GEN_TI * GEN_TI);
    if (io_dtype == SWIMBA_BF16)
        hipLaunchKernelGGL(output_generic_kernel<bf16>, dim3((unsigned)blocks), dim3(GEN_THREADS), shm,
                           st, (const bf16 *)x, (const bf16 *)dt, D, (const bf16 *)Be,
                           (const bf16 *)Ce, idx, w, wc, cs, states, (bf16 *)y, s, skip_w, skip_stride, accumulate);
    else
        hipLaunchKernelGGL(output_generic_kernel<float>, dim3((unsigned)blocks), dim3(GEN_THREADS), shm,
                           st, (const float *)x, (const float *)dt, D, (const float *)Be,
                           (const float *)Ce, idx, w, wc, cs, states, (float *)y, s, skip_w, skip_stride, accumulate);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

}  // namespace swimba
