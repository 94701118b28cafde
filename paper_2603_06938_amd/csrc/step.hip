// Single-token recurrent decode step (paper: selective SSM recurrence per
// channel, with the router-mixed injection and readout of Theorem 1).
// HBM-bound: the fp32 state is read once and written once.
#include "common.hpp"

namespace swimba {

constexpr int STEP_THREADS = 256;

// Routing + mixing of one token, done redundantly by every block of that
// batch row (E logits and k*N elements: negligible next to the 2*P*N*4 state
// bytes).  Leaves Bmix, Cmix in LDS.
template <typename T>
__device__ __forceinline__ void route_and_mix(const T *__restrict__ logits_b,
                                              const T *__restrict__ Be_b, const T *__restrict__ Ce_b,
                                              int E, int K, int G, int N, int g, float *sB, float *sC,
                                              int32_t *s_idx, float *s_w, int tid)
{
    if (tid == 0) route_token([&](int e) { return to_float(logits_b[e]); }, E, K, s_idx, s_w);
    __syncthreads();
    for (int n = tid; n < N; n += STEP_THREADS) {
        float bm = 0.f, cm = 0.f;
        for (int r = 0; r < K; ++r) {
            const int64_t o = ((int64_t)s_idx[r] * G + g) * N + n;
            bm += s_w[r] * to_float(Be_b[o]);
            cm += s_w[r] * to_float(Ce_b[o]);
        }
        sB[n] = bm;
        sC[n] = cm;
    }
    __syncthreads();
}

// ---- N = 128: a wave covers two state rows per access, float4 per lane ----------------
// Block (b,h): lane -> columns n4..n4+3, row group rg = tid/32; rows p = rg + 8*i.
template <typename T, int ROWS_PER_LANE>
__global__ void __launch_bounds__(STEP_THREADS)
step_kernel_n128(const float *state_in, float *state_out, const T *__restrict__ x,
                 const T *__restrict__ dt, const float *__restrict__ A, const float *__restrict__ D,
                 const T *__restrict__ Be, const T *__restrict__ Ce, const T *__restrict__ logits,
                 T *__restrict__ y, int32_t *__restrict__ idx_out, Shape s)
{
    constexpr int N = 128;
    __shared__ float sB[N], sC[N], s_w[SWIMBA_MAX_TOPK];
    __shared__ int32_t s_idx[SWIMBA_MAX_TOPK];
    const int b = blockIdx.x / s.H, h = blockIdx.x % s.H, g = (h * s.G) / s.H;
    const int tid = threadIdx.x;
    const int n4 = (tid & 31) * 4, rg = tid >> 5;
    const int64_t base = ((int64_t)b * s.H + h) * s.P * N;
    const int P = s.P;

    // issue the state loads first: they are the long-latency part
    float4 st[ROWS_PER_LANE];
#pragma unroll
    for (int i = 0; i < ROWS_PER_LANE; ++i) {
        const int p = rg + 8 * i;
        st[i] = (p < P) ? *reinterpret_cast<const float4 *>(state_in + base + (int64_t)p * N + n4)
                        : make_float4(0.f, 0.f, 0.f, 0.f);
    }

    route_and_mix(logits + (int64_t)b * s.E, Be + (int64_t)b * s.E * s.G * N,
                  Ce + (int64_t)b * s.E * s.G * N, s.E, s.K, s.G, N, g, sB, sC, s_idx, s_w, tid);
    if (idx_out && h == 0 && tid < s.K) idx_out[(int64_t)b * s.K + tid] = s_idx[tid];

    const float dtv = to_float(dt[(int64_t)b * s.H + h]);
    const float decay = expf(dtv * A[h]);
    const float dsk = D ? D[h] : 0.f;
    const float4 bm = *reinterpret_cast<const float4 *>(sB + n4);
    const float4 cm = *reinterpret_cast<const float4 *>(sC + n4);

#pragma unroll
    for (int i = 0; i < ROWS_PER_LANE; ++i) {
        const int p = rg + 8 * i;
        if (p < P) {   // uniform over each 32-lane half
            const float xv = to_float(x[((int64_t)b * s.H + h) * P + p]);
            const float u = dtv * xv;
            float4 v = st[i];
            v.x = decay * v.x + u * bm.x;
            v.y = decay * v.y + u * bm.y;
            v.z = decay * v.z + u * bm.z;
            v.w = decay * v.w + u * bm.w;
            *reinterpret_cast<float4 *>(state_out + base + (int64_t)p * N + n4) = v;
            float part = (v.x * cm.x + v.y * cm.y) + (v.z * cm.z + v.w * cm.w);
#pragma unroll
            for (int off = 16; off >= 1; off >>= 1) part += __shfl_xor(part, off);
            if ((tid & 31) == 0) y[((int64_t)b * s.H + h) * P + p] = from_float<T>(part + dsk * xv);
        }
    }
}

// ---- any N: a wave walks one state row at a time ----------------------------------------
template <typename T>
__global__ void __launch_bounds__(STEP_THREADS)
step_kernel_generic(const float *state_in, float *state_out, const T *__restrict__ x,
                    const T *__restrict__ dt, const float *__restrict__ A, const float *__restrict__ D,
                    const T *__restrict__ Be, const T *__restrict__ Ce, const T *__restrict__ logits,
                    T *__restrict__ y, int32_t *__restrict__ idx_out, Shape s)
{
    __shared__ float sB[SWIMBA_MAX_DSTATE], sC[SWIMBA_MAX_DSTATE], s_w[SWIMBA_MAX_TOPK];
    __shared__ int32_t s_idx[SWIMBA_MAX_TOPK];
    const int b = blockIdx.x / s.H, h = blockIdx.x % s.H, g = (h * s.G) / s.H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = s.N, P = s.P;
    const int64_t base = ((int64_t)b * s.H + h) * P * N;

    route_and_mix(logits + (int64_t)b * s.E, Be + (int64_t)b * s.E * s.G * N,
                  Ce + (int64_t)b * s.E * s.G * N, s.E, s.K, s.G, N, g, sB, sC, s_idx, s_w, tid);
    if (idx_out && h == 0 && tid < s.K) idx_out[(int64_t)b * s.K + tid] = s_idx[tid];

    const float dtv = to_float(dt[(int64_t)b * s.H + h]);
    const float decay = expf(dtv * A[h]);
    const float dsk = D ? D[h] : 0.f;
    for (int p = wave; p < P; p += STEP_THREADS / 64) {
        const float xv = to_float(x[((int64_t)b * s.H + h) * P + p]);
        const float u = dtv * xv;
        float part = 0.f;
        for (int n = lane; n < N; n += 64) {
            const float v = decay * state_in[base + (int64_t)p * N + n] + u * sB[n];
            state_out[base + (int64_t)p * N + n] = v;
            part += v * sC[n];
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off);
        if (lane == 0) y[((int64_t)b * s.H + h) * P + p] = from_float<T>(part + dsk * xv);
    }
}

template <typename T>
static swimba_status launch_step_t(const Shape &s, const float *state_in, float *state_out,
                                   const void *x, const void *dt, const float *A, const float *D,
                                   const void *Be, const void *Ce, const void *logits, void *y,
                                   int32_t *idx, hipStream_t st)
{
    const int64_t blocks = (int64_t)s.B * s.H;
    if (blocks == 0) return SWIMBA_OK;
    dim3 grid((unsigned)blocks), block(STEP_THREADS);
    if (s.N == 128 && s.P <= 64)
        hipLaunchKernelGGL((step_kernel_n128<T, 8>), grid, block, 0, st, state_in, state_out,
                           (const T *)x, (const T *)dt, A, D, (const T *)Be, (const T *)Ce,
                           (const T *)logits, (T *)y, idx, s);
    else
        hipLaunchKernelGGL(step_kernel_generic<T>, grid, block, 0, st, state_in, state_out,
                           (const T *)x, (const T *)dt, A, D, (const T *)Be, (const T *)Ce,
                           (const T *)logits, (T *)y, idx, s);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_step(const Shape &s, int io_dtype, const float *state_in, float *state_out,
                          const void *x, const void *dt, const float *A, const float *D,
                          const void *Be, const void *Ce, const void *logits, void *y, int32_t *idx,
                          hipStream_t st)
{
    if (io_dtype == SWIMBA_BF16)
        return launch_step_t<bf16>(s, state_in, state_out, x, dt, A, D, Be, Ce, logits, y, idx, st);
    return launch_step_t<float>(s, state_in, state_out, x, dt, A, D, Be, Ce, logits, y, idx, st);
}

}  // namespace swimba
