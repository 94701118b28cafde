// Single-token recurrent decode step (paper: selective SSM recurrence per
// channel, with the router-mixed injection and readout of Theorem 1).
// Two launches: a tiny kernel routes every token and mixes its B and C streams
// (fp32, into the caller's workspace); the update kernel then only streams the
// fp32 state through once (read, h' = decay*h + dt*x (x) Bmix, y = h'.Cmix, write).
// The update kernel is HBM-bound; its shape (one or two 16-byte accesses per lane,
// small workgroups, non-temporal loads and stores, no dependent load chain) is the
// one that measured fastest for an in-place stream on this chip.
#include "common.hpp"

#include <atomic>

namespace swimba {

// Scratch of swimba_step_static, the decode step for callers that cannot provide (or allocate) a
// workspace: the mixed B and C rows of one step, B*G*2N fp32.  One copy per GPU the library runs
// on, held until the process ends.  In host code the array's name is only a handle for
// hipGetSymbolAddress; kernels and copies get the address that call returns for the current device.
static __device__ __align__(256) float scratch[SWIMBA_STATIC_SCRATCH_BYTES / sizeof(float)];

constexpr int STEP_THREADS = 256;
typedef float __attribute__((ext_vector_type(4))) f32x4_t;

// ---- routing + mixing: block = (b, g), mixed (B; C) rows of N fp32 each ------------------
template <typename T>
__global__ void __launch_bounds__(128)
step_mix_kernel(const T *__restrict__ Be, const T *__restrict__ Ce, const T *__restrict__ logits,
                float *__restrict__ bc, int32_t *__restrict__ idx_out, Shape s)
{
    __shared__ float s_w[SWIMBA_MAX_TOPK];
    __shared__ int32_t s_idx[SWIMBA_MAX_TOPK];
    const int b = blockIdx.x / s.G, g = blockIdx.x % s.G;
    const int tid = threadIdx.x;
    // the logits go through LDS first: one memory latency instead of one per pass of the router
    __shared__ float s_log[SWIMBA_MAX_EXPERTS];
    for (int e = tid; e < s.E; e += 128) s_log[e] = to_float(logits[(int64_t)b * s.E + e]);
    __syncthreads();
    if (tid == 0) route_token([&](int e) { return s_log[e]; }, s.E, s.K, s_idx, s_w);
    __syncthreads();
    if (idx_out && g == 0 && tid < s.K) idx_out[(int64_t)b * s.K + tid] = s_idx[tid];
    const T *Bb = Be + ((int64_t)b * s.E * s.G + g) * s.N;
    const T *Cb = Ce + ((int64_t)b * s.E * s.G + g) * s.N;
    float *out = bc + (int64_t)blockIdx.x * 2 * s.N;
    for (int n = tid; n < s.N; n += 128) {
        float bm = 0.f, cm = 0.f;
        for (int r = 0; r < s.K; ++r) {
            const int64_t o = (int64_t)s_idx[r] * s.G * s.N + n;
            bm += s_w[r] * to_float(Bb[o]);
            cm += s_w[r] * to_float(Cb[o]);
        }
        out[n] = bm;
        out[s.N + n] = cm;
    }
}

// Sums over the 32 lanes of a half wave of NV values per lane at once (NV a power of two, at most
// 16): every butterfly step halves the number of values a lane carries, so NV values cost
// NV shuffles instead of 5 NV.  Returns sum number ((lane & 31) >> 1) % NV... see below: after
// log2(NV) halving steps a lane holds the value whose index is given by its lane bits, the
// remaining steps are plain xor reductions.  Value i ends up (complete) on the lanes whose bits
// 4 .. 5-log2(NV) spell i.
template <int NV>
__device__ __forceinline__ float half_wave_sums(float (&v)[NV], int lane)
{
    int off = 16;
#pragma unroll
    for (int n = NV / 2; n >= 1; n >>= 1, off >>= 1) {
        const bool hi = (lane & off) != 0;
#pragma unroll
        for (int j = 0; j < n; ++j) {
            const float keep = hi ? v[n + j] : v[j];
            const float send = hi ? v[j] : v[n + j];
            v[j] = keep + __shfl_xor(send, off);
        }
    }
    float r = v[0];
    for (; off >= 1; off >>= 1) r += __shfl_xor(r, off);
    return r;
}

// ---- state update, N = 128 ---------------------------------------------------------------
// Block = (b, h, slice of 16 rows p); lane -> columns n4..n4+3, rows p0 = 16*slice + tid/32
// and p0 + 8.
template <typename T>
__global__ void __launch_bounds__(STEP_THREADS)
step_update_n128_kernel(const float *state_in, float *state_out, const T *__restrict__ x,
                        const T *__restrict__ dt, const float *__restrict__ A,
                        const float *__restrict__ D, const float *__restrict__ bc,
                        T *__restrict__ y, Shape s, int slices)
{
    constexpr int N = 128;
    const int sl = blockIdx.x % slices;
    const int h = (blockIdx.x / slices) % s.H;
    const int b = blockIdx.x / (slices * s.H);
    const int g = (h * s.G) / s.H;
    const int tid = threadIdx.x;
    const int n4 = (tid & 31) * 4;
    const int P = s.P;
    const int p0 = sl * 16 + (tid >> 5), p1 = p0 + 8;
    const bool ok0 = p0 < P, ok1 = p1 < P;
    const int q0 = min(p0, P - 1), q1 = min(p1, P - 1);
    const int64_t base = ((int64_t)b * s.H + h) * P * N;

    f32x4_t v0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(state_in + base + (int64_t)q0 * N + n4));
    f32x4_t v1 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(state_in + base + (int64_t)q1 * N + n4));
    const float *mix = bc + ((int64_t)b * s.G + g) * 2 * N + n4;
    const f32x4_t bm = *reinterpret_cast<const f32x4_t *>(mix);
    const f32x4_t cm = *reinterpret_cast<const f32x4_t *>(mix + N);
    const float dtv = to_float(dt[(int64_t)b * s.H + h]);
    const T *xr = x + ((int64_t)b * s.H + h) * P;
    const float x0 = to_float(xr[q0]), x1 = to_float(xr[q1]);
    const float decay = expf(dtv * A[h]);
    const float dsk = D ? D[h] : 0.f;
    const float u0 = dtv * x0, u1 = dtv * x1;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        v0[q] = decay * v0[q] + u0 * bm[q];
        v1[q] = decay * v1[q] + u1 * bm[q];
    }
    float part0 = (v0[0] * cm[0] + v0[1] * cm[1]) + (v0[2] * cm[2] + v0[3] * cm[3]);
    float part1 = (v1[0] * cm[0] + v1[1] * cm[1]) + (v1[2] * cm[2] + v1[3] * cm[3]);
    if (ok0) __builtin_nontemporal_store(v0, reinterpret_cast<f32x4_t *>(state_out + base + (int64_t)p0 * N + n4));
    if (ok1) __builtin_nontemporal_store(v1, reinterpret_cast<f32x4_t *>(state_out + base + (int64_t)p1 * N + n4));
    // both row sums in one butterfly: lanes 0..15 of the half wave end with row p0, 16..31 with p1
    float parts[2] = {part0, part1};
    const float tot = half_wave_sums<2>(parts, tid);
    if ((tid & 15) == 0) {
        T *yr = y + ((int64_t)b * s.H + h) * P;
        const bool second = (tid & 16) != 0;
        if (second ? ok1 : ok0) yr[second ? p1 : p0] = from_float<T>(tot + dsk * (second ? x1 : x0));
    }
}

// ---- several tokens per call, N = 128: same mapping; the state rows stay in registers while
// ---- the L tokens are applied one after the other (one read and one write of the state).
template <typename T>
__global__ void __launch_bounds__(STEP_THREADS)
step_multi_n128_kernel(const float *state_in, float *state_out, const T *__restrict__ x,
                       const T *__restrict__ dt, const float *__restrict__ A,
                       const float *__restrict__ D, const float *__restrict__ bc,
                       T *__restrict__ y, Shape s, int slices)
{
    constexpr int N = 128;
    const int sl = blockIdx.x % slices;
    const int h = (blockIdx.x / slices) % s.H;
    const int b = blockIdx.x / (slices * s.H);
    const int g = (h * s.G) / s.H;
    const int tid = threadIdx.x;
    const int n4 = (tid & 31) * 4;
    const int P = s.P, L = s.L;
    const int p0 = sl * 16 + (tid >> 5), p1 = p0 + 8;
    const bool ok0 = p0 < P, ok1 = p1 < P;
    const int q0 = min(p0, P - 1), q1 = min(p1, P - 1);
    const int64_t base = ((int64_t)b * s.H + h) * P * N;

    f32x4_t v0 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(state_in + base + (int64_t)q0 * N + n4));
    f32x4_t v1 = __builtin_nontemporal_load(reinterpret_cast<const f32x4_t *>(state_in + base + (int64_t)q1 * N + n4));
    const float Ah = A[h];
    const float dsk = D ? D[h] : 0.f;
    for (int t = 0; t < L; ++t) {
        const int64_t bt = (int64_t)b * L + t;
        const float *mix = bc + (bt * s.G + g) * 2 * N + n4;
        const f32x4_t bm = *reinterpret_cast<const f32x4_t *>(mix);
        const f32x4_t cm = *reinterpret_cast<const f32x4_t *>(mix + N);
        const float dtv = to_float(dt[bt * s.H + h]);
        const T *xr = x + (bt * s.H + h) * P;
        const float x0 = to_float(xr[q0]), x1 = to_float(xr[q1]);
        const float decay = expf(dtv * Ah);
        const float u0 = dtv * x0, u1 = dtv * x1;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            v0[q] = decay * v0[q] + u0 * bm[q];
            v1[q] = decay * v1[q] + u1 * bm[q];
        }
        // both row sums in one butterfly (5 shuffles instead of 10: the shuffles, not the arithmetic,
        // are what every further token costs): lanes 0..15 of the half wave end with row p0,
        // 16..31 with p1.  (Reducing 4 or 8 tokens' sums together was built and ran 2.4 x slower.)
        float parts[2] = {(v0[0] * cm[0] + v0[1] * cm[1]) + (v0[2] * cm[2] + v0[3] * cm[3]),
                          (v1[0] * cm[0] + v1[1] * cm[1]) + (v1[2] * cm[2] + v1[3] * cm[3])};
        const float tot = half_wave_sums<2>(parts, tid);
        if ((tid & 15) == 0) {
            T *yr = y + (bt * s.H + h) * P;
            const bool second = (tid & 16) != 0;
            if (second ? ok1 : ok0) yr[second ? p1 : p0] = from_float<T>(tot + dsk * (second ? x1 : x0));
        }
    }
    if (ok0) __builtin_nontemporal_store(v0, reinterpret_cast<f32x4_t *>(state_out + base + (int64_t)p0 * N + n4));
    if (ok1) __builtin_nontemporal_store(v1, reinterpret_cast<f32x4_t *>(state_out + base + (int64_t)p1 * N + n4));
}

// ---- state update, any N: block = (b, h), a wave walks one state row at a time ------------
template <typename T>
__global__ void __launch_bounds__(STEP_THREADS)
step_update_generic_kernel(const float *state_in, float *state_out, const T *__restrict__ x,
                           const T *__restrict__ dt, const float *__restrict__ A,
                           const float *__restrict__ D, const float *__restrict__ bc,
                           T *__restrict__ y, Shape s, int L, int t)
{
    // token t of L per sequence: x, dt, bc and y are indexed by bt = b * L + t
    const int b = blockIdx.x / s.H, h = blockIdx.x % s.H, g = (h * s.G) / s.H;
    const int64_t bt = (int64_t)b * L + t;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int N = s.N, P = s.P;
    const int64_t base = ((int64_t)b * s.H + h) * P * N;
    const float *bm = bc + (bt * s.G + g) * 2 * N;
    const float *cm = bm + N;
    const float dtv = to_float(dt[bt * s.H + h]);
    const float decay = expf(dtv * A[h]);
    const float dsk = D ? D[h] : 0.f;
    for (int p = wave; p < P; p += STEP_THREADS / 64) {
        const float xv = to_float(x[(bt * s.H + h) * P + p]);
        const float u = dtv * xv;
        float part = 0.f;
        for (int n = lane; n < N; n += 64) {
            const float v = decay * state_in[base + (int64_t)p * N + n] + u * bm[n];
            state_out[base + (int64_t)p * N + n] = v;
            part += v * cm[n];
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) part += __shfl_xor(part, off);
        if (lane == 0) y[(bt * s.H + h) * P + p] = from_float<T>(part + dsk * xv);
    }
}

template <typename T>
static swimba_status launch_step_t(const Shape &s, const float *state_in, float *state_out,
                                   const void *x, const void *dt, const float *A, const float *D,
                                   const void *Be, const void *Ce, const void *logits, void *y,
                                   int32_t *idx, float *bc, hipStream_t st)
{
    const int64_t blocks = (int64_t)s.B * s.H;
    if (blocks == 0) return SWIMBA_OK;
    hipLaunchKernelGGL(step_mix_kernel<T>, dim3((unsigned)(s.B * s.G)), dim3(128), 0, st,
                       (const T *)Be, (const T *)Ce, (const T *)logits, bc, idx, s);
    SWIMBA_CHECK_LAUNCH();
    const int slices = (s.P + 15) / 16;
    if (s.N == 128 && blocks * slices < (1ll << 31))
        hipLaunchKernelGGL(step_update_n128_kernel<T>, dim3((unsigned)(blocks * slices)),
                           dim3(STEP_THREADS), 0, st, state_in, state_out, (const T *)x, (const T *)dt,
                           A, D, bc, (T *)y, s, slices);
    else
        hipLaunchKernelGGL(step_update_generic_kernel<T>, dim3((unsigned)blocks), dim3(STEP_THREADS), 0,
                           st, state_in, state_out, (const T *)x, (const T *)dt, A, D, bc, (T *)y, s, 1, 0);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

// L tokens per sequence: x (B,L,H,P), dt (B,L,H), Be/Ce (B,L,E,G,N), logits (B,L,E), y (B,L,H,P),
// idx (B,L,k), bc (B,L,G,2N) fp32.  The token loop of the general-N path is a loop of launches.
template <typename T>
static swimba_status launch_step_multi_t(const Shape &s, const float *state_in, float *state_out,
                                         const void *x, const void *dt, const float *A, const float *D,
                                         const void *Be, const void *Ce, const void *logits, void *y,
                                         int32_t *idx, float *bc, hipStream_t st)
{
    const int64_t blocks = (int64_t)s.B * s.H;
    if (blocks == 0 || s.L == 0) return SWIMBA_OK;
    Shape tok = s;                 // the mix kernel sees B*L independent tokens
    tok.B = s.B * s.L;
    tok.L = 1;
    hipLaunchKernelGGL(step_mix_kernel<T>, dim3((unsigned)(tok.B * s.G)), dim3(128), 0, st, (const T *)Be,
                       (const T *)Ce, (const T *)logits, bc, idx, tok);
    SWIMBA_CHECK_LAUNCH();
    const int slices = (s.P + 15) / 16;
    if (s.N == 128 && blocks * slices < (1ll << 31)) {
        hipLaunchKernelGGL(step_multi_n128_kernel<T>, dim3((unsigned)(blocks * slices)), dim3(STEP_THREADS), 0,
                           st, state_in, state_out, (const T *)x, (const T *)dt, A, D, bc, (T *)y, s, slices);
        SWIMBA_CHECK_LAUNCH();
        return SWIMBA_OK;
    }
    // any N: one launch per token
    for (int t = 0; t < s.L; ++t) {
        hipLaunchKernelGGL(step_update_generic_kernel<T>, dim3((unsigned)blocks), dim3(STEP_THREADS), 0, st,
                           t == 0 ? state_in : state_out, state_out, (const T *)x, (const T *)dt, A, D, bc,
                           (T *)y, s, s.L, t);
        SWIMBA_CHECK_LAUNCH();
    }
    return SWIMBA_OK;
}

swimba_status launch_step_multi(const Shape &s, int io_dtype, const float *state_in, float *state_out,
                                const void *x, const void *dt, const float *A, const float *D,
                                const void *Be, const void *Ce, const void *logits, void *y, int32_t *idx,
                                float *bc, hipStream_t st)
{
    if (io_dtype == SWIMBA_BF16)
        return launch_step_multi_t<bf16>(s, state_in, state_out, x, dt, A, D, Be, Ce, logits, y, idx, bc, st);
    return launch_step_multi_t<float>(s, state_in, state_out, x, dt, A, D, Be, Ce, logits, y, idx, bc, st);
}

// Device address of `scratch` on the current device, looked up once per device.
static swimba_status static_scratch(float **out)
{
    constexpr int MAXDEV = 64;
    static std::atomic<float *> ptr[MAXDEV];
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
    if (dev < 0 || dev >= MAXDEV) return SWIMBA_ERR_UNSUPPORTED;
    float *p = ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress((void **)&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
        ptr[dev].store(p, std::memory_order_release);   // every thread that gets here stores the same address
    }
    *out = p;
    return SWIMBA_OK;
}

swimba_status launch_step_static(const Shape &s, int io_dtype, const float *state_in, float *state_out,
                                 const void *x, const void *dt, const float *A, const float *D,
                                 const void *Be, const void *Ce, const void *logits, void *y, int32_t *idx,
                                 hipStream_t st)
{
    if ((int64_t)s.B * s.G * s.N * 2 * (int64_t)sizeof(float) > (int64_t)SWIMBA_STATIC_SCRATCH_BYTES)
        return SWIMBA_ERR_UNSUPPORTED;
    float *bc = nullptr;
    const swimba_status rs = static_scratch(&bc);
    if (rs != SWIMBA_OK) return rs;
    // the mix kernel overwrites every element the update kernel reads: nothing has to be cleared
    return launch_step(s, io_dtype, state_in, state_out, x, dt, A, D, Be, Ce, logits, y, idx, bc, st);
}

swimba_status launch_step(const Shape &s, int io_dtype, const float *state_in, float *state_out,
                          const void *x, const void *dt, const float *A, const float *D,
                          const void *Be, const void *Ce, const void *logits, void *y, int32_t *idx,
                          float *bc, hipStream_t st)
{
    if (io_dtype == SWIMBA_BF16)
        return launch_step_t<bf16>(s, state_in, state_out, x, dt, A, D, Be, Ce, logits, y, idx, bc, st);
    return launch_step_t<float>(s, state_in, state_out, x, dt, A, D, Be, Ce, logits, y, idx, bc, st);
}

}  // namespace swimba
