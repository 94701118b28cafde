// bf16 MFMA SSD chunk kernels for P = 64, N = 128, Q in {64, 128, 256}
// (paper, background section on SSD: matrix multiplications inside chunks;
// Theorem 1: the mixed streams feed one plain SSM).
//
// Both kernels gather the k active expert rows of every token, mix them with
// the router weights in fp32 and round the mix to bf16 while staging it into
// LDS (or straight into MFMA operand registers): the mixed B/C streams never
// exist in HBM.
//
// MFMA used: v_mfma_f32_32x32x16_bf16.  Lane l of a wave holds
//   A[row = l%32][k = 8*(l/32) + 0..7],  B[k = 8*(l/32) + 0..7][col = l%32],
//   C[row = 8*(v/4) + 4*(l/32) + v%4][col = l%32] in accumulator register v.
// The k index of a contraction may be permuted freely as long as A and B use
// the same permutation; this is used to read 16 contiguous bytes per operand.
#include "common.hpp"

namespace swimba {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float f32x2_t;
typedef __attribute__((ext_vector_type(16))) float f32x16_t;

constexpr int MP = 64;    // headdim
constexpr int MN = 128;   // state size
constexpr int MTHREADS = 256;

__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi)
{
    f32x2_t f = {lo, hi};
    bf16x2_t h = __builtin_convertvector(f, bf16x2_t);   // round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}
__device__ __forceinline__ float bf_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }

__device__ __forceinline__ f32x16_t mfma32(uint4 a, uint4 b, f32x16_t c)
{
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8_t, a),
                                                   __builtin_bit_cast(bf16x8_t, b), c, 0, 0, 0);
}

// acc[0..7] += wgt * (8 bf16 values packed in u)
__device__ __forceinline__ void fma_bf16x8(float *acc, uint4 u, float wgt)
{
    acc[0] += wgt * bf_lo(u.x); acc[1] += wgt * bf_hi(u.x);
    acc[2] += wgt * bf_lo(u.y); acc[3] += wgt * bf_hi(u.y);
    acc[4] += wgt * bf_lo(u.z); acc[5] += wgt * bf_hi(u.z);
    acc[6] += wgt * bf_lo(u.w); acc[7] += wgt * bf_hi(u.w);
}
__device__ __forceinline__ uint4 pack8(const float *a)
{
    return make_uint4(pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(a[4], a[5]),
                      pack_bf16x2(a[6], a[7]));
}

// Workgroups are handed to the 8 XCDs round-robin by block id.  This maps a
// block id to a logical id such that each XCD works on one contiguous range of
// logical ids (neighbouring heads of one chunk share expert rows in that
// XCD's L2).  The grid is padded to a multiple of 8; ids >= total do nothing.
__device__ __forceinline__ int xcd_logical_id(int bid, int nblocks)
{
    const int per = nblocks >> 3;
    return (bid & 7) * per + (bid >> 3);
}
static inline int xcd_padded(int64_t total) { return (int)((total + 7) / 8 * 8); }

// =========================================================================================
// Chunk state:  S_c[p][n] = sum_j coef_j x[j][p] Bmix[j][n],  coef_j = dt_j exp(cs_last - cs_j)
// One workgroup = (batch, chunk, group, a run of `hg` heads of that group).  The
// mixed B tile is staged once, transposed ([n][j]), and reused by the heads.
// =========================================================================================
template <int Q>
__global__ void __launch_bounds__(MTHREADS)
chunk_state_mfma_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dt,
                        const uint16_t *__restrict__ Be, const int32_t *__restrict__ idx,
                        const float *__restrict__ w, const float *__restrict__ cs,
                        float *__restrict__ states, Shape s, int hg, int nhg, int total, int nblocks)
{
    constexpr int STR = Q + 8;                    // row stride of both transposed tiles (elements)
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint16_t *sBt = reinterpret_cast<uint16_t *>(smem_raw);            // [MN][STR]
    uint16_t *sXt = sBt + MN * STR;                                     // [MP][STR]
    float *s_coef = reinterpret_cast<float *>(sXt + MP * STR);          // [Q]

    const int lid = xcd_logical_id(blockIdx.x, nblocks);
    if (lid >= total) return;
    const int hgi = lid % nhg;
    const int g = (lid / nhg) % s.G;
    const int c = (lid / (nhg * s.G)) % s.nc;
    const int b = lid / (nhg * s.G * s.nc);
    const int hpg = s.H / s.G;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kg = lane >> 5;
    const int64_t tok0 = (int64_t)b * s.L + (int64_t)c * Q;   // first token of the chunk
    const int valid = min(Q, s.L - c * Q);                     // tokens of this chunk inside L

    // ---- mixed B, transposed: unit = (8 consecutive tokens) x (8 consecutive n) ----
    for (int u = tid; u < (Q / 8) * 16; u += MTHREADS) {
        const int jg = u >> 4, piece = u & 15;
        float acc[8][8];
#pragma unroll
        for (int jj = 0; jj < 8; ++jj) {
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[jj][e] = 0.f;
            const int j = jg * 8 + jj;
            if (j < valid) {
                const int64_t bt = tok0 + j;
                const uint16_t *rowbase = Be + (bt * s.E * s.G + g) * MN + piece * 8;
                for (int r = 0; r < s.K; ++r) {
                    const int e = idx[bt * s.K + r];
                    const float wr = w[bt * s.K + r];
                    const uint4 v = *reinterpret_cast<const uint4 *>(rowbase + (int64_t)e * s.G * MN);
                    fma_bf16x8(acc[jj], v, wr);
                }
            }
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            float col[8];
#pragma unroll
            for (int jj = 0; jj < 8; ++jj) col[jj] = acc[jj][e];
            *reinterpret_cast<uint4 *>(sBt + (piece * 8 + e) * STR + jg * 8) = pack8(col);
        }
    }

    for (int hh = 0; hh < hg; ++hh) {
        const int hin = hgi * hg + hh;
        if (hin >= hpg) break;
        const int h = g * hpg + hin;
        const float *csr = cs + (((int64_t)b * s.nc + c) * s.H + h) * Q;
        __syncthreads();   // previous head's MFMA reads of sXt / s_coef are done
        if (tid < Q) {
            float cf = 0.f;
            if (tid < valid)
                cf = to_float(bf16{dt[(tok0 + tid) * s.H + h]}) * expf(csr[Q - 1] - csr[tid]);
            s_coef[tid] = cf;
        }
        __syncthreads();
        // ---- coefficient-weighted x, transposed: unit = (8 tokens) x (2 channels) ----
        for (int u = tid; u < (Q / 8) * 32; u += MTHREADS) {
            const int p2 = u & 31, jg = u >> 5;
            float xa[8], xb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = jg * 8 + e;
                uint32_t v = 0;
                if (j < valid)
                    v = *reinterpret_cast<const uint32_t *>(x + ((tok0 + j) * s.H + h) * MP + 2 * p2);
                const float cf = s_coef[j];
                xa[e] = bf_lo(v) * cf;
                xb[e] = bf_hi(v) * cf;
            }
            *reinterpret_cast<uint4 *>(sXt + (2 * p2) * STR + jg * 8) = pack8(xa);
            *reinterpret_cast<uint4 *>(sXt + (2 * p2 + 1) * STR + jg * 8) = pack8(xb);
        }
        __syncthreads();
        // ---- S[p][n]: wave -> 32 columns n, both 32-row halves of p ----
        f32x16_t acc0 = {0}, acc1 = {0};
#pragma unroll 4
        for (int ks = 0; ks < Q / 16; ++ks) {
            const int kb = ks * 16 + kg * 8;
            const uint4 a0 = *reinterpret_cast<const uint4 *>(sXt + l32 * STR + kb);
            const uint4 a1 = *reinterpret_cast<const uint4 *>(sXt + (32 + l32) * STR + kb);
            const uint4 bf = *reinterpret_cast<const uint4 *>(sBt + (wave * 32 + l32) * STR + kb);
            acc0 = mfma32(a0, bf, acc0);
            acc1 = mfma32(a1, bf, acc1);
        }
        float *out = states + (((int64_t)b * s.nc + c) * s.H + h) * MP * MN + wave * 32 + l32;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int p = 8 * (v >> 2) + 4 * kg + (v & 3);
            out[(int64_t)p * MN] = acc0[v];
            out[(int64_t)(32 + p) * MN] = acc1[v];
        }
    }
}

template <int Q>
static swimba_status launch_cs_q(const Shape &s, const void *x, const void *dt, const void *Be,
                                 const int32_t *idx, const float *w, const float *cs, float *states,
                                 hipStream_t st)
{
    const int hpg = s.H / s.G;
    // heads per workgroup: reuse the staged B tile, but keep >= ~2 workgroups per CU
    int hg = hpg;
    while (hg > 1 && (int64_t)s.B * s.nc * s.G * ((hpg + hg - 1) / hg) < 512) hg = (hg + 1) / 2;
    const int nhg = (hpg + hg - 1) / hg;
    const int64_t total = (int64_t)s.B * s.nc * s.G * nhg;
    if (total == 0) return SWIMBA_OK;
    const int nblocks = xcd_padded(total);
    const size_t shm = (size_t)(MN + MP) * (Q + 8) * 2 + Q * sizeof(float);
    static bool attr_set = false;
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute((const void *)chunk_state_mfma_kernel<Q>,
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
        attr_set = true;
    }
    hipLaunchKernelGGL(chunk_state_mfma_kernel<Q>, dim3(nblocks), dim3(MTHREADS), shm, st,
                       (const uint16_t *)x, (const uint16_t *)dt, (const uint16_t *)Be, idx, w, cs,
                       states, s, hg, nhg, (int)total, nblocks);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_chunk_state_mfma(const Shape &s, const void *x, const void *dt, const void *Be,
                                      const int32_t *idx, const float *w, const float *cs,
                                      float *states, hipStream_t st)
{
    switch (s.Q) {
    case 64: return launch_cs_q<64>(s, x, dt, Be, idx, w, cs, states, st);
    case 128: return launch_cs_q<128>(s, x, dt, Be, idx, w, cs, states, st);
    case 256: return launch_cs_q<256>(s, x, dt, Be, idx, w, cs, states, st);
    }
    return SWIMBA_ERR_UNSUPPORTED;
}

// =========================================================================================
// Output:  y_i = sum_{j<=i} (Cmix_i.Bmix_j) exp(cs_i-cs_j) dt_j x_j + exp(cs_i) Cmix_i.H_c + D x_i
// One workgroup = (batch, chunk, head).  The chunk is cut into 32-token tiles; wave w
// owns output tiles {w, NT-1-w} (balanced under the causal mask) and keeps their
// mixed C rows in registers for the whole kernel.  Mixed B and dt-weighted x arrive
// through LDS in blocks of 64 tokens.
//
// Per tile pair (I, J), J <= I:  G^T[j][i] = Bmix_j . Cmix_i on MFMA (acc rows j, cols i),
// decay applied in registers, result used directly as the A operand of Y += M X.
// For J < I the decay factors as exp(cs_i - R_J) * exp(R_J - cs_j) with R_J = cs at the
// last token of tile J; both factors are <= 1 (cs is non-increasing), so nothing
// overflows and only one exp per lane is needed; the second factor is tabulated per
// token.  The diagonal tile uses exp(cs_i - cs_j) under the mask i >= j.
// =========================================================================================
template <int Q>
__global__ void __launch_bounds__(MTHREADS, 2)
output_mfma_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dt,
                   const float *__restrict__ D, const uint16_t *__restrict__ Be,
                   const uint16_t *__restrict__ Ce, const int32_t *__restrict__ idx,
                   const float *__restrict__ w, const float *__restrict__ cs,
                   const uint16_t *__restrict__ Hlp, uint16_t *__restrict__ y, Shape s, int total,
                   int nblocks)
{
    constexpr int NT = Q / 32;                 // 32-token tiles in the chunk
    constexpr int NB = Q / 64;                 // 64-token staging blocks
    constexpr int SLOTS = (NT >= 8) ? 2 : 1;   // output tiles per wave
    constexpr int BSTR = MN + 8;               // row stride of the mixed-B / carried-state tile
    constexpr int XSTR = 64 + 8;               // row stride of the transposed x block
    __shared__ __align__(16) uint16_t sB[64 * BSTR];
    __shared__ __align__(16) uint16_t sX[MP * XSTR];
    __shared__ float s_cs[Q], s_dt[Q], s_f[Q];

    const int lid = xcd_logical_id(blockIdx.x, nblocks);
    if (lid >= total) return;
    const int h = lid % s.H;
    const int c = (lid / s.H) % s.nc;
    const int b = lid / (s.H * s.nc);
    const int g = (h * s.G) / s.H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, kg = lane >> 5;
    const int64_t tok0 = (int64_t)b * s.L + (int64_t)c * Q;
    const int valid = min(Q, s.L - c * Q);

    // tiles owned by this wave (-1 = none)
    int tileI[SLOTS];
    tileI[0] = (wave < NT) ? wave : -1;
    if constexpr (SLOTS == 2) tileI[1] = NT - 1 - wave;

    // ---- per-token scalars of the chunk ----
    if (tid < Q) {
        s_cs[tid] = cs[(((int64_t)b * s.nc + c) * s.H + h) * Q + tid];
        s_dt[tid] = (tid < valid) ? to_float(bf16{dt[(tok0 + tid) * s.H + h]}) : 0.f;
    }
    __syncthreads();
    if (tid < Q) s_f[tid] = expf(s_cs[(tid | 31)] - s_cs[tid]);

    // ---- mixed C rows of the owned tiles -> MFMA operand registers ----
    // lane (i = l32, kg) holds n = 64*kg + 8*ks + 0..7 for ks = 0..7
    uint4 cfrag[SLOTS][8];
    float csi[SLOTS];
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl) {
        float acc[8][8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[ks][e] = 0.f;
        csi[sl] = 0.f;
        if (tileI[sl] >= 0) {
            const int i = tileI[sl] * 32 + l32;
            csi[sl] = s_cs[i];
            if (i < valid) {
                const int64_t bt = tok0 + i;
                const uint16_t *rowbase = Ce + (bt * s.E * s.G + g) * MN + 64 * kg;
                for (int r = 0; r < s.K; ++r) {
                    const int e = idx[bt * s.K + r];
                    const float wr = w[bt * s.K + r];
                    const uint16_t *row = rowbase + (int64_t)e * s.G * MN;
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks)
                        fma_bf16x8(acc[ks], *reinterpret_cast<const uint4 *>(row + ks * 8), wr);
                }
            }
        }
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) cfrag[sl][ks] = pack8(acc[ks]);
    }

    // ---- carried state of the chunk (bf16) -> LDS, then Y_off = exp(cs_i) Cmix_i . H_c ----
    {
        const uint16_t *Hc = Hlp + (((int64_t)b * s.nc + c) * s.H + h) * MP * MN;
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int row = (tid >> 4) + 16 * pass, piece = tid & 15;
            *reinterpret_cast<uint4 *>(sB + row * BSTR + piece * 8) =
                *reinterpret_cast<const uint4 *>(Hc + row * MN + piece * 8);
        }
    }
    __syncthreads();
    f32x16_t yacc[SLOTS][2];
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl) {
        yacc[sl][0] = f32x16_t{0};
        yacc[sl][1] = f32x16_t{0};
        if (tileI[sl] >= 0) {
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) {
                const uint4 h0 = *reinterpret_cast<const uint4 *>(sB + l32 * BSTR + 64 * kg + ks * 8);
                const uint4 h1 = *reinterpret_cast<const uint4 *>(sB + (32 + l32) * BSTR + 64 * kg + ks * 8);
                yacc[sl][0] = mfma32(cfrag[sl][ks], h0, yacc[sl][0]);
                yacc[sl][1] = mfma32(cfrag[sl][ks], h1, yacc[sl][1]);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int il = 8 * (v >> 2) + 4 * kg + (v & 3);
                const float sc = expf(s_cs[tileI[sl] * 32 + il]);
                yacc[sl][0][v] *= sc;
                yacc[sl][1][v] *= sc;
            }
        }
    }

    // ---- intra-chunk part, 64 tokens of j at a time ----
#pragma unroll 1
    for (int jb = 0; jb < NB; ++jb) {
        __syncthreads();   // everyone is done reading sB / sX of the previous block
        // mixed B rows of the block, row-major
#pragma unroll
        for (int pass = 0; pass < 4; ++pass) {
            const int row = (tid >> 4) + 16 * pass, piece = tid & 15;
            const int j = jb * 64 + row;
            float acc[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = 0.f;
            if (j < valid) {
                const int64_t bt = tok0 + j;
                const uint16_t *rowbase = Be + (bt * s.E * s.G + g) * MN + piece * 8;
                for (int r = 0; r < s.K; ++r) {
                    const int e = idx[bt * s.K + r];
                    const float wr = w[bt * s.K + r];
                    fma_bf16x8(acc, *reinterpret_cast<const uint4 *>(rowbase + (int64_t)e * s.G * MN), wr);
                }
            }
            *reinterpret_cast<uint4 *>(sB + row * BSTR + piece * 8) = pack8(acc);
        }
        // dt_j * x_j, transposed to [p][j'], j' = position of j in the operand order
        {
            const int p2 = tid & 31, gi = tid >> 5;
            const int t16 = gi >> 1, kgx = gi & 1;
            float xa[8], xb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int jj = 16 * t16 + 8 * (e >> 2) + 4 * kgx + (e & 3);
                const int j = jb * 64 + jj;
                uint32_t v = 0;
                if (j < valid)
                    v = *reinterpret_cast<const uint32_t *>(x + ((tok0 + j) * s.H + h) * MP + 2 * p2);
                const float d = s_dt[j];
                xa[e] = bf_lo(v) * d;
                xb[e] = bf_hi(v) * d;
            }
            *reinterpret_cast<uint4 *>(sX + (2 * p2) * XSTR + 16 * t16 + 8 * kgx) = pack8(xa);
            *reinterpret_cast<uint4 *>(sX + (2 * p2 + 1) * XSTR + 16 * t16 + 8 * kgx) = pack8(xb);
        }
        __syncthreads();

#pragma unroll
        for (int jt = 0; jt < 2; ++jt) {
            const int J = 2 * jb + jt;
#pragma unroll
            for (int sl = 0; sl < SLOTS; ++sl) {
                const int I = tileI[sl];
                if (I < J) continue;   // uniform per wave
                f32x16_t gacc = {0};
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    const uint4 bfrag =
                        *reinterpret_cast<const uint4 *>(sB + (jt * 32 + l32) * BSTR + 64 * kg + ks * 8);
                    gacc = mfma32(bfrag, cfrag[sl][ks], gacc);
                }
                float m[16];
                if (I > J) {
                    const float ei = expf(csi[sl] - s_cs[J * 32 + 31]);
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int jl = 8 * (v >> 2) + 4 * kg + (v & 3);
                        m[v] = gacc[v] * (ei * s_f[J * 32 + jl]);
                    }
                } else {
#pragma unroll
                    for (int v = 0; v < 16; ++v) {
                        const int jl = 8 * (v >> 2) + 4 * kg + (v & 3);
                        const float dcy = expf(fminf(csi[sl] - s_cs[J * 32 + jl], 0.f));
                        m[v] = (l32 >= jl) ? gacc[v] * dcy : 0.f;
                    }
                }
#pragma unroll
                for (int t = 0; t < 2; ++t) {
                    const uint4 mfrag = pack8(m + 8 * t);
                    const uint4 x0 = *reinterpret_cast<const uint4 *>(sX + l32 * XSTR + jt * 32 + 16 * t + 8 * kg);
                    const uint4 x1 = *reinterpret_cast<const uint4 *>(sX + (32 + l32) * XSTR + jt * 32 + 16 * t + 8 * kg);
                    yacc[sl][0] = mfma32(mfrag, x0, yacc[sl][0]);
                    yacc[sl][1] = mfma32(mfrag, x1, yacc[sl][1]);
                }
            }
        }
    }

    // ---- y = acc + D x ----
    const float dsk = D ? D[h] : 0.f;
#pragma unroll
    for (int sl = 0; sl < SLOTS; ++sl) {
        if (tileI[sl] < 0) continue;
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = tileI[sl] * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
            if (i < valid) {
                const int64_t off = ((tok0 + i) * s.H + h) * MP + l32;
                y[off] = bf16_bits_rne(yacc[sl][0][v] + dsk * to_float(bf16{x[off]}));
                y[off + 32] = bf16_bits_rne(yacc[sl][1][v] + dsk * to_float(bf16{x[off + 32]}));
            }
        }
    }
}

template <int Q>
static swimba_status launch_out_q(const Shape &s, const void *x, const void *dt, const float *D,
                                  const void *Be, const void *Ce, const int32_t *idx, const float *w,
                                  const float *cs, const void *Hlp, void *y, hipStream_t st)
{
    const int64_t total = (int64_t)s.B * s.nc * s.H;
    if (total == 0) return SWIMBA_OK;
    const int nblocks = xcd_padded(total);
    hipLaunchKernelGGL(output_mfma_kernel<Q>, dim3(nblocks), dim3(MTHREADS), 0, st,
                       (const uint16_t *)x, (const uint16_t *)dt, D, (const uint16_t *)Be,
                       (const uint16_t *)Ce, idx, w, cs, (const uint16_t *)Hlp, (uint16_t *)y, s,
                       (int)total, nblocks);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_output_mfma(const Shape &s, const void *x, const void *dt, const float *D,
                                 const void *Be, const void *Ce, const int32_t *idx, const float *w,
                                 const float *cs, const void *states_lp, void *y, hipStream_t st)
{
    switch (s.Q) {
    case 64: return launch_out_q<64>(s, x, dt, D, Be, Ce, idx, w, cs, states_lp, y, st);
    case 128: return launch_out_q<128>(s, x, dt, D, Be, Ce, idx, w, cs, states_lp, y, st);
    case 256: return launch_out_q<256>(s, x, dt, D, Be, Ce, idx, w, cs, states_lp, y, st);
    }
    return SWIMBA_ERR_UNSUPPORTED;
}

}  // namespace swimba
