// Routed expert in-projection (paper, MoE-parameterized SSM: the expert streams are
// expert-specific linear projections of the same token features, and only the experts of the
// active set K_t enter the mix): for every token t and every e in K_t
//   B_t^(e)[c] = sum_d W_B[e][c][d] u_t[d],   C_t^(e)[c] = sum_d W_C[e][c][d] u_t[d],
// written either into the dense (B,L,E,G,N) layout (rows of inactive experts are not touched:
// the mixer never reads them) or, with `compact`, into (B,L,k,G,N): row r of a token is the
// stream of its r-th selected expert, so no buffer with an expert axis exists at all.
//
// Three launches: clear the per-expert counters; route every token and append the entry
// t*k + r to the list of its r-th expert (LDS counters per block, one global atomic per block
// and expert); a grouped GEMM over (expert, 64-entry tile of its list, 256 output columns).
// The GEMM is a dense contraction, so it runs on v_mfma_f32_32x32x16_bf16.  Both operands
// are stored with the contraction index d contiguous (weights as (out, in), like a linear
// layer), which is the 8-consecutive-k operand layout.  The product is computed transposed,
// out^T[c][token], with the weight rows permuted so that a lane ends up with 16 consecutive
// output columns of one token (two 16-byte stores).
#include "common.hpp"

namespace swimba {

typedef __attribute__((ext_vector_type(8))) __bf16 pj_bf16x8_t;
typedef __attribute__((ext_vector_type(2))) __bf16 pj_bf16x2_t;
typedef __attribute__((ext_vector_type(2))) float pj_f32x2_t;
typedef __attribute__((ext_vector_type(16))) float pj_f32x16_t;

constexpr int PJ_TOK = 64;     // list entries (tokens) per workgroup tile
constexpr int PJ_COLS = 256;   // output columns per workgroup: 4 waves x 64

__global__ void proj_clear_kernel(int32_t *counts, int E)
{
    for (int e = threadIdx.x; e < E; e += blockDim.x) counts[e] = 0;
}

// one token per lane: top-k routing, then one list entry per active expert
template <typename T>
__global__ void __launch_bounds__(256)
proj_route_kernel(const T *__restrict__ logits, int32_t *__restrict__ idx, float *__restrict__ w,
                  int32_t *__restrict__ counts, int32_t *__restrict__ lists, int64_t tokens, int E, int K)
{
    __shared__ int32_t s_cnt[SWIMBA_MAX_EXPERTS], s_base[SWIMBA_MAX_EXPERTS];
    extern __shared__ int32_t s_loc[];                       // [256][K] rank inside the block
    const int tid = threadIdx.x;
    const int64_t t = (int64_t)blockIdx.x * 256 + tid;
    for (int e = tid; e < E; e += 256) s_cnt[e] = 0;
    __syncthreads();
    if (t < tokens) {
        const T *g = logits + t * E;
        route_token([&](int e) { return to_float(g[e]); }, E, K, idx + t * K, w + t * K);
        for (int r = 0; r < K; ++r) s_loc[tid * K + r] = atomicAdd(&s_cnt[idx[t * K + r]], 1);
    }
    __syncthreads();
    for (int e = tid; e < E; e += 256) s_base[e] = s_cnt[e] ? atomicAdd(&counts[e], s_cnt[e]) : 0;
    __syncthreads();
    if (t < tokens) {
        for (int r = 0; r < K; ++r) {
            const int e = idx[t * K + r];
            lists[(int64_t)e * tokens + s_base[e] + s_loc[tid * K + r]] = (int32_t)(t * K + r);
        }
    }
}

__device__ __forceinline__ uint32_t pj_pack(float lo, float hi)
{
    pj_f32x2_t f = {lo, hi};
    pj_bf16x2_t h = __builtin_convertvector(f, pj_bf16x2_t);   // round to nearest even
    return __builtin_bit_cast(uint32_t, h);
}

// Workgroup = (expert, 64-entry tile of its token list, block of 256 output columns);
// wave w owns columns 64w..64w+63 of the block and all 64 entries: 2 x 2 MFMA tiles.
// The contraction runs in stages of 64 features.  A stage of both operands (256 weight rows,
// 64 token rows, 128 bytes each) is read with fully coalesced 16-byte loads (8 lanes per
// row), parked in registers while the previous stage is multiplied, and then passed through
// LDS, from where the lanes read their operand registers.
constexpr int PJ_KT = 64;             // features per stage
constexpr int PJ_STR = PJ_KT + 8;     // LDS row stride (elements): rows stay 16-byte aligned
constexpr int PJ_UD = 2;              // stages the token-row loads run ahead (even); 6 measured no faster

__global__ void __launch_bounds__(256)
proj_mfma_kernel(const uint16_t *__restrict__ u, const uint16_t *__restrict__ WB,
                 const uint16_t *__restrict__ WC, const int32_t *__restrict__ counts,
                 const int32_t *__restrict__ lists, uint16_t *__restrict__ Be, uint16_t *__restrict__ Ce,
                 int64_t tokens, int E, int K, int GN, int Dm, int tiles_max, int compact)
{
    __shared__ __align__(16) uint16_t sW[PJ_COLS * PJ_STR];
    __shared__ __align__(16) uint16_t sU[PJ_TOK * PJ_STR];
    // Consecutive block ids go to consecutive XCDs (8 of them, each with its own L2).  Expert e
    // is served by XCD e % 8 only, so that an XCD's L2 holds the weights of E/8 experts instead
    // of all of them (3 MB of weights per 8 experts at 768 features would fill a 4 MB L2).
    const int xcd = blockIdx.x & 7, j = blockIdx.x >> 3;
    const int e = xcd + 8 * (j / tiles_max), tile = j % tiles_max;
    if (e >= E) return;
    const int cnt = counts[e];
    if (tile * PJ_TOK >= cnt) return;                        // whole workgroup: no barrier is skipped
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int colblk = blockIdx.y * PJ_COLS;                 // first column of the block in [B | C]
    const int col0 = colblk + wave * 64;
    const bool active = col0 < 2 * GN;                       // wave-uniform; idle waves still stage
    const int l32 = lane & 31, kg = lane >> 5;
    const int nvalid = min(PJ_TOK, cnt - tile * PJ_TOK);
    const int32_t *lst = lists + (int64_t)e * tokens + tile * PJ_TOK;

    // ---- staging map: lane -> 16-byte piece `piece` of rows row0 + 32 i ----
    const int piece = tid & 7, row0 = tid >> 3;
    const uint16_t *wsrc[8], *usrc[2];
#pragma unroll
    for (int i = 0; i < 8; ++i) {
        const int c = min(colblk + row0 + 32 * i, 2 * GN - 1);          // rows past [B | C] repeat the last one
        wsrc[i] = (c < GN ? WB + ((int64_t)e * GN + c) * Dm : WC + ((int64_t)e * GN + c - GN) * Dm);
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) usrc[i] = u + (int64_t)(lst[min(row0 + 32 * i, nvalid - 1)] / K) * Dm;
    // Register sets: the weight rows of stage i + 2 (L2 hits) and the token rows of stage i + PJ_UD
    // (scattered 128-byte reads that mostly come from HBM) are requested while stage i is
    // multiplied.  All loads are clamped and
    // unconditional, so that the waits on them stay exact counts; the issues past the last
    // stage re-read it and are not used.
    const int k_last = ((Dm - 1) / PJ_KT) * PJ_KT;
    uint4 wreg[2][8], ureg[PJ_UD][2];
    auto load_w = [&](uint4 (&wr)[8], int k0) __attribute__((always_inline)) {
        const int kk = min(min(k0, k_last) + piece * 8, Dm - 8);   // a short last stage stays inside the row
#pragma unroll
        for (int i = 0; i < 8; ++i) wr[i] = *reinterpret_cast<const uint4 *>(wsrc[i] + kk);
    };
    auto load_u = [&](uint4 (&ur)[2], int k0) __attribute__((always_inline)) {
        const int kk = min(min(k0, k_last) + piece * 8, Dm - 8);
#pragma unroll
        for (int i = 0; i < 2; ++i) ur[i] = *reinterpret_cast<const uint4 *>(usrc[i] + kk);
    };

    // Operand row r of a 32-column weight tile must hold column 16*((r>>2)&1) + 4*(r>>3) + (r&3)
    // for accumulator register v of lane (l32, kg) to be column 16 kg + v of the tile.  The
    // permutation is applied when the rows are staged (column x goes to LDS row wrow), so the
    // lanes of a wave read consecutive LDS rows: no bank conflicts.
    const int wrow = 8 * ((row0 >> 2) & 3) + 4 * ((row0 >> 4) & 1) + (row0 & 3);
    const uint16_t *aop[2], *bop[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        aop[q] = sW + (wave * 64 + 32 * q + l32) * PJ_STR + 8 * kg;
        bop[q] = sU + (32 * q + l32) * PJ_STR + 8 * kg;
    }
    pj_f32x16_t acc[2][2];
#pragma unroll
    for (int ct = 0; ct < 2; ++ct)
#pragma unroll
        for (int rt = 0; rt < 2; ++rt) acc[ct][rt] = pj_f32x16_t{0};

    // one stage: registers -> LDS, refill the registers two stages ahead, multiply from LDS
    auto stage = [&](uint4 (&wr)[8], uint4 (&ur)[2], int k0) __attribute__((always_inline)) {
        lds_barrier();                                       // every wave is done with the previous stage
        // pieces past the end of a short last stage are staged as zeros: every stage is 4 k-steps
        const bool inside = k0 + piece * 8 < Dm;
#pragma unroll
        for (int i = 0; i < 8; ++i)
            *reinterpret_cast<uint4 *>(sW + (wrow + 32 * i) * PJ_STR + piece * 8) =
                inside ? wr[i] : make_uint4(0, 0, 0, 0);
#pragma unroll
        for (int i = 0; i < 2; ++i)
            *reinterpret_cast<uint4 *>(sU + (row0 + 32 * i) * PJ_STR + piece * 8) =
                inside ? ur[i] : make_uint4(0, 0, 0, 0);
        lds_barrier();
        load_w(wr, k0 + 2 * PJ_KT);
        load_u(ur, k0 + PJ_UD * PJ_KT);
        if (active) {
#pragma unroll
            for (int s4 = 0; s4 < PJ_KT / 16; ++s4) {
                uint4 a[2], b[2];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    a[q] = *reinterpret_cast<const uint4 *>(aop[q] + 16 * s4);
                    b[q] = *reinterpret_cast<const uint4 *>(bop[q] + 16 * s4);
                }
#pragma unroll
                for (int ct = 0; ct < 2; ++ct)
#pragma unroll
                    for (int rt = 0; rt < 2; ++rt)
                        acc[ct][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                            __builtin_bit_cast(pj_bf16x8_t, a[ct]), __builtin_bit_cast(pj_bf16x8_t, b[rt]),
                            acc[ct][rt], 0, 0, 0);
            }
        }
    };
    // prologue in the order the loop consumes (scheduling barriers keep the issue order)
#pragma unroll
    for (int d = 0; d < PJ_UD; ++d) {
        if (d < 2) load_w(wreg[d], d * PJ_KT);
        load_u(ureg[d], d * PJ_KT);
        __builtin_amdgcn_sched_barrier(0);
    }
    // straight-line groups of PJ_UD stages (a stage count that is not a multiple runs all-zero
    // stages): no branch between the register sets
    for (int k0 = 0; k0 < Dm; k0 += PJ_UD * PJ_KT) {
#pragma unroll
        for (int d = 0; d < PJ_UD; ++d) stage(wreg[d & 1], ureg[d], k0 + d * PJ_KT);
    }
    if (!active) return;
    const bool isB = col0 < GN;
    const int cc = isB ? col0 : col0 - GN;                   // column inside the B (or C) row
    uint16_t *out = isB ? Be : Ce;
#pragma unroll
    for (int rt = 0; rt < 2; ++rt) {
        if (32 * rt + l32 < nvalid) {
            const int64_t ent = lst[32 * rt + l32];                       // t*K + r
            const int64_t row = compact ? ent : (ent / K) * E + e;
#pragma unroll
            for (int ct = 0; ct < 2; ++ct) {
                uint16_t *dst = out + row * GN + cc + 32 * ct + 16 * kg;
                const pj_f32x16_t v = acc[ct][rt];
                *reinterpret_cast<uint4 *>(dst) =
                    make_uint4(pj_pack(v[0], v[1]), pj_pack(v[2], v[3]), pj_pack(v[4], v[5]), pj_pack(v[6], v[7]));
                *reinterpret_cast<uint4 *>(dst + 8) =
                    make_uint4(pj_pack(v[8], v[9]), pj_pack(v[10], v[11]), pj_pack(v[12], v[13]), pj_pack(v[14], v[15]));
            }
        }
    }
}

// any shape, fp32 arithmetic: block = (token, slot), the token's features in LDS, one lane
// per output column of [B | C]
template <typename T>
__global__ void __launch_bounds__(256)
proj_generic_kernel(const T *__restrict__ u, const T *__restrict__ WB, const T *__restrict__ WC,
                    const int32_t *__restrict__ idx, T *__restrict__ Be, T *__restrict__ Ce, int E, int K,
                    int GN, int Dm, int compact)
{
    extern __shared__ float s_u[];
    const int64_t t = blockIdx.x / K;
    const int e = idx[blockIdx.x];
    const int64_t row = compact ? (int64_t)blockIdx.x : t * E + e;
    for (int d = threadIdx.x; d < Dm; d += 256) s_u[d] = to_float(u[t * Dm + d]);
    __syncthreads();
    for (int c = threadIdx.x; c < 2 * GN; c += 256) {
        const bool isB = c < GN;
        const int cc = isB ? c : c - GN;
        const T *wr = (isB ? WB : WC) + ((int64_t)e * GN + cc) * Dm;
        float acc = 0.f;
        for (int d = 0; d < Dm; ++d) acc += to_float(wr[d]) * s_u[d];
        (isB ? Be : Ce)[row * GN + cc] = from_float<T>(acc);
    }
}

swimba_status launch_expert_proj(int64_t tokens, int E, int K, int GN, int Dm, int io_dtype, const void *u,
                                 const void *WB, const void *WC, const void *logits, void *Be, void *Ce,
                                 int32_t *idx, float *w, int32_t *counts, int32_t *lists, int compact,
                                 hipStream_t st)
{
    if (tokens == 0) return SWIMBA_OK;
    if (tokens * K > 0x7fffffffll) return SWIMBA_ERR_UNSUPPORTED;   // list entries are 32-bit
    const bool mfma = io_dtype == SWIMBA_BF16 && Dm % 16 == 0 && GN % 64 == 0;
    const unsigned rgrid = (unsigned)((tokens + 255) / 256);
    if (!mfma) {
        swimba_status rs = launch_router(tokens, E, K, io_dtype, logits, idx, w, st);
        if (rs != SWIMBA_OK) return rs;
        const size_t shm = (size_t)Dm * sizeof(float);
        if (io_dtype == SWIMBA_BF16)
            hipLaunchKernelGGL(proj_generic_kernel<bf16>, dim3((unsigned)(tokens * K)), dim3(256), shm, st,
                               (const bf16 *)u, (const bf16 *)WB, (const bf16 *)WC, idx, (bf16 *)Be, (bf16 *)Ce, E,
                               K, GN, Dm, compact);
        else
            hipLaunchKernelGGL(proj_generic_kernel<float>, dim3((unsigned)(tokens * K)), dim3(256), shm, st,
                               (const float *)u, (const float *)WB, (const float *)WC, idx, (float *)Be,
                               (float *)Ce, E, K, GN, Dm, compact);
        SWIMBA_CHECK_LAUNCH();
        return SWIMBA_OK;
    }
    hipLaunchKernelGGL(proj_clear_kernel, dim3(1), dim3(256), 0, st, counts, E);
    SWIMBA_CHECK_LAUNCH();
    hipLaunchKernelGGL(proj_route_kernel<bf16>, dim3(rgrid), dim3(256), (size_t)256 * K * sizeof(int32_t), st,
                       (const bf16 *)logits, idx, w, counts, lists, tokens, E, K);
    SWIMBA_CHECK_LAUNCH();
    const int tiles_max = (int)((tokens + PJ_TOK - 1) / PJ_TOK);
    const dim3 grid((unsigned)((int64_t)8 * ((E + 7) / 8) * tiles_max), (unsigned)((2 * GN + PJ_COLS - 1) / PJ_COLS));
    hipLaunchKernelGGL(proj_mfma_kernel, grid, dim3(256), 0, st, (const uint16_t *)u, (const uint16_t *)WB,
                       (const uint16_t *)WC, counts, lists, (uint16_t *)Be, (uint16_t *)Ce, tokens, E, K, GN, Dm,
                       tiles_max, compact);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

// idx[t*K + r] = r: with streams stored per selected slot, slot r is "expert" r
__global__ void slot_ids_kernel(int32_t *idx, int64_t n, int K)
{
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) idx[i] = (int32_t)(i % K);
}

swimba_status launch_slot_ids(int32_t *idx, int64_t tokens, int K, hipStream_t st)
{
    const int64_t n = tokens * K;
    if (n == 0) return SWIMBA_OK;
    hipLaunchKernelGGL(slot_ids_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, idx, n, K);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

}  // namespace swimba
