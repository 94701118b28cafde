// Routed expert in-projection (paper, MoE-parameterized SSM: the expert streams are
// expert-specific linear projections of the same token features, and only the experts of the
// active set K_t enter the mix): for every token t and every e in K_t
//   B_t^(e)[c] = sum_d W_B[e][c][d] u_t[d],   C_t^(e)[c] = sum_d W_C[e][c][d] u_t[d],
// written either into the dense (B,L,E,G,N) layout (rows of inactive experts are not touched:
// the mixer never reads them) or, with `compact`, into (B,L,k,G,N): row r of a token is the
// stream of its r-th selected expert, so no buffer with an expert axis exists at all.
// The experts' input streams X^(e) (the mixed state update in its full form injects
// sum_e pi_e x^(e) (x) B^(e)) are a third block of output columns of the same product,
//   x_t^(e)[c] = sum_d W_X[e][c][d] u_t[d],  c over (head, channel),
// written the same way into (B,L,E,H,P) or (B,L,k,H,P).
//
// Three launches: clear the per-expert counters; route every token and append the entry
// t*k + r to the list of its r-th expert (LDS counters per block, one global atomic per block
// and expert); a grouped GEMM over (share of an expert's list, 256 output columns).
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

constexpr int PJ_COLS = 256;   // output columns per workgroup: 4 column groups of 64

// The output columns of the product are the concatenation [B | C | X] of up to three blocks, each
// with its own weight tensor (E, n, Dm) and its own output tensor (rows of n columns).
struct ProjBlocks {
    const void *W[3];
    void *out[3];
    int n[3];       // columns of the block (0: absent); multiples of 64 on the MFMA path
    int tot;        // n[0] + n[1] + n[2]
};
// block of column c and the column inside it
__device__ __forceinline__ int proj_block_of(const ProjBlocks &pb, int c, int &local)
{
    const int s = (c >= pb.n[0]) + (c >= pb.n[0] + pb.n[1]);
    local = c - (s > 0 ? pb.n[0] : 0) - (s > 1 ? pb.n[1] : 0);
    return s;
}

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

// Workgroup = (share of one expert's list, block of 256 output columns), 8 waves: wave w owns
// columns 64 (w & 3) .. + 63 of the block and one of two row groups.  The `nslots` workgroups
// that fit on the chip at once (one per compute unit) are divided among the experts in
// proportion to their list lengths (known on the device only), and a workgroup walks its share
// in passes of up to 192 entries (6 row tiles of 32, at most 3 per row group): the whole launch
// is one round of co-resident workgroups, whatever the routing.  (With fixed 64-entry tiles and
// two workgroups per compute unit the 130M-shaped layer had 517 workgroups for 512 places, and
// the second round of five cost 12 us; every workgroup also streamed the weights for 64 entries
// only.)  Measured on that layer (29 us): everything but the k-steps 8.5 us, MFMAs alone + 10 us,
// operand reads from LDS alone + 14 us (about 60 bytes per clock and compute unit, no bank
// conflicts), both + 22 us: the operand reads are the limit.  One wave per SIMD with 4 x 3 tiles
// (7 reads per 12 MFMAs instead of 5 per 6) measured slower (34 us): nothing hides its waits.
// The contraction runs in stages of 64 features.  A stage of both operands (256 weight rows,
// 192 token rows, 128 bytes each) is read with fully coalesced 16-byte loads (8 lanes per
// row), parked in registers while the previous stage is multiplied, and then passed through
// LDS, from where the lanes read their operand registers.
constexpr int PJ_THREADS = 512;
constexpr int PJ_KT = 64;             // features per stage
constexpr int PJ_STR = PJ_KT + 8;     // LDS row stride (elements): rows stay 16-byte aligned
constexpr int PJ_UD = 2;              // stages the loads run ahead (even)
constexpr int PJ_RT = 3;              // row tiles (of 32 list entries) per wave and pass
constexpr int PJ_ROWS = 2 * 32 * PJ_RT;   // list entries per workgroup and pass

// workgroups expert e gets out of nslots, given its list length
__device__ __forceinline__ int proj_share(int cnt, int nslots, int64_t total)
{
    return cnt > 0 ? max(1, (int)((int64_t)nslots * cnt / total)) : 0;
}

__global__ void __launch_bounds__(PJ_THREADS) __attribute__((amdgpu_waves_per_eu(2, 2)))
proj_mfma_kernel(const uint16_t *__restrict__ u, ProjBlocks pb, const int32_t *__restrict__ counts,
                 const int32_t *__restrict__ lists, int64_t tokens, int E, int K, int Dm, int nslots,
                 int compact)
{
    __shared__ __align__(16) uint16_t sW[PJ_COLS * PJ_STR];
    __shared__ __align__(16) uint16_t sU[PJ_ROWS * PJ_STR];
    __shared__ int32_t s_share[SWIMBA_MAX_EXPERTS];
    __shared__ int32_t s_sel[2];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t total = tokens * K;

    // ---- which expert, which part of its list: prefix sum of the shares (E <= 256 = 4 per lane) ----
    if (tid < SWIMBA_MAX_EXPERTS) s_share[tid] = tid < E ? proj_share(counts[tid], nslots, total) : 0;
    if (tid == 0) s_sel[0] = -1;
    __syncthreads();
    if (wave == 0) {
        int v[4], sum = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) { v[q] = s_share[4 * lane + q]; sum += v[q]; }
        int incl = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const int t = __shfl_up(incl, d);
            if (lane >= d) incl += t;
        }
        int r = (int)blockIdx.x - (incl - sum);
        if (r >= 0 && r < sum) {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                if (r >= 0 && r < v[q]) { s_sel[0] = 4 * lane + q; s_sel[1] = r; }
                r -= v[q];          // negative from the match on: no later q matches
            }
        }
    }
    __syncthreads();
    const int e = __builtin_amdgcn_readfirstlane(s_sel[0]);
    if (e < 0) return;                                       // whole workgroup: no barrier is skipped
    const int part = __builtin_amdgcn_readfirstlane(s_sel[1]);
    const int cnt = counts[e];
    const int nparts = proj_share(cnt, nslots, total);
    const int n32 = (cnt + 31) / 32;
    const int t_begin = (int)((int64_t)part * n32 / nparts), t_end = (int)((int64_t)(part + 1) * n32 / nparts);
    const int nt = t_end - t_begin;
    if (nt <= 0) return;
    const int npass = (nt + 2 * PJ_RT - 1) / (2 * PJ_RT);

    const int cw = wave & 3, rg = wave >> 2;                 // column group, row group of the wave
    const int colblk = blockIdx.y * PJ_COLS;                 // first column of the workgroup in [B | C | X]
    const int col0 = colblk + cw * 64;
    const bool active = col0 < pb.tot;                       // wave-uniform; idle waves still stage
    const int l32 = lane & 31, kg = lane >> 5;

    // ---- staging map: lane -> 16-byte piece `piece` of rows row0 + 64 i ----
    const int piece = tid & 7, row0 = tid >> 3;              // row0 = 32 rg + (row inside a 32-block)
    // Every block has a multiple of 32 columns, so the 32 rows of a staging step of one wave lie in
    // one weight tensor: a uniform base (scalar registers) + one per-lane offset for all four.
    const uint16_t *wbase[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        int cl;
        const int sb = proj_block_of(pb, min(colblk + 64 * i + 32 * rg, pb.tot - 32), cl);   // past the end: the last rows again
        wbase[i] = (const uint16_t *)pb.W[sb] + ((int64_t)e * pb.n[sb] + cl) * Dm;
    }
    const int r32 = row0 & 31;
    const int wlane = r32 * Dm;
    const int k_last = ((Dm - 1) / PJ_KT) * PJ_KT;
    // Operand row r of a 32-column weight tile must hold column 16*((r>>2)&1) + 4*(r>>3) + (r&3)
    // for accumulator register v of lane (l32, kg) to be column 16 kg + v of the tile.  The
    // permutation is applied when the rows are staged (column x goes to LDS row wrow), so the
    // lanes of a wave read consecutive LDS rows: no bank conflicts.
    const int wrow = 8 * ((r32 >> 2) & 3) + 4 * ((r32 >> 4) & 1) + (r32 & 3) + 32 * rg;
    const uint16_t *aop[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) aop[q] = sW + (cw * 64 + 32 * q + l32) * PJ_STR + 8 * kg;
    int cc;                                                  // column inside the row of the wave's block
    const int ob = proj_block_of(pb, min(col0, pb.tot - 64), cc);
    uint16_t *out = (uint16_t *)pb.out[ob];
    const int ncol = pb.n[ob];                               // row length of that output

    for (int pass = 0; pass < npass; ++pass) {
        const int p_begin = t_begin + (int)((int64_t)pass * nt / npass);
        const int p_end = t_begin + (int)((int64_t)(pass + 1) * nt / npass);
        const int ptiles = p_end - p_begin;                              // 1..6 row tiles
        const int half = (ptiles + 1) / 2;
        const int tbase = rg ? half : 0;                                 // first tile of this wave's row group
        const int nrt = rg ? ptiles - half : half;                       // its tiles: 0..3, wave-uniform
        const int nvalid = min(32 * p_end, cnt) - 32 * p_begin;          // entries of this pass
        const int32_t *lst = lists + (int64_t)e * tokens + 32 * p_begin;
        const uint16_t *usrc[PJ_RT];
#pragma unroll
        for (int i = 0; i < PJ_RT; ++i) usrc[i] = u + (int64_t)(lst[min(row0 + 64 * i, nvalid - 1)] / K) * Dm;
        const uint16_t *bop = sU + (32 * tbase + l32) * PJ_STR + 8 * kg;
        // Register sets: the weight rows (L2 hits) and the token rows (scattered 128-byte reads
        // that mostly come from HBM) of stage i + 2 are requested while stage i is multiplied.
        // All loads are clamped and unconditional, so that the waits on them stay exact counts;
        // the issues past the last stage re-read it and are not used.
        uint4 wreg[2][4], ureg[PJ_UD][PJ_RT];
        auto load_w = [&](uint4 (&wr)[4], int k0) __attribute__((always_inline)) {
            const int kk = min(min(k0, k_last) + piece * 8, Dm - 8);   // a short last stage stays inside the row
#pragma unroll
            for (int i = 0; i < 4; ++i) wr[i] = *reinterpret_cast<const uint4 *>(wbase[i] + (wlane + kk));
        };
        auto load_u = [&](uint4 (&ur)[PJ_RT], int k0) __attribute__((always_inline)) {
            const int kk = min(min(k0, k_last) + piece * 8, Dm - 8);
#pragma unroll
            for (int i = 0; i < PJ_RT; ++i) ur[i] = *reinterpret_cast<const uint4 *>(usrc[i] + kk);
        };
        pj_f32x16_t acc[2][PJ_RT];
#pragma unroll
        for (int ct = 0; ct < 2; ++ct)
#pragma unroll
            for (int rt = 0; rt < PJ_RT; ++rt) acc[ct][rt] = pj_f32x16_t{0};

        // the 4 k-steps of a stage; the operands of k-step s + 1 are read from LDS before the
        // MFMAs of k-step s are issued (two operand sets rotated by name)
        auto read_ops = [&](uint4 (&a)[2], uint4 (&b)[PJ_RT], int s4) __attribute__((always_inline)) {
#pragma unroll
            for (int q = 0; q < 2; ++q) a[q] = *reinterpret_cast<const uint4 *>(aop[q] + 16 * s4);
#pragma unroll
            for (int rt = 0; rt < PJ_RT; ++rt)
                b[rt] = *reinterpret_cast<const uint4 *>(bop + 32 * rt * PJ_STR + 16 * s4);
        };
        auto mfmas = [&](const uint4 (&a)[2], const uint4 (&b)[PJ_RT]) __attribute__((always_inline)) {
#pragma unroll
            for (int rt = 0; rt < PJ_RT; ++rt)
#pragma unroll
                for (int ct = 0; ct < 2; ++ct)
                    acc[ct][rt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                        __builtin_bit_cast(pj_bf16x8_t, a[ct]), __builtin_bit_cast(pj_bf16x8_t, b[rt]),
                        acc[ct][rt], 0, 0, 0);
        };
        auto multiply = [&]() __attribute__((always_inline)) {
            uint4 a0[2], b0[PJ_RT], a1[2], b1[PJ_RT];
            read_ops(a0, b0, 0);
            read_ops(a1, b1, 1);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(a0, b0);
            __builtin_amdgcn_sched_barrier(0);
            read_ops(a0, b0, 2);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(a1, b1);
            __builtin_amdgcn_sched_barrier(0);
            read_ops(a1, b1, 3);
            __builtin_amdgcn_sched_barrier(0);
            mfmas(a0, b0);
            mfmas(a1, b1);
        };
        // one stage: registers -> LDS, refill the registers two stages ahead, multiply from LDS
        auto stage = [&](uint4 (&wr)[4], uint4 (&ur)[PJ_RT], int k0) __attribute__((always_inline)) {
            lds_barrier();                                       // every wave is done with the previous stage
            // pieces past the end of a short last stage are staged as zeros: every stage is 4 k-steps
            const bool inside = k0 + piece * 8 < Dm;
#pragma unroll
            for (int i = 0; i < 4; ++i)
                *reinterpret_cast<uint4 *>(sW + (wrow + 64 * i) * PJ_STR + piece * 8) =
                    inside ? wr[i] : make_uint4(0, 0, 0, 0);
#pragma unroll
            for (int i = 0; i < PJ_RT; ++i)
                *reinterpret_cast<uint4 *>(sU + (row0 + 64 * i) * PJ_STR + piece * 8) =
                    inside ? ur[i] : make_uint4(0, 0, 0, 0);
            lds_barrier();
            load_w(wr, k0 + 2 * PJ_KT);
            load_u(ur, k0 + PJ_UD * PJ_KT);
            // All three row tiles are multiplied whether the wave has that many or not (the rows are
            // staged clamped, the epilogue skips them): a branch per row tile inside the k-steps made
            // every pair of MFMAs wait for its own LDS read, and one code path per tile count spills.
            if (active) multiply();
        };
        // prologue in the order the loop consumes (scheduling barriers keep the issue order)
#pragma unroll
        for (int d = 0; d < PJ_UD; ++d) {
            load_w(wreg[d], d * PJ_KT);
            load_u(ureg[d], d * PJ_KT);
            __builtin_amdgcn_sched_barrier(0);
        }
        // straight-line groups of PJ_UD stages (a stage count that is not a multiple runs all-zero
        // stages): no branch between the register sets
        for (int k0 = 0; k0 < Dm; k0 += PJ_UD * PJ_KT) {
#pragma unroll
            for (int d = 0; d < PJ_UD; ++d) stage(wreg[d], ureg[d], k0 + d * PJ_KT);
        }
        if (active) {
#pragma unroll
            for (int rt = 0; rt < PJ_RT; ++rt) {
                const int prow = 32 * (tbase + rt) + l32;                         // entry inside the pass
                if (rt < nrt && prow < nvalid) {
                    const int64_t ent = lst[prow];                                // t*K + r
                    const int64_t row = compact ? ent : (ent / K) * E + e;
#pragma unroll
                    for (int ct = 0; ct < 2; ++ct) {
                        uint16_t *dst = out + row * ncol + cc + 32 * ct + 16 * kg;
                        const pj_f32x16_t v = acc[ct][rt];
                        *reinterpret_cast<uint4 *>(dst) =
                            make_uint4(pj_pack(v[0], v[1]), pj_pack(v[2], v[3]), pj_pack(v[4], v[5]), pj_pack(v[6], v[7]));
                        *reinterpret_cast<uint4 *>(dst + 8) = make_uint4(pj_pack(v[8], v[9]), pj_pack(v[10], v[11]),
                                                                         pj_pack(v[12], v[13]), pj_pack(v[14], v[15]));
                    }
                }
            }
        }
    }
}

// any shape, fp32 arithmetic: block = (token, slot), the token's features in LDS, one lane
// per output column of [B | C]
template <typename T>
__global__ void __launch_bounds__(256)
proj_generic_kernel(const T *__restrict__ u, ProjBlocks pb, const int32_t *__restrict__ idx, int E, int K,
                    int Dm, int compact)
{
    extern __shared__ float s_u[];
    const int64_t t = blockIdx.x / K;
    const int e = idx[blockIdx.x];
    const int64_t row = compact ? (int64_t)blockIdx.x : t * E + e;
    for (int d = threadIdx.x; d < Dm; d += 256) s_u[d] = to_float(u[t * Dm + d]);
    __syncthreads();
    for (int c = threadIdx.x; c < pb.tot; c += 256) {
        int cc;
        const int sb = proj_block_of(pb, c, cc);
        const T *wr = (const T *)pb.W[sb] + ((int64_t)e * pb.n[sb] + cc) * Dm;
        float acc = 0.f;
        for (int d = 0; d < Dm; ++d) acc += to_float(wr[d]) * s_u[d];
        ((T *)pb.out[sb])[row * pb.n[sb] + cc] = from_float<T>(acc);
    }
}

bool expert_proj_on_mfma(int io_dtype, int GN, int HP, int Dm)
{
    return io_dtype == SWIMBA_BF16 && Dm % 16 == 0 && GN % 64 == 0 && HP % 64 == 0;
}

// WX / Xo / HP: the third block of columns (input streams), nullptr / nullptr / 0 when not wanted
swimba_status launch_expert_proj(int64_t tokens, int E, int K, int GN, int Dm, int io_dtype, const void *u,
                                 const void *WB, const void *WC, const void *logits, void *Be, void *Ce,
                                 int32_t *idx, float *w, int32_t *counts, int32_t *lists, int compact,
                                 hipStream_t st, const void *WX, void *Xo, int HP)
{
    if (tokens == 0) return SWIMBA_OK;
    if (tokens * K > 0x7fffffffll) return SWIMBA_ERR_UNSUPPORTED;   // list entries are 32-bit
    ProjBlocks pb;
    pb.W[0] = WB; pb.W[1] = WC; pb.W[2] = WX;
    pb.out[0] = Be; pb.out[1] = Ce; pb.out[2] = Xo;
    pb.n[0] = GN; pb.n[1] = GN; pb.n[2] = WX ? HP : 0;
    pb.tot = 2 * GN + pb.n[2];
    const bool mfma = expert_proj_on_mfma(io_dtype, GN, pb.n[2], Dm);
    const unsigned rgrid = (unsigned)((tokens + 255) / 256);
    if (!mfma) {
        swimba_status rs = launch_router(tokens, E, K, io_dtype, logits, idx, w, st);
        if (rs != SWIMBA_OK) return rs;
        const size_t shm = (size_t)Dm * sizeof(float);
        if (io_dtype == SWIMBA_BF16)
            hipLaunchKernelGGL(proj_generic_kernel<bf16>, dim3((unsigned)(tokens * K)), dim3(256), shm, st,
                               (const bf16 *)u, pb, idx, E, K, Dm, compact);
        else
            hipLaunchKernelGGL(proj_generic_kernel<float>, dim3((unsigned)(tokens * K)), dim3(256), shm, st,
                               (const float *)u, pb, idx, E, K, Dm, compact);
        SWIMBA_CHECK_LAUNCH();
        return SWIMBA_OK;
    }
    hipLaunchKernelGGL(proj_clear_kernel, dim3(1), dim3(256), 0, st, counts, E);
    SWIMBA_CHECK_LAUNCH();
    hipLaunchKernelGGL(proj_route_kernel<bf16>, dim3(rgrid), dim3(256), (size_t)256 * K * sizeof(int32_t), st,
                       (const bf16 *)logits, idx, w, counts, lists, tokens, E, K);
    SWIMBA_CHECK_LAUNCH();
    // one place per compute unit (a workgroup is 8 waves with up to 256 registers each), shared
    // by the column blocks; the kernel divides them among the experts
    int devid = 0, ncu = 0;
    hipError_t he = hipGetDevice(&devid);
    if (he == hipSuccess) he = hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, devid);
    if (he != hipSuccess) { set_last_hip_error((int)he); return SWIMBA_ERR_HIP; }
    const int colblocks = (pb.tot + PJ_COLS - 1) / PJ_COLS;
    const int nslots = max(1, ncu / colblocks);
    const dim3 grid((unsigned)(nslots + E), (unsigned)colblocks);   // the shares sum to at most nslots + E
    hipLaunchKernelGGL(proj_mfma_kernel, grid, dim3(PJ_THREADS), 0, st, (const uint16_t *)u, pb, counts, lists,
                       tokens, E, K, Dm, nslots, compact);
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
