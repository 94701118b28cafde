// Router + expert mixing + G^T tiles of a whole chunk in one persistent kernel, for the single-pass
// forward on shapes with many (batch, chunk, group) triples (paper, Theorem 1: the mixed streams
// Bmix_t = sum_{e in K_t} pi_{t,e} B_t^(e), Cmix likewise, feed one plain SSM; SSD background: the
// intra-chunk work is the masked product of Cmix Bmix^T with x).
//
// mix_rows_kernel works on 32 tokens and has to write the mixed B rows twice (as MFMA operand
// registers for the tile products, and token-innermost for the state build) because the tiles
// G^T = Bmix . Cmix^T of a chunk need the rows of other 32-token tiles.  Here a workgroup owns all
// Q tokens of one (batch, chunk, group): the mixed rows stay in LDS, from where they leave as
//   cmix    (B, nc, G, NT, 8, 64, 8)  mixed C rows as operand registers (as mix_rows_kernel writes them)
//   bmix_t8 (B, nc, G, Q/8, N, 8)     mixed B rows, tokens innermost in the order of t8_token
//   cb      (B, nc, G, NP, 2, 64, 8)  the causal 32 x 32 tiles of Bmix . Cmix^T (as cb_pair writes them)
// and the operand-register image of the mixed B rows is never written or read back: 200 MB less
// traffic and no tile pass on the long-sequence workload.
//
// The workgroups are persistent (one per compute unit, 152 KB of LDS) and walk their items with
// the expert rows of the next item already requested: the routing runs two items ahead, and as
// soon as the B rows (then the C rows) of item i have been mixed out of their registers the
// gather of item i + 1 refills them, so loads are in flight while the tiles of item i are computed
// and stored (up to two experts per token; a lane owns one 16-byte piece of eight token rows, 16
// lanes read one whole 256-byte expert row).
#include "common.hpp"
#include "mfma_util.hpp"

#include <atomic>

namespace swimba {

constexpr int MC_THREADS = 512;
constexpr int MC_ROW = MN + 8;       // LDS row stride of the mixed rows (elements)
constexpr int MC_EMAX = 16;          // experts the in-register routing takes
constexpr int MC_KMAX = 2;           // active experts per token the gather registers take

// route_token with the logits in registers: the same comparisons and the same arithmetic in the same
// order, every loop unrolled over MC_EMAX slots so that no index is dynamic
__device__ __forceinline__ void route_token_regs(const float (&v)[MC_EMAX], int E, int K, int32_t *idx, float *w)
{
    float m = -INFINITY;
#pragma unroll
    for (int e = 0; e < MC_EMAX; ++e)
        if (e < E) m = fmaxf(m, v[e]);
    float Z = 0.f;
#pragma unroll
    for (int e = 0; e < MC_EMAX; ++e)
        if (e < E) Z += route_exp(v[e] - m);
    const float invZ = 1.0f / Z;
    float pv = 0.f;
    int pi = -1;
#pragma unroll
    for (int r = 0; r < MC_KMAX; ++r) {
        if (r < K) {
            int best = -1;
            float bv = 0.f;
#pragma unroll
            for (int e = 0; e < MC_EMAX; ++e) {
                const bool after = (r == 0) || (v[e] < pv) || (v[e] == pv && e > pi);
                if (e < E && after && (best < 0 || v[e] > bv)) { best = e; bv = v[e]; }
            }
            if (best < 0) { best = (pi + 1) % E; bv = -INFINITY; }   // logits outside the contract: a valid index
            idx[r] = best;
            w[r] = route_exp(bv - m) * invZ;
            pv = bv;
            pi = best;
        }
    }
}

// 8 x 8 transpose of 16-bit values: in[r] holds 8 values of row r, out[c] the 8 values of column c
__device__ __forceinline__ void transpose8x8_b16(const uint4 (&in)[8], uint4 (&out)[8])
{
    // 2 x 2 blocks of 16-bit values inside pairs of rows, then 32-bit and 64-bit moves
    uint32_t a[8][4];
#pragma unroll
    for (int r = 0; r < 8; r += 2) {
        const uint32_t x[4] = {in[r].x, in[r].y, in[r].z, in[r].w}, y[4] = {in[r + 1].x, in[r + 1].y, in[r + 1].z, in[r + 1].w};
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            a[r][q] = __builtin_amdgcn_perm(y[q], x[q], 0x05040100u);       // (x.lo, y.lo): column 2q, rows r, r+1
            a[r + 1][q] = __builtin_amdgcn_perm(y[q], x[q], 0x07060302u);   // (x.hi, y.hi): column 2q+1
        }
    }
    // a[r][q] (r even) = column 2q, rows r, r+1;  a[r+1][q] = column 2q+1, rows r, r+1
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        out[2 * q] = make_uint4(a[0][q], a[2][q], a[4][q], a[6][q]);
        out[2 * q + 1] = make_uint4(a[1][q], a[3][q], a[5][q], a[7][q]);
    }
}

// Lane (slot, piece): the 16-byte piece `piece` (8 state indices) of the eight tokens of octet `slot`
// in the order of t8_token, so that after the mix the lane holds an 8 x 8 block that goes out,
// transposed in registers, as eight consecutive 16-byte pieces of the token-innermost image.
template <int Q>
__global__ void __launch_bounds__(MC_THREADS, 2)
mix_chunk_kernel(const uint16_t *__restrict__ Be, const uint16_t *__restrict__ Ce,
                 const uint16_t *__restrict__ logits, int32_t *__restrict__ idx_out, float *__restrict__ w_out,
                 uint16_t *__restrict__ cmix, uint16_t *__restrict__ bmix_t8, uint16_t *__restrict__ cb, Shape s,
                 int nbcg, const float *__restrict__ w_sel)
{
    constexpr int NT = Q / 32, NP = NT * (NT + 1) / 2;
    constexpr int NOCT = Q / 8;                           // token octets of a chunk (at most 32 = the row slots)
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint16_t *s_B = reinterpret_cast<uint16_t *>(smem_raw);        // [Q][MC_ROW] mixed B rows
    uint16_t *s_C = s_B + Q * MC_ROW;                              // [Q][MC_ROW] mixed C rows
    int32_t *s_idx = reinterpret_cast<int32_t *>(s_C + Q * MC_ROW);    // [3][Q][MC_KMAX]
    float *s_w = reinterpret_cast<float *>(s_idx + 3 * Q * MC_KMAX);   // [3][Q][MC_KMAX]

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int K = s.K;
    const bool sel = (w_sel != nullptr);
    const int rowsE = sel ? K : s.E;                     // rows per token in Be / Ce
    const int estride = s.G * s.N;
    const int tokstride = rowsE * estride;
    const int piece = tid & 15;
    const int slot = min(tid >> 4, NOCT - 1);            // lanes past the last octet repeat it and store nothing
    const bool owner = (tid >> 4) < NOCT;
    const bool pin = piece * 8 < s.N;                    // pieces past the caller's N stay zero (padding)
    const int pc = pin ? piece : 0;

    // routing of item `it` into table `buf` (threads 0 .. Q-1, one token each)
    auto route = [&](int it, int buf) __attribute__((always_inline)) {
        if (tid < Q) {
            const int g = it % s.G, c = (it / s.G) % s.nc, b = it / (s.G * s.nc);
            const int valid = min(Q, s.L - c * Q);
            const int64_t tok = (int64_t)b * s.L + (int64_t)c * Q + min(tid, valid - 1);
            int32_t id[MC_KMAX] = {0, 0};
            float ww[MC_KMAX] = {0.f, 0.f};
            if (sel) {
#pragma unroll
                for (int r = 0; r < MC_KMAX; ++r)
                    if (r < K) { id[r] = r; ww[r] = w_sel[tok * K + r]; }
            } else {
                const uint16_t *gl = logits + tok * s.E;
                // all loads first, conversions after (a value consumed where it is loaded is waited for on
                // the spot); a row of 16 logits is two 16-byte loads
                float v[MC_EMAX];
                if (s.E == MC_EMAX && (reinterpret_cast<uintptr_t>(logits) & 15u) == 0) {   // (the interface asks for element alignment only)
                    const uint4 q0 = *reinterpret_cast<const uint4 *>(gl), q1 = *reinterpret_cast<const uint4 *>(gl + 8);
                    unpack8(v, q0);
                    unpack8(v + 8, q1);
                } else {
                    uint16_t raw[MC_EMAX];
#pragma unroll
                    for (int e = 0; e < MC_EMAX; ++e) raw[e] = gl[min(e, s.E - 1)];
#pragma unroll
                    for (int e = 0; e < MC_EMAX; ++e) v[e] = to_float(bf16{raw[e]});
                }
                route_token_regs(v, s.E, K, id, ww);
                if (g == 0 && tid < valid) {
#pragma unroll
                    for (int r = 0; r < MC_KMAX; ++r)
                        if (r < K) { idx_out[tok * K + r] = id[r]; w_out[tok * K + r] = ww[r]; }
                }
            }
            const bool on = tid < valid;                 // rows past the end of the sequence mix to zero
#pragma unroll
            for (int r = 0; r < MC_KMAX; ++r) {
                s_idx[(buf * Q + tid) * MC_KMAX + r] = (r < K) ? id[r] : id[0];
                s_w[(buf * Q + tid) * MC_KMAX + r] = (on && r < K) ? ww[r] : 0.f;
            }
        }
    };

    // expert rows of one stream of item `it`, all loads unconditional
    uint4 vb[8][MC_KMAX], vc[8][MC_KMAX];
    auto gather = [&](uint4 (&v)[8][MC_KMAX], const uint16_t *Se, int it, int buf, int slot) __attribute__((always_inline)) {
        const int g = it % s.G, c = (it / s.G) % s.nc, b = it / (s.G * s.nc);
        const int valid = min(Q, s.L - c * Q);
        const int64_t tok0 = (int64_t)b * s.L + (int64_t)c * Q;
        const uint16_t *Sg = Se + (tok0 * rowsE * s.G + g) * s.N + pc * 8;
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int j = t8_token(8 * slot + p);
            const int64_t rowoff = (int64_t)min(j, valid - 1) * tokstride;
#pragma unroll
            for (int r = 0; r < MC_KMAX; ++r)
                v[p][r] = *reinterpret_cast<const uint4 *>(Sg + rowoff + s_idx[(buf * Q + j) * MC_KMAX + r] * estride);
        }
    };
    // the gathered rows of one stream, weighted and summed in fp32, as bf16: into LDS, and kept in `rows`
    auto mix = [&](const uint4 (&v)[8][MC_KMAX], uint16_t *s_S, int buf, uint4 *rows, int slot) __attribute__((always_inline)) {
#pragma unroll
        for (int p = 0; p < 8; ++p) {
            const int j = t8_token(8 * slot + p);
            float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int r = 0; r < MC_KMAX; ++r) fma_bf16x8(a, v[p][r], pin ? s_w[(buf * Q + j) * MC_KMAX + r] : 0.f);
            const uint4 row = pack8(a);
            if (rows) rows[p] = row;
            if (owner) *reinterpret_cast<uint4 *>(s_S + j * MC_ROW + piece * 8) = row;
        }
    };

    const int step = gridDim.x;
    int it = blockIdx.x;
    if (it >= nbcg) return;
    // routing runs two items ahead of the mix, the gathers one item ahead
    route(it, 0);
    if (it + step < nbcg) route(it + step, 1);
    lds_barrier();
    gather(vb, Be, it, 0, slot);
    gather(vc, Ce, it, 0, slot);
    for (int n = 0; it < nbcg; it += step, ++n) {
        const int buf = n % 3, buf1 = (n + 1) % 3, buf2 = (n + 2) % 3;
        const int nxt = it + step;
        const bool more = nxt < nbcg;                      // workgroup-uniform
        const int64_t bcg = it;                            // items are (batch, chunk, group) in layout order
        // The lane's octet goes through an opaque copy once per item: the row offsets, LDS addresses and
        // token indices derived from it are rebuilt where they are used instead of staying in registers
        // for the whole loop (they would push the gathered rows into scratch memory).
        int sl = slot;
        asm volatile("" : "+v"(sl));
        {
            // ---- mixed B rows; 8 tokens innermost, the lane's 8 x 8 block, transposed, is 128 contiguous bytes ----
            uint4 rows[8], cols[8];
            mix(vb, s_B, buf, rows, sl);
            transpose8x8_b16(rows, cols);
            if (owner) {
                uint16_t *dst = bmix_t8 + ((bcg * NOCT + sl) * MN + piece * 8) * 8;
#pragma unroll
                for (int q = 0; q < 8; ++q) *reinterpret_cast<uint4 *>(dst + q * 8) = cols[q];
            }
        }
        mix(vc, s_C, buf, nullptr, sl);
        if (nxt + step < nbcg) route(nxt + step, buf2);
        // The rows of the next item: in flight until it is mixed.  Nothing below may wait on memory
        // (memory operations retire in order: a wait on anything younger would wait for these too).
        if (more) {
            gather(vb, Be, nxt, buf1, sl);
            gather(vc, Ce, nxt, buf1, sl);
        }
        lds_barrier();
        int ln = lane;                                      // opaque like the octet above
        asm volatile("" : "+v"(ln));
        const int l32 = ln & 31, kg = ln >> 5;

        // ---- mixed C rows as operand registers: lane (l32, kg) holds n = 64 kg + 8 ks .. + 7 of token l32 ----
        if (wave < NT) {
            const uint16_t *src = s_C + (32 * wave + l32) * MC_ROW + 64 * kg;
            uint16_t *dst = cmix + (((bcg * NT + wave) * 8) * 64 + ln) * 8;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                *reinterpret_cast<uint4 *>(dst + ks * 64 * 8) = *reinterpret_cast<const uint4 *>(src + ks * 8);
        }
        // ---- G^T tiles: pair p = I(I+1)/2 + J, G^T[j][i] = Bmix_j . Cmix_i, both operands from LDS ----
        for (int p = wave; p < NP; p += MC_THREADS / 64) {
            int I = 0;
            while ((I + 1) * (I + 2) / 2 <= p) ++I;
            const int J = p - I * (I + 1) / 2;
            const uint16_t *bs = s_B + (32 * J + l32) * MC_ROW + 64 * kg;
            const uint16_t *cs = s_C + (32 * I + l32) * MC_ROW + 64 * kg;
            f32x16_t acc = {0};
#pragma unroll
            for (int half = 0; half < 2; ++half) {       // operands in two halves: the gathered rows hold most registers
                uint4 bf[4], cf[4];
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) {
                    bf[ks] = *reinterpret_cast<const uint4 *>(bs + (4 * half + ks) * 8);
                    cf[ks] = *reinterpret_cast<const uint4 *>(cs + (4 * half + ks) * 8);
                }
#pragma unroll
                for (int ks = 0; ks < 4; ++ks) acc = mfma32(bf[ks], cf[ks], acc);
            }
            float m[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) m[v] = acc[v];
            uint16_t *dst = cb + ((bcg * NP + p) * 2 * 64 + ln) * 8;
            *reinterpret_cast<uint4 *>(dst) = pack8(m);
            *reinterpret_cast<uint4 *>(dst + 64 * 8) = pack8(m + 8);
        }
        lds_barrier();                                      // the mixed rows are free for the next item
    }
}

// true when the chunk-level kernel takes this problem (the caller has checked the MFMA shape); with
// routing inside it needs the logits of a token in registers
bool mix_chunk_covers(const Shape &s, bool selected)
{
    const int64_t nbcg = (int64_t)s.B * s.nc * s.G;
    return (selected || s.E <= MC_EMAX) && s.K <= MC_KMAX && nbcg < ((int64_t)1 << 31);
}

template <int Q>
static swimba_status launch_mc_q(const Shape &s, const void *Be, const void *Ce, const void *logits, int32_t *idx,
                                 float *w, void *cmix, void *bmix_t8, void *cb, const float *w_sel, int ncu,
                                 hipStream_t st)
{
    const int64_t nbcg = (int64_t)s.B * s.nc * s.G;
    if (nbcg == 0) return SWIMBA_OK;
    const size_t shm = (size_t)2 * Q * MC_ROW * 2 + (size_t)3 * Q * MC_KMAX * 8;
    // more than 64 KB of dynamic LDS has to be allowed once per device
    static std::atomic<uint64_t> attr_set{0};            // one bit per device ordinal
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
    const uint64_t bit = 1ull << (dev & 63);
    if (!(attr_set.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute((const void *)mix_chunk_kernel<Q>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                (int)shm);
        if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
        attr_set.fetch_or(bit, std::memory_order_release);
    }
    const unsigned grid = (unsigned)(nbcg < ncu ? nbcg : ncu);
    hipLaunchKernelGGL(mix_chunk_kernel<Q>, dim3(grid), dim3(MC_THREADS), shm, st, (const uint16_t *)Be,
                       (const uint16_t *)Ce, (const uint16_t *)logits, idx, w, (uint16_t *)cmix, (uint16_t *)bmix_t8,
                       (uint16_t *)cb, s, (int)nbcg, w_sel);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

// logits / idx / w: routing inside (w_sel == nullptr); w_sel: rows of the selected experts with given weights
swimba_status launch_mix_chunk_mfma(const Shape &s, const void *Be, const void *Ce, const void *logits, int32_t *idx,
                                    float *w, void *cmix, void *bmix_t8, void *cb, const float *w_sel, int ncu,
                                    hipStream_t st)
{
    if (!mix_chunk_covers(s, w_sel != nullptr) || ncu < 1) return SWIMBA_ERR_UNSUPPORTED;
    switch (s.Q) {
    case 64: return launch_mc_q<64>(s, Be, Ce, logits, idx, w, cmix, bmix_t8, cb, w_sel, ncu, st);
    case 128: return launch_mc_q<128>(s, Be, Ce, logits, idx, w, cmix, bmix_t8, cb, w_sel, ncu, st);
    case 256: return launch_mc_q<256>(s, Be, Ce, logits, idx, w, cmix, bmix_t8, cb, w_sel, ncu, st);
    }
    return SWIMBA_ERR_UNSUPPORTED;
}

}  // namespace swimba
