// Single-pass SSD forward on bf16 MFMA: chunk states never reach HBM and x is read once.
// (paper, background section on SSD: matrix multiplications inside chunks, a linear recurrence
// between chunks; complexity theorem: the cost that matters is evolving the state; per-channel
// independence of the recurrence makes the split over channels exact.)
//
//   prep   one launch in front of the pass: the causal 32x32 tiles of G^T = Bmix . Cmix^T per
//          (batch, chunk, group), and per (batch, chunk, head) the tables
//              cs2_j = log2(e) * (inclusive cumsum of dt*A inside the chunk)
//              f_j   = dt_j * exp(R_J - cs_j),  R_J = cs at the last token of j's 32-token tile
//              coef_j = dt_j * exp(cs_last - cs_j)
//   pass   workgroup = (batch, head, slice of 32 channels), 4 waves.  It walks the chunks of its
//          sequence in order with the slice's running state, 128 x 32 fp32, in MFMA
//          accumulators (wave w owns state rows n = 32w .. 32w+31).  Per chunk:
//            stage   x^T (pure transpose) and xs^T = (f x)^T into LDS, the state as bf16 into LDS
//            Y^T   = H_c . Cmix^T scaled by exp(cs_i)                            (wave: 2 token tiles)
//            Y^T  += sum_{J<I} exp(cs_i - R_J) * (xs^T_J . G^T_JI)                (tiles left of the diagonal)
//            Y^T  += x^T_I . (G^T_II * exp(cs_i - cs_j) dt_j [j <= i])           (diagonal tile)
//            y     = Y + D x, stored straight from the accumulators
//            H    <- exp(cs_last) H + sum_J exp(cs_last - R_J) * (Bmix_J^T . xs_J)   (wave: its 32 rows)
//
// Exponent safety: every exponential has a non-positive argument (cs is non-increasing), the
// decay is only ever formed from differences.  f_j underflows only where the true contribution
// of token j beyond its tile is below the fp32 range as well.  Left of the diagonal the tile of
// G^T goes into the MFMA exactly as stored; the per-token factor exp(cs_i - R_J) is a per-lane
// scalar applied to the 16 partial sums (rows of Y^T are channels, columns are tokens).
//
// All operands shared by the heads of a group (mixed rows, G^T tiles) are read from the images
// the mix kernel and prep wrote; block ids are mapped so that the workgroups of one (batch,
// group) run on one XCD and find them in its L2.
#include "common.hpp"
#include "mfma_util.hpp"

#include <atomic>

namespace swimba {

// =========================================================================================
// prep: blocks [0, ncb) compute the G^T tiles (two forms, see the launcher); the blocks behind
// them the cumsum tables, workgroup = (batch, chunk, block of 16 heads).
// =========================================================================================
template <int Q>
__global__ void __launch_bounds__(MTHREADS)
prep_kernel(const uint16_t *__restrict__ dt, const float *__restrict__ A, const uint16_t *__restrict__ cmix,
            const uint16_t *__restrict__ bfrag, uint16_t *__restrict__ cb, float *__restrict__ cs2,
            float *__restrict__ fdec, float *__restrict__ cdec, Shape s, int64_t nbcg, int64_t ncb, int fine)
{
    constexpr int NT = Q / 32;
    constexpr int NP = NT * (NT + 1) / 2;
    constexpr int HB = 16;                       // heads per workgroup
    constexpr int NSEG = MTHREADS / HB;          // segments a head's tokens are scanned in
    // one LDS area for both kinds of workgroup
    constexpr size_t LDS_CB = (size_t)NT * 8 * 64 * 16;                       // mixed B rows of the chunk
    constexpr size_t LDS_CUM = (size_t)(2 * Q * (HB + 1) + NSEG * HB) * sizeof(float);
    __shared__ __align__(16) unsigned char s_raw[LDS_CB > LDS_CUM ? LDS_CB : LDS_CUM];
    if (fine && (int64_t)blockIdx.x < ncb) {
        // ---- G^T tiles, one wave per tile pair (few (batch, chunk, group) triples: this form
        // ---- spreads them over the whole chip) ----
        constexpr int PB = (NP + 3) / 4;
        const int64_t id = xcd_logical_id(blockIdx.x, (int)ncb);
        const int64_t bcg = id / PB;
        const int p = (int)(id % PB) * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        if (bcg < nbcg && p < NP) cb_pair(cmix, bfrag, cb, NT, bcg, p, threadIdx.x & 63);
        return;
    }
    if (!fine && (int64_t)blockIdx.x < ncb) {
        // ---- G^T tiles of one (batch, chunk, group).  The mixed B rows of the whole chunk go
        // ---- through LDS once (they are the A operand of every pair of their column of tiles);
        // ---- with eight tiles wave w computes the rows of tiles w and 7-w: nine pairs for every wave.
        const int64_t bcg = blockIdx.x;
        const int tid = threadIdx.x, lane = tid & 63;
        const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
        uint4 *sB = reinterpret_cast<uint4 *>(s_raw);                                    // [NT][8][64]
        const uint4 *gB = reinterpret_cast<const uint4 *>(bfrag) + bcg * (NT * 8 * 64);
#pragma unroll
        for (int i = 0; i < NT * 8 * 64 / MTHREADS; ++i) sB[tid + i * MTHREADS] = gB[tid + i * MTHREADS];
        __syncthreads();
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const int I = t == 0 ? wave : NT - 1 - wave;
            if (I >= NT || (t == 1 && NT < 8)) continue;          // at most four tiles: one per wave
            uint4 cf[8];
            const uint16_t *cs = cmix + (((bcg * NT + I) * 8) * 64 + lane) * 8;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks) cf[ks] = *reinterpret_cast<const uint4 *>(cs + ks * 64 * 8);
            for (int J = 0; J <= I; ++J) {
                f32x16_t acc = {0};
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) acc = mfma32(sB[(J * 8 + ks) * 64 + lane], cf[ks], acc);
                float m[16];
#pragma unroll
                for (int v = 0; v < 16; ++v) m[v] = acc[v];
                uint16_t *dst = cb + ((bcg * NP + I * (I + 1) / 2 + J) * 2 * 64 + lane) * 8;
                *reinterpret_cast<uint4 *>(dst) = pack8(m);
                *reinterpret_cast<uint4 *>(dst + 64 * 8) = pack8(m + 8);
            }
        }
        return;
    }
    float (*s_a)[HB + 1] = reinterpret_cast<float (*)[HB + 1]>(s_raw);                   // dt*A, then its cumsum
    float (*s_d)[HB + 1] = reinterpret_cast<float (*)[HB + 1]>(s_raw) + Q;               // dt
    float (*s_tot)[HB] = reinterpret_cast<float (*)[HB]>(reinterpret_cast<float *>(s_raw) + 2 * Q * (HB + 1));
    const int nhb = (s.H + HB - 1) / HB;
    const int id = (int)((int64_t)blockIdx.x - ncb);
    const int hb = id % nhb;
    const int c = (id / nhb) % s.nc;
    const int b = id / (nhb * s.nc);
    const int tid = threadIdx.x;
    const int64_t tok0 = (int64_t)b * s.L + (int64_t)c * Q;
    const int valid = min(Q, s.L - c * Q);
    if (s.H % 8 == 0 && (reinterpret_cast<uintptr_t>(dt) & 15u) == 0) {
        // eight heads of a token per load (16 bytes; the rows are 2H bytes long, so every piece is aligned
        // when the tensor is: the interface asks for element alignment only)
        for (int i = tid; i < Q * (HB / 8); i += MTHREADS) {
            const int j = i / (HB / 8), h8 = (i % (HB / 8)) * 8, h = hb * HB + h8;
            uint4 raw = make_uint4(0u, 0u, 0u, 0u);
            const bool in = h < s.H && j < valid;
            if (in) raw = *reinterpret_cast<const uint4 *>(dt + (tok0 + j) * s.H + h);
            float dv[8];
            unpack8(dv, raw);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                s_a[j][h8 + e] = in ? dv[e] * A[h + e] : 0.f;
                s_d[j][h8 + e] = dv[e];
            }
        }
    } else {
        for (int i = tid; i < Q * HB; i += MTHREADS) {
            const int j = i / HB, hh = i % HB, h = hb * HB + hh;
            float dtv = 0.f, a = 0.f;
            if (h < s.H && j < valid) {
                dtv = to_float(bf16{dt[(tok0 + j) * s.H + h]});
                a = dtv * A[h];
            }
            s_a[j][hh] = a;
            s_d[j][hh] = dtv;
        }
    }
    __syncthreads();
    // the segments of a head are scanned by one lane each, then offset by the totals before them
    constexpr int SEG = Q / NSEG;
    const int hh = tid % HB, seg = tid / HB;
    {
        float run = 0.f;
        for (int j = seg * SEG; j < (seg + 1) * SEG; ++j) { run += s_a[j][hh]; s_a[j][hh] = run; }
        s_tot[seg][hh] = run;
    }
    __syncthreads();
    {
        float base = 0.f;
        for (int q = 0; q < seg; ++q) base += s_tot[q][hh];
        if (seg > 0)
            for (int j = seg * SEG; j < (seg + 1) * SEG; ++j) s_a[j][hh] += base;
    }
    __syncthreads();
    for (int i = tid; i < Q * HB; i += MTHREADS) {
        const int j = i % Q, hl = i / Q, h = hb * HB + hl;
        if (h >= s.H) continue;
        const float csv = s_a[j][hl], r = s_a[j | 31][hl];
        const int64_t o = (((int64_t)b * s.nc + c) * s.H + h) * Q + j;
        cs2[o] = csv * LOG2E;
        fdec[o] = s_d[j][hl] * fast_exp2((r - csv) * LOG2E);
        cdec[o] = s_d[j][hl] * fast_exp2((s_a[Q - 1][hl] - csv) * LOG2E);
    }
}

// =========================================================================================
// pass.  Workgroup = (batch, head, slice of 32 channels), 8 waves in two roles:
//   waves 0..3 (compute) hold the state and do every contraction of the chunk in hand;
//   waves 4..7 (stage)   fetch the NEXT chunks' own inputs (x, dt, the tables: the loads with
//                        HBM latency) and write the transposed x tiles and the per-token tables
//                        of chunk c+1 into the other half of a double-buffered LDS area.
// Loads complete in issue order within a wave, so a wave that waits for an operand it asked
// for a moment ago also waits for everything it asked for before; keeping the long-latency
// loads in waves of their own lets the compute waves wait for L2-resident operands only.
// One workgroup barrier per chunk.
// LDS per buffer: xd^T = x^T, xs^T = (f x)^T, xc^T = (coef x)^T as [channel][token position]
// bf16 tiles, cs2 and dt tables, and the bf16 image of the state carried into the chunk.
// =========================================================================================
constexpr int PASS_THREADS = 512;

template <int Q>
struct PassLds {
    static constexpr int XSTR = Q + 8;           // row stride of the transposed x tiles
    static constexpr int HSTR = MN + 8;          // row stride of the state tile
    static constexpr int TILE = 32 * XSTR;       // elements per x tile
    static constexpr int HT = 32 * HSTR;
    // per buffer: three x tiles, the state tile, two tables
    static constexpr size_t BUF_BYTES = (size_t)(3 * TILE + HT) * 2 + 2 * Q * sizeof(float);
    static constexpr int YT = Q * 32;            // elements of one output tile, [token][channel]
    static constexpr size_t ID_BYTES = 2 * 2 * 64 * 16;   // D I as operand registers, two bf16 terms
    static constexpr size_t BYTES = 2 * BUF_BYTES + 2 * (size_t)YT * 2 + ID_BYTES;
};

template <int Q>
__global__ void __launch_bounds__(PASS_THREADS)
pass_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dt, const float *__restrict__ D,
            const uint16_t *__restrict__ cmix, const uint16_t *__restrict__ bt8,
            const uint16_t *__restrict__ cb, const float *__restrict__ cs2, const float *__restrict__ fdec,
            const float *__restrict__ cdec, const float *__restrict__ h0, float *__restrict__ h_final,
            uint16_t *__restrict__ y, Shape s, int NS, int total, int nblocks)
{
    using Lds = PassLds<Q>;
    constexpr int NT = Q / 32;                   // 32-token tiles per chunk
    constexpr int NP = NT * (NT + 1) / 2;
    constexpr int KS = Q / 16;                   // k-steps of the state contraction
    constexpr int XSTR = Lds::XSTR, HSTR = Lds::HSTR;
    constexpr int TPW = NT >= 8 ? 2 : 1;         // output tiles per compute wave
    constexpr int NQ = TPW == 2 ? NT + 1 : NT;   // tile pairs per compute wave
    constexpr int UNITS = (Q / 8) * 16;          // x staging units: 8 tokens x 2 channels
    constexpr int XU = (UNITS + 255) / 256;      // units per staging lane
    constexpr int CBD = NQ < 4 ? NQ : 4;         // G^T tiles in flight
    extern __shared__ __align__(16) unsigned char smem_raw[];
    auto lds_xd = [&](int buf) { return reinterpret_cast<uint16_t *>(smem_raw + buf * Lds::BUF_BYTES); };
    auto lds_xs = [&](int buf) { return lds_xd(buf) + Lds::TILE; };
    auto lds_xc = [&](int buf) { return lds_xd(buf) + 2 * Lds::TILE; };
    auto lds_h = [&](int buf) { return lds_xd(buf) + 3 * Lds::TILE; };
    auto lds_cs = [&](int buf) { return reinterpret_cast<float *>(lds_xd(buf) + 3 * Lds::TILE + Lds::HT); };
    auto lds_dt = [&](int buf) { return lds_cs(buf) + Q; };
    auto lds_y = [&](int buf) { return reinterpret_cast<uint16_t *>(smem_raw + 2 * Lds::BUF_BYTES) + buf * Lds::YT; };
    uint4 *lds_id = reinterpret_cast<uint4 *>(smem_raw + 2 * Lds::BUF_BYTES + 2 * (size_t)Lds::YT * 2);   // [part][t][lane]

    const int lid = xcd_logical_id(blockIdx.x, nblocks);
    if (lid >= total) return;
    const int sl = lid % NS;
    const int h = (lid / NS) % s.H;
    const int b = lid / (NS * s.H);
    const int g = (h * s.G) / s.H;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kg = lane >> 5;
    const int P0 = 32 * sl;
    const int tokstride = s.H * s.P;

    if (wave >= 4) {
        // =============================== stage waves ===============================
        const int pt0 = tid - 256;
        // The lane's indices are derived from an opaque copy once per chunk (see the compute waves):
        // pt = lane of the stage group, p2s = the two channels it stages (channels past P are
        // staged as zeros), tq = its token in the per-token tables.
#define SWIMBA_PASS_LANE_IDS()                                                                             \
        int pt = pt0;                                                                                      \
        asm volatile("" : "+v"(pt));                                                                       \
        const int p2s = pt & 15;                                                                           \
        const bool pok = P0 + 2 * p2s < s.P;                                                               \
        const unsigned pcl = pok ? (unsigned)(P0 + 2 * p2s) : 0u;                                          \
        const int tq = min(pt, Q - 1);
        // Two register sets for x, A and B: the loads of chunk c+2 and c+3 are in flight while
        // chunk c+1 is staged, so a load from HBM has two chunk times to arrive.  The per-token
        // tables (small, re-read by the sibling slice) follow one chunk ahead in one set.
        uint32_t xvA[XU][8], xvB[XU][8];
        float4 fv[XU][2], cv[XU][2];             // the tables: one set, requested one chunk ahead
        float cs_raw;
        uint16_t dt_raw;
        // x of chunk c_ into set S_, clamped and unconditional
#define SWIMBA_PASS_ISSUE(S_, c_)                                                                          \
        {                                                                                                  \
            const int cc_ = min((c_), s.nc - 1);                                                           \
            const int64_t tok0_ = (int64_t)b * s.L + (int64_t)cc_ * Q;                                     \
            const int valid_ = min(Q, s.L - cc_ * Q);                                                      \
            const uint16_t *xh_ = x + (tok0_ * s.H + h) * s.P;                                             \
            _Pragma("unroll") for (int it = 0; it < XU; ++it) {                                            \
                const int u = min(pt + it * 256, UNITS - 1);                                               \
                const int gi = u >> 4, t16 = gi >> 1, kgx = gi & 1;                                        \
                _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                            \
                    const int j = 16 * t16 + 8 * (e >> 2) + 4 * kgx + (e & 3);                             \
                    xv##S_[it][e] = *reinterpret_cast<const uint32_t *>(                                   \
                        xh_ + ((unsigned)min(j, valid_ - 1) * (unsigned)tokstride + pcl));                 \
                }                                                                                          \
            }                                                                                              \
        }
        // the tables of chunk c_
#define SWIMBA_PASS_ISSUE_TABLES(c_)                                                                       \
        {                                                                                                  \
            const int cc_ = min((c_), s.nc - 1);                                                           \
            const int64_t tok0_ = (int64_t)b * s.L + (int64_t)cc_ * Q;                                     \
            const int valid_ = min(Q, s.L - cc_ * Q);                                                      \
            const int64_t tb_ = (((int64_t)b * s.nc + cc_) * s.H + h) * Q;                                 \
            cs_raw = (cs2 + tb_)[(unsigned)tq];                                                            \
            dt_raw = (dt + tok0_ * s.H + h)[(unsigned)min(tq, valid_ - 1) * (unsigned)s.H];                \
            _Pragma("unroll") for (int it = 0; it < XU; ++it) {                                            \
                const int u = min(pt + it * 256, UNITS - 1);                                               \
                const int gi = u >> 4, t16 = gi >> 1, kgx = gi & 1;                                        \
                const unsigned to_ = (unsigned)(16 * t16 + 4 * kgx);                                       \
                fv[it][0] = *reinterpret_cast<const float4 *>(fdec + tb_ + to_);                           \
                fv[it][1] = *reinterpret_cast<const float4 *>(fdec + tb_ + to_ + 8u);                      \
                cv[it][0] = *reinterpret_cast<const float4 *>(cdec + tb_ + to_);                           \
                cv[it][1] = *reinterpret_cast<const float4 *>(cdec + tb_ + to_ + 8u);                      \
            }                                                                                              \
        }
        // tables and the three transposed tiles of chunk c_ (held in set S_) -> buffer buf_
#define SWIMBA_PASS_STAGE(S_, c_, buf_)                                                                    \
        {                                                                                                  \
            const int valid_ = min(Q, s.L - min((c_), s.nc - 1) * Q);                                      \
            if (pt < Q) {                                                                                  \
                lds_cs(buf_)[pt] = cs_raw;                                                             \
                lds_dt(buf_)[pt] = (pt < valid_) ? to_float(bf16{dt_raw}) : 0.f;                       \
            }                                                                                              \
            _Pragma("unroll") for (int it = 0; it < XU; ++it) {                                            \
                const int u = pt + it * 256;                                                               \
                if (XU * 256 > UNITS && u >= UNITS) break;                                                 \
                const int gi = u >> 4, t16 = gi >> 1, kgx = gi & 1;                                        \
                const float fj[8] = {fv[it][0].x, fv[it][0].y, fv[it][0].z, fv[it][0].w,                   \
                                     fv[it][1].x, fv[it][1].y, fv[it][1].z, fv[it][1].w};                  \
                const float cj[8] = {cv[it][0].x, cv[it][0].y, cv[it][0].z, cv[it][0].w,                   \
                                     cv[it][1].x, cv[it][1].y, cv[it][1].z, cv[it][1].w};                  \
                uint32_t r[8];                                                                             \
                float xa[8], xb[8], ca[8], cbv[8];                                                         \
                _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                            \
                    const int j = 16 * t16 + 8 * (e >> 2) + 4 * kgx + (e & 3);                             \
                    r[e] = (pok && j < valid_) ? xv##S_[it][e] : 0u;                                       \
                    const float lo_ = bf_lo(r[e]), hi_ = bf_hi(r[e]);                                      \
                    xa[e] = lo_ * fj[e]; xb[e] = hi_ * fj[e];                                              \
                    ca[e] = lo_ * cj[e]; cbv[e] = hi_ * cj[e];                                             \
                }                                                                                          \
                uint4 lo, hi;                                                                              \
                lo.x = __builtin_amdgcn_perm(r[1], r[0], 0x05040100u);                                     \
                lo.y = __builtin_amdgcn_perm(r[3], r[2], 0x05040100u);                                     \
                lo.z = __builtin_amdgcn_perm(r[5], r[4], 0x05040100u);                                     \
                lo.w = __builtin_amdgcn_perm(r[7], r[6], 0x05040100u);                                     \
                hi.x = __builtin_amdgcn_perm(r[1], r[0], 0x07060302u);                                     \
                hi.y = __builtin_amdgcn_perm(r[3], r[2], 0x07060302u);                                     \
                hi.z = __builtin_amdgcn_perm(r[5], r[4], 0x07060302u);                                     \
                hi.w = __builtin_amdgcn_perm(r[7], r[6], 0x07060302u);                                     \
                const int off = 16 * t16 + 8 * kgx;                                                        \
                *reinterpret_cast<uint4 *>(lds_xd(buf_) + (2 * p2s) * XSTR + off) = lo;                    \
                *reinterpret_cast<uint4 *>(lds_xd(buf_) + (2 * p2s + 1) * XSTR + off) = hi;                \
                *reinterpret_cast<uint4 *>(lds_xs(buf_) + (2 * p2s) * XSTR + off) = pack8(xa);             \
                *reinterpret_cast<uint4 *>(lds_xs(buf_) + (2 * p2s + 1) * XSTR + off) = pack8(xb);         \
                *reinterpret_cast<uint4 *>(lds_xc(buf_) + (2 * p2s) * XSTR + off) = pack8(ca);             \
                *reinterpret_cast<uint4 *>(lds_xc(buf_) + (2 * p2s + 1) * XSTR + off) = pack8(cbv);        \
            }                                                                                              \
        }
        // the output tile the compute waves left in LDS for chunk c_ -> y, as whole 64-byte rows
#define SWIMBA_PASS_STORE_Y(c_)                                                                            \
        {                                                                                                  \
            const int cc_ = (c_);                                                                          \
            const int valid_ = min(Q, s.L - cc_ * Q);                                                      \
            const uint16_t *sy_ = lds_y(cc_ & 1);                                                          \
            uint16_t *yh_ = y + (((int64_t)b * s.L + (int64_t)cc_ * Q) * s.H + h) * s.P + P0;              \
            _Pragma("unroll") for (int it = 0; it < Q * 4 / 256; ++it) {                                   \
                const int pi = pt + it * 256, tk = pi >> 2, part = pi & 3;                                 \
                const uint4 v_ = *reinterpret_cast<const uint4 *>(sy_ + tk * 32 + part * 8);               \
                if (tk < valid_ && P0 + part * 8 < s.P)                                                    \
                    *reinterpret_cast<uint4 *>(yh_ + ((unsigned)tk * (unsigned)tokstride + (unsigned)(part * 8))) = v_; \
            }                                                                                              \
        }
        // ---- running state: S^T[n = 32 sw + 8a + 4kg + b][p = P0 + l32] in register 4a + b ----
        const int sw = wave - 4;
        f32x16_t st;
        {
            const int p = P0 + l32;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int n0 = 32 * sw + 8 * a + 4 * kg;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (h0 && p < s.P && n0 < s.N)
                    v = *reinterpret_cast<const float4 *>(h0 + (((int64_t)b * s.H + h) * s.P + p) * s.N + n0);
                st[4 * a + 0] = v.x; st[4 * a + 1] = v.y; st[4 * a + 2] = v.z; st[4 * a + 3] = v.w;
            }
        }
        // the bf16 image of the state the compute waves read for the next chunk
#define SWIMBA_PASS_PUT_STATE(buf_)                                                                        \
        _Pragma("unroll") for (int a = 0; a < 4; ++a) {                                                    \
            const int n0 = 32 * sw + 8 * a + 4 * kg;                                                       \
            uint2 v;                                                                                       \
            v.x = pack_bf16x2(st[4 * a + 0], st[4 * a + 1]);                                               \
            v.y = pack_bf16x2(st[4 * a + 2], st[4 * a + 3]);                                               \
            *reinterpret_cast<uint2 *>(lds_h(buf_) + l32 * HSTR + n0) = v;                                 \
        }
        // mixed B rows of this wave's state rows, chunk c_ (operand of the state update): L2
        const unsigned bt_off = (unsigned)(kg * MN + sw * 32 + l32) * 8u;    // + ks * 2 * MN * 8
        uint4 bt[KS];
#define SWIMBA_PASS_LOAD_BT(c_)                                                                            \
        {                                                                                                  \
            const uint16_t *bt_c = bt8 + (((int64_t)b * s.nc + min((c_), s.nc - 1)) * s.G + g) * ((Q / 8) * MN * 8); \
            _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                              \
                bt[ks] = *reinterpret_cast<const uint4 *>(bt_c + bt_off + (unsigned)ks * (2 * MN * 8));    \
        }
        // H <- exp(cs_last) H + Bmix^T . (coef x) for the chunk staged in buffer buf_, then its bf16
        // image for the next chunk; the mixed B rows of the chunk after it are requested right behind
#define SWIMBA_PASS_STATE_UPDATE(c_, buf_)                                                                 \
        {                                                                                                  \
            const float dec = fast_exp2(lds_cs(buf_)[Q - 1]);                                              \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) st[v] *= dec;                                   \
            const uint16_t *sB = lds_xc(buf_) + l32 * XSTR + 8 * kg;                                       \
            _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                              \
                st = mfma32(bt[ks], *reinterpret_cast<const uint4 *>(sB + ks * 16), st);                   \
            __builtin_amdgcn_sched_barrier(0);                                                             \
            SWIMBA_PASS_LOAD_BT((c_) + 1);                                                                 \
            __builtin_amdgcn_sched_barrier(0);                                                             \
            SWIMBA_PASS_PUT_STATE((buf_) ^ 1);                                                             \
        }
        SWIMBA_PASS_PUT_STATE(0);
        {
            SWIMBA_PASS_LANE_IDS();
            SWIMBA_PASS_ISSUE(A, 0);
            SWIMBA_PASS_ISSUE_TABLES(0);
            SWIMBA_PASS_ISSUE(B, 1);
            SWIMBA_PASS_LOAD_BT(0);
            SWIMBA_PASS_STAGE(A, 0, 0);
            SWIMBA_PASS_ISSUE_TABLES(1);
            SWIMBA_PASS_ISSUE(A, 2);
        }
        // Iteration c updates the state with chunk c, stores the output of chunk c-1 and stages chunk
        // c+1 into the buffer nobody reads during it (past the end: the last chunk once more, which
        // nobody will read).  Even c: set B, odd c: set A.
        for (int c = 0; c < s.nc; c += 2) {
            {
                SWIMBA_PASS_LANE_IDS();
                lds_barrier();
                SWIMBA_PASS_STATE_UPDATE(c, 0);
                if (c > 0) SWIMBA_PASS_STORE_Y(c - 1);
                SWIMBA_PASS_STAGE(B, c + 1, 1);
                SWIMBA_PASS_ISSUE_TABLES(c + 2);
                SWIMBA_PASS_ISSUE(B, c + 3);
            }
            if (c + 1 < s.nc) {
                SWIMBA_PASS_LANE_IDS();
                lds_barrier();
                SWIMBA_PASS_STATE_UPDATE(c + 1, 1);
                SWIMBA_PASS_STORE_Y(c);
                SWIMBA_PASS_STAGE(A, c + 2, 0);
                SWIMBA_PASS_ISSUE_TABLES(c + 3);
                SWIMBA_PASS_ISSUE(A, c + 4);
            }
        }
        lds_barrier();
        {
            SWIMBA_PASS_LANE_IDS();
            SWIMBA_PASS_STORE_Y(s.nc - 1);
        }
        if (h_final) {
            const int p = P0 + l32;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int n0 = 32 * sw + 8 * a + 4 * kg;
                if (p < s.P && n0 < s.N)
                    *reinterpret_cast<float4 *>(h_final + (((int64_t)b * s.H + h) * s.P + p) * s.N + n0) =
                        make_float4(st[4 * a + 0], st[4 * a + 1], st[4 * a + 2], st[4 * a + 3]);
            }
        }
#undef SWIMBA_PASS_PUT_STATE
#undef SWIMBA_PASS_LOAD_BT
#undef SWIMBA_PASS_STATE_UPDATE
#undef SWIMBA_PASS_LANE_IDS
#undef SWIMBA_PASS_ISSUE
#undef SWIMBA_PASS_ISSUE_TABLES
#undef SWIMBA_PASS_STAGE
#undef SWIMBA_PASS_STORE_Y
        return;
    }

    // =============================== compute waves ===============================
    // channel held by operand row l32 of the Y^T contractions: accumulator row 8a + 4kg + b is then
    // channel 16kg + 4a + b, so a lane ends with 16 consecutive channels of one token
    const int prow = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);
    const int I0 = min(wave, NT - 1);                       // first output tile of the wave
    const int I1 = NT - 1 - wave;                           // second one (TPW == 2)
    const bool wave_on = wave < NT;                         // Q = 64: waves 2, 3 own no output tile
    const unsigned lane8_0 = (unsigned)lane * 8u;

    // Skip term as one more contraction of the diagonal tile: Y^T += x^T . (D I), with D split into
    // two bf16 terms (16 significant bits; y is rounded to 8).  B operand of k-step t: lane
    // (column i = l32, kg) holds rows j = 16t + 8(e>>2) + 4kg + (e&3); the entry is D where j == i.
    // The operand registers are kept in LDS (every wave writes the same values before the first
    // barrier) and read back where a diagonal tile needs them.
    const bool has_D = D != nullptr;
    if (wave == 0) {
        const float dv = has_D ? D[h] : 0.f;
        const uint32_t dh = bf16_bits_rne(dv);
        const uint32_t dl = bf16_bits_rne(dv - __uint_as_float(dh << 16));
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            uint32_t wh[4], wl[4];
#pragma unroll
            for (int e2 = 0; e2 < 4; ++e2) {
                const int e = 2 * e2;
                const int j0 = 16 * t + 8 * (e >> 2) + 4 * kg + (e & 3), j1 = j0 + 1;
                wh[e2] = (j0 == l32 ? dh : 0u) | (j1 == l32 ? dh << 16 : 0u);
                wl[e2] = (j0 == l32 ? dl : 0u) | (j1 == l32 ? dl << 16 : 0u);
            }
            lds_id[(0 * 2 + t) * 64 + lane] = make_uint4(wh[0], wh[1], wh[2], wh[3]);
            lds_id[(1 * 2 + t) * 64 + lane] = make_uint4(wl[0], wl[1], wl[2], wl[3]);
        }
    }

    // Operand loads run ahead of their use in register slots rotated by name: the mixed C rows of
    // the next tile are requested as soon as those in hand have gone into their contractions, a
    // G^T tile CBS steps ahead of its step, across the chunk boundary.
    constexpr int CBS = NQ < 5 ? NQ : 5;          // register slots of G^T tiles
    constexpr int NQP = (NQ + CBS - 1) / CBS * CBS;   // steps per chunk padded to a multiple of CBS,
                                                  // so that step q always finds its tile in slot q % CBS
    uint4 cfrag[8];           // mixed C rows of one output tile at a time
    uint4 cbt[CBS][2];
#define SWIMBA_PASS_LOAD_C(c_, I_)                                                                         \
    {                                                                                                      \
        const uint16_t *cm_ = cmix + (((int64_t)b * s.nc + (c_)) * s.G + g) * (NT * 8 * 64 * 8);           \
        const unsigned o = (unsigned)(I_) * (8 * 64 * 8) + lane8;                                          \
        _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)                                                   \
            cfrag[ks] = *reinterpret_cast<const uint4 *>(cm_ + o + ks * 64 * 8);                           \
    }
#define SWIMBA_PASS_LOAD_CB(c_, q_)                                                                        \
    {                                                                                                      \
        const uint16_t *cb_ = cb + (((int64_t)b * s.nc + (c_)) * s.G + g) * (NP * 2 * 64 * 8);             \
        const bool first_ = TPW == 1 || (q_) <= wave;                                                      \
        const int I_ = first_ ? I0 : I1;                                                                   \
        const int J_ = min(first_ ? (q_) : (q_) - wave - 1, I_);                                           \
        const unsigned o_ = (unsigned)(I_ * (I_ + 1) / 2 + J_) * (2 * 64 * 8) + lane8;                     \
        cbt[(q_) % CBS][0] = *reinterpret_cast<const uint4 *>(cb_ + o_);                                   \
        cbt[(q_) % CBS][1] = *reinterpret_cast<const uint4 *>(cb_ + o_ + 64 * 8);                          \
    }
    {
        unsigned lane8 = lane8_0;
        SWIMBA_PASS_LOAD_C(0, I0);
#pragma unroll
        for (int q = 0; q < CBS; ++q) SWIMBA_PASS_LOAD_CB(0, q);
    }

    for (int c = 0; c < s.nc; ++c) {
        const int buf = c & 1;
        const int cn = min(c + 1, s.nc - 1);               // next chunk (the last one asks for itself again)
        // The lane's offsets are made opaque once per chunk: otherwise every address derived from
        // them (one per tile pair, per k-step, ...) is computed in front of the loop and kept in a
        // register of its own across it, which pushes the kernel over its register budget.
        unsigned lane8 = lane8_0, prowx = (unsigned)prow;
        asm volatile("" : "+v"(lane8), "+v"(prowx));

        lds_barrier();          // chunk c is staged, the state image of chunk c is written
        const uint16_t *sXd = lds_xd(buf), *sXs = lds_xs(buf), *sH = lds_h(buf);
        const float *s_cs = lds_cs(buf), *s_dt = lds_dt(buf);

        if (wave_on) {
            f32x16_t yt[TPW];
            float csi[TPW];
            // ---- Y^T = exp(cs_i) H_c . Cmix^T for the first tile; the second tile's mixed C rows
            // ---- take the buffer's place and its readout follows half-way through the steps ----
            {
                f32x16_t acc = {0};
#pragma unroll
                for (int ks = 0; ks < 8; ++ks)
                    acc = mfma32(*reinterpret_cast<const uint4 *>(sH + prowx * HSTR + 64 * kg + ks * 8), cfrag[ks], acc);
                __builtin_amdgcn_sched_barrier(0);
                if (TPW == 2) SWIMBA_PASS_LOAD_C(c, I1) else SWIMBA_PASS_LOAD_C(cn, I0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < TPW; ++t) csi[t] = s_cs[(t == 0 ? I0 : I1) * 32 + l32];
                const float sc = fast_exp2(csi[0]);
#pragma unroll
                for (int v = 0; v < 16; ++v) yt[0][v] = sc * acc[v];
                if (TPW == 2) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) yt[TPW - 1][v] = 0.f;
                }
            }
            // ---- intra-chunk part ----
            const uint16_t *sXsr = sXs + prowx * XSTR + 8 * kg;
            const uint16_t *sXdr = sXd + prowx * XSTR + 8 * kg;
#pragma unroll
            for (int q = 0; q < NQP; ++q) {
                if (TPW == 2 && q == NQ / 2) {
                    f32x16_t acc = {0};
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks)
                        acc = mfma32(*reinterpret_cast<const uint4 *>(sH + prowx * HSTR + 64 * kg + ks * 8), cfrag[ks], acc);
                    __builtin_amdgcn_sched_barrier(0);
                    SWIMBA_PASS_LOAD_C(cn, I0);
                    __builtin_amdgcn_sched_barrier(0);
                    const float sc = fast_exp2(csi[TPW - 1]);
#pragma unroll
                    for (int v = 0; v < 16; ++v) yt[TPW - 1][v] += sc * acc[v];
                }
                const bool first = TPW == 1 || q <= wave;
                const int I = first ? I0 : I1;
                const int J = first ? q : q - wave - 1;
                const bool on = q < NQ && (TPW == 2 || q <= wave);
                const float ci = first ? csi[0] : csi[TPW - 1];
                if (on && J < I) {
                    f32x16_t tmp = {0};
                    tmp = mfma32(*reinterpret_cast<const uint4 *>(sXsr + J * 32), cbt[q % CBS][0], tmp);
                    tmp = mfma32(*reinterpret_cast<const uint4 *>(sXsr + J * 32 + 16), cbt[q % CBS][1], tmp);
                    const float ei = fast_exp2(ci - s_cs[J * 32 + 31]);
                    if (first) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) yt[0][v] += ei * tmp[v];
                    } else {
#pragma unroll
                        for (int v = 0; v < 16; ++v) yt[TPW - 1][v] += ei * tmp[v];
                    }
                } else if (on) {
                    // diagonal tile: direct masked form on the unscaled x
                    float m[16];
                    unpack8(m, cbt[q % CBS][0]);
                    unpack8(m + 8, cbt[q % CBS][1]);
                    const float *cj = s_cs + J * 32 + 4 * kg;
                    const float *dj = s_dt + J * 32 + 4 * kg;
                    // All eight table rows are requested before the first is used (one LDS round trip
                    // instead of four); left alone, the compiler sinks each read under the lane mask
                    // of the select that consumes it and waits for every one in turn.
                    float4 c4[4], d4[4];
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        c4[a] = *reinterpret_cast<const float4 *>(cj + 8 * a);
                        d4[a] = *reinterpret_cast<const float4 *>(dj + 8 * a);
                    }
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int a = 0; a < 4; ++a) {
                        const float cc[4] = {c4[a].x, c4[a].y, c4[a].z, c4[a].w};
                        const float dd[4] = {d4[a].x, d4[a].y, d4[a].z, d4[a].w};
#pragma unroll
                        for (int bb = 0; bb < 4; ++bb) {
                            const int jl = 8 * a + 4 * kg + bb;
                            // masked entries (j > i) get a hugely negative exponent: exp2 -> 0; the
                            // cumsum is non-increasing up to its last rounding, so the argument of a
                            // kept entry is at most a rounding error above zero
                            const float arg = (l32 >= jl) ? ci - cc[bb] : -1.0e30f;
                            m[4 * a + bb] *= fast_exp2(arg) * dd[bb];
                        }
                    }
                    const uint4 m0 = pack8(m), m1 = pack8(m + 8);
                    const uint4 x0 = *reinterpret_cast<const uint4 *>(sXdr + J * 32);
                    const uint4 x1 = *reinterpret_cast<const uint4 *>(sXdr + J * 32 + 16);
                    if (first) {
                        yt[0] = mfma32(x0, m0, yt[0]);
                        yt[0] = mfma32(x1, m1, yt[0]);
                        if (has_D) {
                            yt[0] = mfma32(x0, lds_id[0 * 64 + lane], yt[0]);
                            yt[0] = mfma32(x1, lds_id[1 * 64 + lane], yt[0]);
                            yt[0] = mfma32(x0, lds_id[2 * 64 + lane], yt[0]);
                            yt[0] = mfma32(x1, lds_id[3 * 64 + lane], yt[0]);
                        }
                    } else {
                        yt[TPW - 1] = mfma32(x0, m0, yt[TPW - 1]);
                        yt[TPW - 1] = mfma32(x1, m1, yt[TPW - 1]);
                        if (has_D) {
                            yt[TPW - 1] = mfma32(x0, lds_id[0 * 64 + lane], yt[TPW - 1]);
                            yt[TPW - 1] = mfma32(x1, lds_id[1 * 64 + lane], yt[TPW - 1]);
                            yt[TPW - 1] = mfma32(x0, lds_id[2 * 64 + lane], yt[TPW - 1]);
                            yt[TPW - 1] = mfma32(x1, lds_id[3 * 64 + lane], yt[TPW - 1]);
                        }
                    }
                }
                // the slot this step has just emptied takes the tile of step q + CBS (past the
                // chunk's last step: of the next chunk; padding steps have no tile)
                __builtin_amdgcn_sched_barrier(0);
                if (q + CBS < NQ) SWIMBA_PASS_LOAD_CB(c, q + CBS)
                else if (q + CBS >= NQP && q + CBS - NQP < NQ) SWIMBA_PASS_LOAD_CB(cn, q + CBS - NQP);
                __builtin_amdgcn_sched_barrier(0);
            }
            // ---- the output tile as bf16 into LDS ([token][channel]); the stage waves store it ----
            uint16_t *sY = lds_y(buf);
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                float o0[8], o1[8];
#pragma unroll
                for (int e = 0; e < 8; ++e) { o0[e] = yt[t][e]; o1[e] = yt[t][8 + e]; }
                uint16_t *dst = sY + ((t == 0 ? I0 : I1) * 32 + l32) * 32 + 16 * kg;
                *reinterpret_cast<uint4 *>(dst) = pack8(o0);
                *reinterpret_cast<uint4 *>(dst + 8) = pack8(o1);
            }
        }
    }
    lds_barrier();              // the stage waves store the last chunk's output after this one
#undef SWIMBA_PASS_LOAD_C
#undef SWIMBA_PASS_LOAD_CB
}

template <int Q>
static swimba_status launch_prep_q(const Shape &s, const void *dt, const float *A, const void *cmix,
                                   const void *bfrag, void *cb, float *cs2, float *fdec, float *cdec,
                                   hipStream_t st, bool tiles)
{
    constexpr int NT = Q / 32;
    const int64_t nbcg = (int64_t)s.B * s.nc * s.G;
    if (nbcg == 0) return SWIMBA_OK;
    // G^T tiles: one workgroup per (batch, chunk, group) with the mixed B rows shared through LDS
    // where there are enough of them to fill the chip (49 against 55 us on the long-sequence
    // workload, 1024 triples), one wave per tile pair otherwise (12 against 17 us with 64 triples)
    const int fine = nbcg < 512;
    // (tiles == false: the tiles exist already, only the tables are made)
    const int64_t ncb = !tiles ? 0 : fine ? xcd_padded(nbcg * ((NT * (NT + 1) / 2 + 3) / 4)) : nbcg;
    const int64_t ncum = (int64_t)s.B * s.nc * ((s.H + 15) / 16);
    hipLaunchKernelGGL(prep_kernel<Q>, dim3((unsigned)(ncb + ncum)), dim3(MTHREADS), 0, st, (const uint16_t *)dt, A,
                       (const uint16_t *)cmix, (const uint16_t *)bfrag, (uint16_t *)cb, cs2, fdec, cdec, s, nbcg, ncb,
                       fine);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_prep_mfma(const Shape &s, const void *dt, const float *A, const void *cmix, const void *bfrag,
                               void *cb, float *cs2, float *fdec, float *cdec, hipStream_t st, bool tiles)
{
    switch (s.Q) {
    case 64: return launch_prep_q<64>(s, dt, A, cmix, bfrag, cb, cs2, fdec, cdec, st, tiles);
    case 128: return launch_prep_q<128>(s, dt, A, cmix, bfrag, cb, cs2, fdec, cdec, st, tiles);
    case 256: return launch_prep_q<256>(s, dt, A, cmix, bfrag, cb, cs2, fdec, cdec, st, tiles);
    }
    return SWIMBA_ERR_UNSUPPORTED;
}

template <int Q>
static swimba_status launch_pass_q(const Shape &s, const void *x, const void *dt, const float *D, const void *cmix,
                                   const void *bt8, const void *cb, const float *cs2, const float *fdec,
                                   const float *cdec, const float *h0, float *h_final, void *y, hipStream_t st)
{
    const int NS = (s.P + 31) / 32;
    const int64_t total = (int64_t)s.B * s.H * NS;
    if (total == 0 || s.nc == 0) return SWIMBA_OK;
    const int nblocks = xcd_padded(total);
    const size_t shm = PassLds<Q>::BYTES;
    // more than 64 KB of dynamic LDS has to be allowed once per device (a plain attribute call:
    // legal under stream capture, but the first call on a device is best made before capturing)
    static std::atomic<uint64_t> attr_set{0};            // one bit per device ordinal
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
    const uint64_t bit = 1ull << (dev & 63);
    if (!(attr_set.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute((const void *)pass_kernel<Q>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
        attr_set.fetch_or(bit, std::memory_order_release);
    }
    hipLaunchKernelGGL(pass_kernel<Q>, dim3(nblocks), dim3(PASS_THREADS), shm, st, (const uint16_t *)x,
                       (const uint16_t *)dt, D, (const uint16_t *)cmix, (const uint16_t *)bt8, (const uint16_t *)cb,
                       cs2, fdec, cdec, h0, h_final, (uint16_t *)y, s, NS, (int)total, nblocks);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_pass_mfma(const Shape &s, const void *x, const void *dt, const float *D, const void *cmix,
                               const void *bt8, const void *cb, const float *cs2, const float *fdec,
                               const float *cdec, const float *h0, float *h_final, void *y, hipStream_t st)
{
    switch (s.Q) {
    case 64: return launch_pass_q<64>(s, x, dt, D, cmix, bt8, cb, cs2, fdec, cdec, h0, h_final, y, st);
    case 128: return launch_pass_q<128>(s, x, dt, D, cmix, bt8, cb, cs2, fdec, cdec, h0, h_final, y, st);
    case 256: return launch_pass_q<256>(s, x, dt, D, cmix, bt8, cb, cs2, fdec, cdec, h0, h_final, y, st);
    }
    return SWIMBA_ERR_UNSUPPORTED;
}

}  // namespace swimba
