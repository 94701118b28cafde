// Single-pass SSD forward, one workgroup per (batch, head) with all 64 channels of the head
// (paper, background section on SSD: matrix multiplications inside chunks, a linear recurrence
// between chunks; the recurrence of a head is independent of every other head's).
//
// Same algorithm, inputs (prep's tiles and tables, the mixed rows) and roles as pass_kernel
// (fused_pass.hip), which gives a workgroup 32 channels.  A workgroup's time per chunk is
// dominated by the operands every workgroup of a (batch, group) reads through its compute unit's
// vector memory path (mixed C rows, mixed B rows, G^T tiles: 200 KB per chunk); with 64 channels
// those bytes serve twice the work.  To fit LDS only ONE transposed x tile is kept (a pure bf16
// transpose) and every per-token factor goes into the shared operand instead of into x:
//   tiles left of the diagonal   M^T[j][i] = G^T[j][i] * exp(cs_i - R_J) * f_j      f_j = dt_j exp(R_J - cs_j)
//   diagonal tile                M^T[j][i] = G^T[j][i] * exp(cs_i - cs_j) dt_j  [j <= i]
//   state build                  H <- exp(cs_last) H + (Bmix^T * coef) . x        coef_j = dt_j exp(cs_last - cs_j)
// (R_J = cs at the last token of tile J; every exponent is non-positive).  The output tile of a
// compute wave goes through a scratch area of its own in LDS and leaves as whole 128-byte rows.
//   waves 0..3 (compute): carried-state readout, tile pairs, skip term, y stores
//   waves 4..7 (stage):   x two chunks ahead and the per-token tables one chunk ahead into the
//                         other half of a double-buffered LDS area; they own the running state
//                         (128 x 64 fp32 in accumulators, wave w rows n = 32w .. 32w+31) and
//                         publish its bf16 image for the next chunk's readout.
// One LDS-only workgroup barrier per chunk.
//
// Split pass: the recurrence between chunks is linear in the state, so a sequence can be walked as
// nseg segments of whole chunks side by side once the states at the segment boundaries are known;
// launch_boundary_states_mfma builds them from the chunk states in front of each boundary, and the
// pass kernel then treats (sequence, segment) as its batch index.
#include "common.hpp"
#include "mfma_util.hpp"

#include <atomic>

namespace swimba {

constexpr int PASS64_THREADS = 512;

template <int Q>
struct Pass64Lds {
    static constexpr int XSTR = Q + 8;           // row stride of the transposed x tile
    static constexpr int HSTR = MN + 8;          // row stride of the state image
    static constexpr int XT = MP * XSTR;         // elements of the x tile, [channel][token position]
    static constexpr int HT = MP * HSTR;         // elements of the state image, [channel][n]
    // per buffer: x tile, state image, four per-token tables (cs2, dt, f, coef)
    static constexpr size_t BUF_BYTES = (size_t)(XT + HT) * 2 + 4 * Q * sizeof(float);
    static constexpr size_t YSCR_BYTES = 4 * 32 * MP * 2;      // one 32-token output tile per compute wave
    static constexpr size_t ID_BYTES = 2 * 2 * 64 * 16;        // D I as operand registers, two bf16 terms
    static constexpr size_t BYTES = 2 * BUF_BYTES + YSCR_BYTES + ID_BYTES;
};

template <int Q>
__global__ void __launch_bounds__(PASS64_THREADS)
pass64_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dt, const float *__restrict__ D,
              const uint16_t *__restrict__ cmix, const uint16_t *__restrict__ bt8,
              const uint16_t *__restrict__ cb, const float *__restrict__ cs2, const float *__restrict__ fdec,
              const float *__restrict__ cdec, const float *__restrict__ h0, float *__restrict__ h_final,
              uint16_t *__restrict__ y, Shape s, int total, int nblocks, int nseg,
              const float *__restrict__ hmid)
{
    using Lds = Pass64Lds<Q>;
    constexpr int NT = Q / 32;                   // 32-token tiles per chunk
    constexpr int NP = NT * (NT + 1) / 2;
    constexpr int KS = Q / 16;                   // k-steps of the state contraction
    constexpr int XSTR = Lds::XSTR, HSTR = Lds::HSTR;
    constexpr int TPW = NT >= 8 ? 2 : 1;         // output tiles per compute wave
    constexpr int NQ = TPW == 2 ? NT + 1 : NT;   // tile pairs per compute wave
    constexpr int UNITS = (Q / 8) * 32;          // x staging units: 8 tokens x 2 channels
    constexpr int XU = (UNITS + 255) / 256;      // units per staging lane
    extern __shared__ __align__(16) unsigned char smem_raw[];
    auto lds_x = [&](int buf) { return reinterpret_cast<uint16_t *>(smem_raw + buf * Lds::BUF_BYTES); };
    auto lds_h = [&](int buf) { return lds_x(buf) + Lds::XT; };
    auto lds_cs = [&](int buf) { return reinterpret_cast<float *>(lds_x(buf) + Lds::XT + Lds::HT); };
    auto lds_dt = [&](int buf) { return lds_cs(buf) + Q; };
    auto lds_f = [&](int buf) { return lds_cs(buf) + 2 * Q; };
    auto lds_c = [&](int buf) { return lds_cs(buf) + 3 * Q; };
    uint16_t *lds_y = reinterpret_cast<uint16_t *>(smem_raw + 2 * Lds::BUF_BYTES);
    uint4 *lds_id = reinterpret_cast<uint4 *>(smem_raw + 2 * Lds::BUF_BYTES + Lds::YSCR_BYTES);   // [part][t][lane]

    const int lid = xcd_logical_id(blockIdx.x, nblocks);
    if (lid >= total) return;
    const int h = lid % s.H;
    const int b = lid / s.H;
    const int g = (h * s.G) / s.H;
    // With nseg > 1 the shape is that of the segments: "batch" b is segment b % nseg of sequence
    // b / nseg (equal segments of whole chunks, so every token and chunk index is the same number in
    // both views).  A segment behind the first starts from the state at its boundary, which a launch
    // in front of this one has left in hmid (B, nseg - 1, H, P, N); only the last one ends in h_final.
    {
        const int seq = b / nseg, seg = b - seq * nseg;
        const int64_t hpn = (int64_t)s.P * s.N;
        if (seg > 0) h0 = hmid + (((int64_t)seq * (nseg - 1) + seg - 1) * s.H + h) * hpn;
        else if (h0) h0 += ((int64_t)seq * s.H + h) * hpn;
        h_final = (h_final && seg == nseg - 1) ? h_final + ((int64_t)seq * s.H + h) * hpn : nullptr;
    }
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kg = lane >> 5;
    const int tokstride = s.H * s.P;

    if (wave >= 4) {
        // =============================== stage waves ===============================
        const int pt0 = tid - 256;
        // The lane's indices are derived from an opaque copy once per chunk: the addresses built from
        // them are recomputed where they are used instead of staying in registers across the loop.
#define SWIMBA_P64_LANE_IDS()                                                                              \
        int pt = pt0;                                                                                      \
        asm volatile("" : "+v"(pt));                                                                       \
        const int tq = min(pt, Q - 1);
        // Two register sets for x, A and B: the loads of chunk c+2 and c+3 are in flight while chunk
        // c+1 is staged.  The per-token tables follow one chunk ahead in one set.
        uint32_t xvA[XU][8], xvB[XU][8];
        float cs_raw, f_raw, c_raw;
        uint16_t dt_raw;
        // x of chunk c_ into set S_, clamped and unconditional
#define SWIMBA_P64_ISSUE(S_, c_)                                                                           \
        {                                                                                                  \
            const int cc_ = min((c_), s.nc - 1);                                                           \
            const int64_t tok0_ = (int64_t)b * s.L + (int64_t)cc_ * Q;                                     \
            const int valid_ = min(Q, s.L - cc_ * Q);                                                      \
            const uint16_t *xh_ = x + (tok0_ * s.H + h) * s.P;                                             \
            _Pragma("unroll") for (int it = 0; it < XU; ++it) {                                            \
                const int u = min(pt + it * 256, UNITS - 1);                                               \
                const int p2 = u & 31, gi = u >> 5, t16 = gi >> 1, kgx = gi & 1;                           \
                const unsigned pcl = (2 * p2 < s.P) ? (unsigned)(2 * p2) : 0u;                             \
                _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                            \
                    const int j = 16 * t16 + 8 * (e >> 2) + 4 * kgx + (e & 3);                             \
                    xv##S_[it][e] = *reinterpret_cast<const uint32_t *>(                                   \
                        xh_ + ((unsigned)min(j, valid_ - 1) * (unsigned)tokstride + pcl));                 \
                }                                                                                          \
            }                                                                                              \
        }
        // the tables of chunk c_: one token per lane
#define SWIMBA_P64_ISSUE_TABLES(c_)                                                                        \
        {                                                                                                  \
            const int cc_ = min((c_), s.nc - 1);                                                           \
            const int64_t tok0_ = (int64_t)b * s.L + (int64_t)cc_ * Q;                                     \
            const int valid_ = min(Q, s.L - cc_ * Q);                                                      \
            const int64_t tb_ = (((int64_t)b * s.nc + cc_) * s.H + h) * Q;                                 \
            cs_raw = (cs2 + tb_)[(unsigned)tq];                                                            \
            f_raw = (fdec + tb_)[(unsigned)tq];                                                            \
            c_raw = (cdec + tb_)[(unsigned)tq];                                                            \
            dt_raw = (dt + tok0_ * s.H + h)[(unsigned)min(tq, valid_ - 1) * (unsigned)s.H];                \
        }
        // tables and the transposed tile of chunk c_ (held in set S_) -> buffer buf_
#define SWIMBA_P64_STAGE(S_, c_, buf_)                                                                     \
        {                                                                                                  \
            const int valid_ = min(Q, s.L - min((c_), s.nc - 1) * Q);                                      \
            if (pt < Q) {                                                                                  \
                lds_cs(buf_)[pt] = cs_raw;                                                                 \
                lds_dt(buf_)[pt] = (pt < valid_) ? to_float(bf16{dt_raw}) : 0.f;                           \
                lds_f(buf_)[pt] = f_raw;                                                                   \
                lds_c(buf_)[pt] = c_raw;                                                                   \
            }                                                                                              \
            _Pragma("unroll") for (int it = 0; it < XU; ++it) {                                            \
                const int u = pt + it * 256;                                                               \
                if (XU * 256 > UNITS && u >= UNITS) break;                                                 \
                const int p2 = u & 31, gi = u >> 5, t16 = gi >> 1, kgx = gi & 1;                           \
                const bool pok = 2 * p2 < s.P;                                                             \
                uint32_t r[8];                                                                             \
                _Pragma("unroll") for (int e = 0; e < 8; ++e) {                                            \
                    const int j = 16 * t16 + 8 * (e >> 2) + 4 * kgx + (e & 3);                             \
                    r[e] = (pok && j < valid_) ? xv##S_[it][e] : 0u;                                       \
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
                *reinterpret_cast<uint4 *>(lds_x(buf_) + (2 * p2) * XSTR + off) = lo;                      \
                *reinterpret_cast<uint4 *>(lds_x(buf_) + (2 * p2 + 1) * XSTR + off) = hi;                  \
            }                                                                                              \
        }
        // ---- running state: S^T[n = 32 sw + 8a + 4kg + b][p = l32 + 32 half] in register 4a + b of st[half] ----
        const int sw = wave - 4;
        f32x16_t st[2];
#pragma unroll
        for (int hf = 0; hf < 2; ++hf) {
            const int p = l32 + 32 * hf;
#pragma unroll
            for (int a = 0; a < 4; ++a) {
                const int n0 = 32 * sw + 8 * a + 4 * kg;
                float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
                if (h0 && p < s.P && n0 < s.N)
                    v = *reinterpret_cast<const float4 *>(h0 + (int64_t)p * s.N + n0);
                st[hf][4 * a + 0] = v.x; st[hf][4 * a + 1] = v.y; st[hf][4 * a + 2] = v.z; st[hf][4 * a + 3] = v.w;
            }
        }
        // the bf16 image of the state the compute waves read for the next chunk
#define SWIMBA_P64_PUT_STATE(buf_)                                                                         \
        _Pragma("unroll") for (int hf = 0; hf < 2; ++hf)                                                   \
        _Pragma("unroll") for (int a = 0; a < 4; ++a) {                                                    \
            const int n0 = 32 * sw + 8 * a + 4 * kg;                                                       \
            uint2 v;                                                                                       \
            v.x = pack_bf16x2(st[hf][4 * a + 0], st[hf][4 * a + 1]);                                       \
            v.y = pack_bf16x2(st[hf][4 * a + 2], st[hf][4 * a + 3]);                                       \
            *reinterpret_cast<uint2 *>(lds_h(buf_) + (l32 + 32 * hf) * HSTR + n0) = v;                     \
        }
        // mixed B rows of this wave's state rows, chunk c_ (operand of the state update): L2
        const unsigned bt_off = (unsigned)(kg * MN + sw * 32 + l32) * 8u;    // + ks * 2 * MN * 8
        uint4 bt[KS];
#define SWIMBA_P64_LOAD_BT(c_)                                                                             \
        {                                                                                                  \
            const uint16_t *bt_c = bt8 + (((int64_t)b * s.nc + min((c_), s.nc - 1)) * s.G + g) * ((Q / 8) * MN * 8); \
            _Pragma("unroll") for (int ks = 0; ks < KS; ++ks)                                              \
                bt[ks] = *reinterpret_cast<const uint4 *>(bt_c + bt_off + (unsigned)ks * (2 * MN * 8));    \
        }
        // H <- exp(cs_last) H + (Bmix^T * coef) . x for the chunk staged in buffer buf_, then its bf16 image
        // for the next chunk; the mixed B rows of the chunk after it are requested right behind.
        // k-step ks of lane group kg covers positions 16 ks + 8 kg + e = tokens 16 ks + 8 (e>>2) + 4 kg + (e&3).
#define SWIMBA_P64_STATE_UPDATE(c_, buf_)                                                                  \
        {                                                                                                  \
            const float dec = fast_exp2(lds_cs(buf_)[Q - 1]);                                              \
            _Pragma("unroll") for (int v = 0; v < 16; ++v) { st[0][v] *= dec; st[1][v] *= dec; }           \
            const uint16_t *sB0 = lds_x(buf_) + l32 * XSTR + 8 * kg;                                       \
            const uint16_t *sB1 = sB0 + 32 * XSTR;                                                         \
            const float *cj = lds_c(buf_) + 4 * kg;                                                        \
            _Pragma("unroll") for (int ks = 0; ks < KS; ++ks) {                                            \
                const float4 c0 = *reinterpret_cast<const float4 *>(cj + 16 * ks);                         \
                const float4 c1 = *reinterpret_cast<const float4 *>(cj + 16 * ks + 8);                     \
                float bv[8];                                                                               \
                unpack8(bv, bt[ks]);                                                                       \
                bv[0] *= c0.x; bv[1] *= c0.y; bv[2] *= c0.z; bv[3] *= c0.w;                                \
                bv[4] *= c1.x; bv[5] *= c1.y; bv[6] *= c1.z; bv[7] *= c1.w;                                \
                const uint4 ba = pack8(bv);                                                                \
                st[0] = mfma32(ba, *reinterpret_cast<const uint4 *>(sB0 + ks * 16), st[0]);                \
                st[1] = mfma32(ba, *reinterpret_cast<const uint4 *>(sB1 + ks * 16), st[1]);                \
            }                                                                                              \
            __builtin_amdgcn_sched_barrier(0);                                                             \
            SWIMBA_P64_LOAD_BT((c_) + 1);                                                                  \
            __builtin_amdgcn_sched_barrier(0);                                                             \
            SWIMBA_P64_PUT_STATE((buf_) ^ 1);                                                              \
        }
        SWIMBA_P64_PUT_STATE(0);
        {
            SWIMBA_P64_LANE_IDS();
            SWIMBA_P64_ISSUE(A, 0);
            SWIMBA_P64_ISSUE_TABLES(0);
            SWIMBA_P64_ISSUE(B, 1);
            SWIMBA_P64_LOAD_BT(0);
            SWIMBA_P64_STAGE(A, 0, 0);
            SWIMBA_P64_ISSUE_TABLES(1);
            SWIMBA_P64_ISSUE(A, 2);
        }
        // Iteration c updates the state with chunk c and stages chunk c+1 into the buffer nobody reads
        // during it (past the end: the last chunk once more, which nobody will read).  Even c: set B,
        // odd c: set A.
        for (int c = 0; c < s.nc; c += 2) {
            {
                SWIMBA_P64_LANE_IDS();
                lds_barrier();
                SWIMBA_P64_STATE_UPDATE(c, 0);
                SWIMBA_P64_STAGE(B, c + 1, 1);
                SWIMBA_P64_ISSUE_TABLES(c + 2);
                SWIMBA_P64_ISSUE(B, c + 3);
            }
            if (c + 1 < s.nc) {
                SWIMBA_P64_LANE_IDS();
                lds_barrier();
                SWIMBA_P64_STATE_UPDATE(c + 1, 1);
                SWIMBA_P64_STAGE(A, c + 2, 0);
                SWIMBA_P64_ISSUE_TABLES(c + 3);
                SWIMBA_P64_ISSUE(A, c + 4);
            }
        }
        lds_barrier();
        if (h_final) {
#pragma unroll
            for (int hf = 0; hf < 2; ++hf) {
                const int p = l32 + 32 * hf;
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const int n0 = 32 * sw + 8 * a + 4 * kg;
                    if (p < s.P && n0 < s.N)
                        *reinterpret_cast<float4 *>(h_final + (int64_t)p * s.N + n0) =
                            make_float4(st[hf][4 * a + 0], st[hf][4 * a + 1], st[hf][4 * a + 2], st[hf][4 * a + 3]);
                }
            }
        }
#undef SWIMBA_P64_PUT_STATE
#undef SWIMBA_P64_LOAD_BT
#undef SWIMBA_P64_STATE_UPDATE
#undef SWIMBA_P64_LANE_IDS
#undef SWIMBA_P64_ISSUE
#undef SWIMBA_P64_ISSUE_TABLES
#undef SWIMBA_P64_STAGE
        return;
    }

    // =============================== compute waves ===============================
    // channel held by operand row l32 of the Y^T contractions: accumulator row 8a + 4kg + b is then
    // channel 16kg + 4a + b of its 32-channel half, so a lane ends with 16 consecutive channels of one token
    const int prow = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);
    const int I0 = min(wave, NT - 1);                       // first output tile of the wave
    const int I1 = NT - 1 - wave;                           // second one (TPW == 2)
    const bool wave_on = wave < NT;                         // Q = 64: waves 2, 3 own no output tile
    const unsigned lane8_0 = (unsigned)lane * 8u;

    // Skip term as one more contraction of the diagonal tile: Y^T += x^T . (D I), with D split into
    // two bf16 terms.  B operand of k-step t: lane (column i = l32, kg) holds rows
    // j = 16t + 8(e>>2) + 4kg + (e&3); the entry is D where j == i.  Kept in LDS.
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
    constexpr int CBS = NQ < 3 ? NQ : 3;          // register slots of G^T tiles (three steps cover the L2 latency)
    constexpr int NQP = (NQ + CBS - 1) / CBS * CBS;   // steps per chunk padded to a multiple of CBS
    uint4 cfrag[8];           // mixed C rows of one output tile at a time
    uint4 cbt[CBS][2];
#define SWIMBA_P64_LOAD_C(c_, I_)                                                                          \
    {                                                                                                      \
        const uint16_t *cm_ = cmix + (((int64_t)b * s.nc + (c_)) * s.G + g) * (NT * 8 * 64 * 8);           \
        const unsigned o = (unsigned)(I_) * (8 * 64 * 8) + lane8;                                          \
        _Pragma("unroll") for (int ks = 0; ks < 8; ++ks)                                                   \
            cfrag[ks] = *reinterpret_cast<const uint4 *>(cm_ + o + ks * 64 * 8);                           \
    }
#define SWIMBA_P64_LOAD_CB(c_, q_)                                                                         \
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
        SWIMBA_P64_LOAD_C(0, I0);
#pragma unroll
        for (int q = 0; q < CBS; ++q) SWIMBA_P64_LOAD_CB(0, q);
    }

    for (int c = 0; c < s.nc; ++c) {
        const int buf = c & 1;
        const int cn = min(c + 1, s.nc - 1);               // next chunk (the last one asks for itself again)
        unsigned lane8 = lane8_0, prowx = (unsigned)prow;
        asm volatile("" : "+v"(lane8), "+v"(prowx));

        lds_barrier();          // chunk c is staged, the state image of chunk c is written
        const uint16_t *sX = lds_x(buf), *sH = lds_h(buf);
        const float *s_cs = lds_cs(buf), *s_dt = lds_dt(buf), *s_f = lds_f(buf);

        if (wave_on) {
            f32x16_t yt[TPW][2];
            float csi[TPW];
            const uint16_t *sHr = sH + prowx * HSTR + 64 * kg;
            // The decay table rows and the pivot of an off-diagonal step are read one step ahead of
            // it (those of step 0 here, behind the readout's contractions).
            float4 fpre[4];
            float rpre;
#define SWIMBA_P64_LOAD_F(J_)                                                                              \
    {                                                                                                      \
        const float *fj_ = s_f + (J_) * 32 + 4 * kg;                                                       \
        _Pragma("unroll") for (int a = 0; a < 4; ++a) fpre[a] = *reinterpret_cast<const float4 *>(fj_ + 8 * a); \
        rpre = s_cs[(J_) * 32 + 31];                                                                       \
    }
            SWIMBA_P64_LOAD_F(0);
            // ---- Y^T = exp(cs_i) H_c . Cmix^T for the first tile; the second tile's mixed C rows
            // ---- take the buffer's place and its readout follows half-way through the steps ----
            {
                f32x16_t a0 = {0}, a1 = {0};
#pragma unroll
                for (int ks = 0; ks < 8; ++ks) {
                    a0 = mfma32(*reinterpret_cast<const uint4 *>(sHr + ks * 8), cfrag[ks], a0);
                    a1 = mfma32(*reinterpret_cast<const uint4 *>(sHr + 32 * HSTR + ks * 8), cfrag[ks], a1);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (TPW == 2) SWIMBA_P64_LOAD_C(c, I1) else SWIMBA_P64_LOAD_C(cn, I0);
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int t = 0; t < TPW; ++t) csi[t] = s_cs[(t == 0 ? I0 : I1) * 32 + l32];
                const float sc = fast_exp2(csi[0]);
#pragma unroll
                for (int v = 0; v < 16; ++v) { yt[0][0][v] = sc * a0[v]; yt[0][1][v] = sc * a1[v]; }
                if (TPW == 2) {
#pragma unroll
                    for (int v = 0; v < 16; ++v) { yt[TPW - 1][0][v] = 0.f; yt[TPW - 1][1][v] = 0.f; }
                }
            }
            // ---- intra-chunk part ----
            const uint16_t *sXr = sX + prowx * XSTR + 8 * kg;     // operand rows of channel half 0 (+ 32 XSTR: half 1)
#pragma unroll
            for (int q = 0; q < NQP; ++q) {
                if (TPW == 2 && q == NQ / 2) {
                    f32x16_t a0 = {0}, a1 = {0};
#pragma unroll
                    for (int ks = 0; ks < 8; ++ks) {
                        a0 = mfma32(*reinterpret_cast<const uint4 *>(sHr + ks * 8), cfrag[ks], a0);
                        a1 = mfma32(*reinterpret_cast<const uint4 *>(sHr + 32 * HSTR + ks * 8), cfrag[ks], a1);
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    SWIMBA_P64_LOAD_C(cn, I0);
                    __builtin_amdgcn_sched_barrier(0);
                    const float sc = fast_exp2(csi[TPW - 1]);
#pragma unroll
                    for (int v = 0; v < 16; ++v) { yt[TPW - 1][0][v] += sc * a0[v]; yt[TPW - 1][1][v] += sc * a1[v]; }
                }
                const bool first = TPW == 1 || q <= wave;
                const int I = first ? I0 : I1;
                const int J = first ? q : q - wave - 1;
                const bool on = q < NQ && (TPW == 2 || q <= wave);
                const float ci = first ? csi[0] : csi[TPW - 1];
                if (on) {
                    // M^T = G^T tile times the decay and dt, rounded to bf16: the B operand of both halves
                    float m[16];
                    unpack8(m, cbt[q % CBS][0]);
                    unpack8(m + 8, cbt[q % CBS][1]);
                    if (J < I) {
                        // dt_j exp(R_J - cs_j) from the table, exp(cs_i - R_J) once per lane
                        const float ei = fast_exp2(ci - rpre);
#pragma unroll
                        for (int a = 0; a < 4; ++a) {
                            const float4 f4 = fpre[a];
                            m[4 * a + 0] *= ei * f4.x;
                            m[4 * a + 1] *= ei * f4.y;
                            m[4 * a + 2] *= ei * f4.z;
                            m[4 * a + 3] *= ei * f4.w;
                        }
                    } else {
                        // diagonal tile: direct masked form
                        const float *cj = s_cs + J * 32 + 4 * kg;
                        const float *dj = s_dt + J * 32 + 4 * kg;
                        // all eight table rows are requested before the first is used: one LDS round
                        // trip instead of four, and no read sunk under the lane mask of its select
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
                                // masked entries (j > i) get a hugely negative exponent: exp2 -> 0
                                const float arg = (l32 >= jl) ? ci - cc[bb] : -1.0e30f;
                                m[4 * a + bb] *= fast_exp2(arg) * dd[bb];
                            }
                        }
                    }
                    if (q + 1 < NQ) {
                        const int Jn = (TPW == 1 || q + 1 <= wave) ? q + 1 : q - wave;
                        SWIMBA_P64_LOAD_F(Jn);
                    }
                    const uint4 m0 = pack8(m), m1 = pack8(m + 8);
                    const uint4 x00 = *reinterpret_cast<const uint4 *>(sXr + J * 32);
                    const uint4 x01 = *reinterpret_cast<const uint4 *>(sXr + J * 32 + 16);
                    const uint4 x10 = *reinterpret_cast<const uint4 *>(sXr + 32 * XSTR + J * 32);
                    const uint4 x11 = *reinterpret_cast<const uint4 *>(sXr + 32 * XSTR + J * 32 + 16);
                    const bool diag = !(J < I) && has_D;
                    if (first) {
                        yt[0][0] = mfma32(x00, m0, yt[0][0]);
                        yt[0][1] = mfma32(x10, m0, yt[0][1]);
                        yt[0][0] = mfma32(x01, m1, yt[0][0]);
                        yt[0][1] = mfma32(x11, m1, yt[0][1]);
                        if (diag) {
#pragma unroll
                            for (int part = 0; part < 2; ++part) {
                                yt[0][0] = mfma32(x00, lds_id[(2 * part) * 64 + lane], yt[0][0]);
                                yt[0][1] = mfma32(x10, lds_id[(2 * part) * 64 + lane], yt[0][1]);
                                yt[0][0] = mfma32(x01, lds_id[(2 * part + 1) * 64 + lane], yt[0][0]);
                                yt[0][1] = mfma32(x11, lds_id[(2 * part + 1) * 64 + lane], yt[0][1]);
                            }
                        }
                    } else {
                        yt[TPW - 1][0] = mfma32(x00, m0, yt[TPW - 1][0]);
                        yt[TPW - 1][1] = mfma32(x10, m0, yt[TPW - 1][1]);
                        yt[TPW - 1][0] = mfma32(x01, m1, yt[TPW - 1][0]);
                        yt[TPW - 1][1] = mfma32(x11, m1, yt[TPW - 1][1]);
                        if (diag) {
#pragma unroll
                            for (int part = 0; part < 2; ++part) {
                                yt[TPW - 1][0] = mfma32(x00, lds_id[(2 * part) * 64 + lane], yt[TPW - 1][0]);
                                yt[TPW - 1][1] = mfma32(x10, lds_id[(2 * part) * 64 + lane], yt[TPW - 1][1]);
                                yt[TPW - 1][0] = mfma32(x01, lds_id[(2 * part + 1) * 64 + lane], yt[TPW - 1][0]);
                                yt[TPW - 1][1] = mfma32(x11, lds_id[(2 * part + 1) * 64 + lane], yt[TPW - 1][1]);
                            }
                        }
                    }
                }
                // the slot this step has just emptied takes the tile of step q + CBS (past the
                // chunk's last step: of the next chunk; padding steps have no tile)
                __builtin_amdgcn_sched_barrier(0);
                if (q + CBS < NQ) SWIMBA_P64_LOAD_CB(c, q + CBS)
                else if (q + CBS >= NQP && q + CBS - NQP < NQ) SWIMBA_P64_LOAD_CB(cn, q + CBS - NQP);
                __builtin_amdgcn_sched_barrier(0);
            }
            // ---- the output tiles: bf16 through the wave's own LDS scratch (piece index XOR-swizzled by
            // ---- the row), then out as whole 128-byte rows ----
            const int valid = min(Q, s.L - c * Q);
            uint16_t *scr = lds_y + wave * (32 * MP);
            uint16_t *yh = y + (((int64_t)b * s.L + (int64_t)c * Q) * s.H + h) * s.P;
#pragma unroll
            for (int t = 0; t < TPW; ++t) {
                const int I = (t == 0) ? I0 : I1;
                // lane -> (row, 16-byte piece) of the stores, from an opaque copy: eight row addresses kept
                // across the chunk loop would not fit the register budget
                int ln = lane;
                asm volatile("" : "+v"(ln));
                const int erow = ln >> 3, epiece = ln & 7;
                const int l32s = ln & 31, kgs = ln >> 5;
                {
                    float a0[16], a1[16];
#pragma unroll
                    for (int v = 0; v < 16; ++v) { a0[v] = yt[t][0][v]; a1[v] = yt[t][1][v]; }
                    uint16_t *dst = scr + l32s * MP;             // lane holds channels 16kg..16kg+15 (+32)
                    const int sw = l32s & 7;
                    *reinterpret_cast<uint4 *>(dst + (((2 * kgs) ^ sw) << 3)) = pack8(a0);
                    *reinterpret_cast<uint4 *>(dst + (((2 * kgs + 1) ^ sw) << 3)) = pack8(a0 + 8);
                    *reinterpret_cast<uint4 *>(dst + (((4 + 2 * kgs) ^ sw) << 3)) = pack8(a1);
                    *reinterpret_cast<uint4 *>(dst + (((5 + 2 * kgs) ^ sw) << 3)) = pack8(a1 + 8);
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
#pragma unroll
                for (int q4 = 0; q4 < 4; ++q4) {
                    const int row = erow + 8 * q4, i = I * 32 + row;
                    const uint4 v = *reinterpret_cast<const uint4 *>(scr + row * MP + ((epiece ^ (row & 7)) << 3));
                    if (i < valid && epiece * 8 < s.P)
                        store_nt(yh + (unsigned)i * (unsigned)tokstride + epiece * 8, v);
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
            }
        }
    }
    lds_barrier();              // pairs with the stage waves' last barrier
#undef SWIMBA_P64_LOAD_C
#undef SWIMBA_P64_LOAD_F
#undef SWIMBA_P64_LOAD_CB
}

// =========================================================================================
// States at the segment boundaries of a split pass.  The chunk-state kernel has left S_c (bf16,
// padded to 64 x 128) for the chunks in front of the last boundary that still count at the
// boundary behind them; this kernel walks the chunks of one (sequence, head) in order,
// h <- a_c h + S_c with a_c = exp2(cs2_c[Q-1]) and S_c = 0 for the chunks whose factor up to the
// boundary is below 2^SPLIT_KEEP_LOG2 (they are not read), and stores h at every boundary.
// Workgroup = (sequence, head, quarter of the state); a lane owns eight consecutive n of one channel.
// =========================================================================================
__global__ void __launch_bounds__(256)
boundary_states_kernel(const uint16_t *__restrict__ states_lp, const float *__restrict__ cs2,
                       const float *__restrict__ h0, float *__restrict__ hmid, Shape s, int nseg)
{
    // s is the shape of the segments: s.B = sequences * nseg, s.nc = chunks per segment
    __shared__ float s_tot[PASS_SPLIT_MAX_CHUNKS];
    __shared__ int s_first;
    const int part = blockIdx.x & 3;
    const int h = (blockIdx.x >> 2) % s.H;
    const int seq = (blockIdx.x >> 2) / s.H;
    const int e = (part * 256 + threadIdx.x) * 8;        // element of the padded 64 x 128 state
    const int p = e / MN, n0 = e % MN;
    const bool inside = p < s.P && n0 < s.N;             // N is a multiple of 8
    float hv[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    if (h0 && inside) {
        const float *src = h0 + (((int64_t)seq * s.H + h) * s.P + p) * s.N + n0;
        const float4 v0 = *reinterpret_cast<const float4 *>(src), v1 = *reinterpret_cast<const float4 *>(src + 4);
        hv[0] = v0.x; hv[1] = v0.y; hv[2] = v0.z; hv[3] = v0.w; hv[4] = v1.x; hv[5] = v1.y; hv[6] = v1.z; hv[7] = v1.w;
    }
    for (int seg = 0; seg + 1 < nseg; ++seg) {
        const int b = seq * nseg + seg;
        const float *tot = cs2 + (((int64_t)b * s.nc) * s.H + h) * s.Q + (s.Q - 1);      // + c * H * Q
        __syncthreads();                                  // the previous segment's totals are no longer read
        for (int c = threadIdx.x; c < s.nc; c += 256) s_tot[c] = tot[(int64_t)c * s.H * s.Q];
        __syncthreads();
        if (threadIdx.x == 0) {
            // first chunk of the segment that still counts at the boundary
            int first = s.nc - 1;
            float suf = 0.f;
            while (first > 0) {
                suf += s_tot[first];
                if (suf < SPLIT_KEEP_LOG2) break;
                --first;
            }
            s_first = first;
        }
        __syncthreads();
        const int first = s_first;
        {
            // the chunks in front of it only decay what is carried in
            float a = 0.f;
            for (int c = 0; c < first; ++c) a += s_tot[c];
            a = fast_exp2(a);
#pragma unroll
            for (int v = 0; v < 8; ++v) hv[v] *= a;
        }
        const uint16_t *src = states_lp + (((int64_t)b * s.nc) * s.H + h) * (MP * MN) + e;   // + c * H * MP * MN
        constexpr int AHEAD = 16;                         // chunk states requested together
        for (int c0 = first; c0 < s.nc; c0 += AHEAD) {
            uint4 sv[AHEAD];
#pragma unroll
            for (int u = 0; u < AHEAD; ++u)
                sv[u] = *reinterpret_cast<const uint4 *>(src + (int64_t)min(c0 + u, s.nc - 1) * s.H * (MP * MN));
#pragma unroll
            for (int u = 0; u < AHEAD; ++u) {
                if (c0 + u < s.nc) {
                    const float a = fast_exp2(s_tot[c0 + u]);
                    float f[8];
                    unpack8(f, sv[u]);
#pragma unroll
                    for (int v = 0; v < 8; ++v) hv[v] = a * hv[v] + f[v];
                }
            }
        }
        if (inside) {
            float *dst = hmid + ((((int64_t)seq * (nseg - 1) + seg) * s.H + h) * s.P + p) * s.N + n0;
            *reinterpret_cast<float4 *>(dst) = make_float4(hv[0], hv[1], hv[2], hv[3]);
            *reinterpret_cast<float4 *>(dst + 4) = make_float4(hv[4], hv[5], hv[6], hv[7]);
        }
    }
}

// the shape of the nseg equal segments of whole chunks a sequence splits into
static bool segment_shape(const Shape &s, int nseg, Shape *sv)
{
    *sv = s;
    if (nseg == 1) return true;
    if (nseg < 1 || nseg > PASS_SPLIT_MAX_SEGMENTS || s.nc % nseg != 0 || (int64_t)s.nc * s.Q != s.L ||
        s.nc / nseg > PASS_SPLIT_MAX_CHUNKS)
        return false;
    sv->B = s.B * nseg; sv->L = s.L / nseg; sv->nc = s.nc / nseg;
    return true;
}

// chunk states in front of the boundaries (those that still count there), then the boundary states
swimba_status launch_boundary_states_mfma(const Shape &s, int nseg, const void *x, const void *dt, const float *A,
                                          const void *bt8, const float *cs2, void *states_lp, const float *h0,
                                          float *hmid, hipStream_t st)
{
    Shape sv;
    if (nseg < 2 || !segment_shape(s, nseg, &sv)) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)s.B * s.H == 0 || s.nc == 0) return SWIMBA_OK;
    swimba_status rc = launch_chunk_state_mfma(sv, x, dt, A, bt8, nullptr, states_lp, st, 1, nullptr, nullptr, nullptr,
                                               nseg, cs2);
    if (rc != SWIMBA_OK) return rc;
    hipLaunchKernelGGL(boundary_states_kernel, dim3((unsigned)((int64_t)s.B * s.H * 4)), dim3(256), 0, st,
                       (const uint16_t *)states_lp, cs2, h0, hmid, sv, nseg);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

template <int Q>
static swimba_status launch_pass64_q(const Shape &s, const void *x, const void *dt, const float *D, const void *cmix,
                                     const void *bt8, const void *cb, const float *cs2, const float *fdec,
                                     const float *cdec, const float *h0, float *h_final, void *y, hipStream_t st,
                                     int nseg, const float *hmid)
{
    const int64_t total = (int64_t)s.B * s.H;
    if (total == 0 || s.nc == 0) return SWIMBA_OK;
    const int nblocks = xcd_padded(total);
    const size_t shm = Pass64Lds<Q>::BYTES;
    // more than 64 KB of dynamic LDS has to be allowed once per device
    static std::atomic<uint64_t> attr_set{0};            // one bit per device ordinal
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
    const uint64_t bit = 1ull << (dev & 63);
    if (!(attr_set.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute((const void *)pass64_kernel<Q>, hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
        attr_set.fetch_or(bit, std::memory_order_release);
    }
    hipLaunchKernelGGL(pass64_kernel<Q>, dim3(nblocks), dim3(PASS64_THREADS), shm, st, (const uint16_t *)x,
                       (const uint16_t *)dt, D, (const uint16_t *)cmix, (const uint16_t *)bt8, (const uint16_t *)cb,
                       cs2, fdec, cdec, h0, h_final, (uint16_t *)y, s, (int)total, nblocks, nseg, hmid);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_pass64_mfma(const Shape &s, const void *x, const void *dt, const float *D, const void *cmix,
                                 const void *bt8, const void *cb, const float *cs2, const float *fdec,
                                 const float *cdec, const float *h0, float *h_final, void *y, hipStream_t st,
                                 int nseg, const float *hmid)
{
    // nseg > 1: every sequence as nseg chains of its own, each from the boundary state in hmid
    Shape sv;
    if (!segment_shape(s, nseg, &sv) || (nseg > 1 && !hmid)) return SWIMBA_ERR_UNSUPPORTED;
    switch (s.Q) {
    case 64: return launch_pass64_q<64>(sv, x, dt, D, cmix, bt8, cb, cs2, fdec, cdec, h0, h_final, y, st, nseg, hmid);
    case 128: return launch_pass64_q<128>(sv, x, dt, D, cmix, bt8, cb, cs2, fdec, cdec, h0, h_final, y, st, nseg, hmid);
    case 256: return launch_pass64_q<256>(sv, x, dt, D, cmix, bt8, cb, cs2, fdec, cdec, h0, h_final, y, st, nseg, hmid);
    }
    return SWIMBA_ERR_UNSUPPORTED;
}

}  // namespace swimba
