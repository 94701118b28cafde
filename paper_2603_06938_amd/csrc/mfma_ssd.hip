// bf16 MFMA SSD chunk kernels for P = 64, N = 128 (smaller P and N, multiples of 8, run zero-padded: x is
// staged with zero channels, the mixed expert rows get zero columns), Q in {64, 128, 256}
// (paper, background section on SSD: matrix multiplications inside chunks;
// Theorem 1: the mixed streams feed one plain SSM).
//
// Four kernels:
//   mix_rows     per (batch, chunk, group, 32-token tile): routes the tile's tokens,
//                gathers their k active expert rows, mixes them with the router weights
//                in fp32 and writes, in bf16 and in the register layout of the MFMA
//                operands that consume them, the mixed C rows, the mixed B rows, and
//                the mixed B rows transposed in groups of 8 tokens.  Shared by all
//                heads of the group.
//   scan_cb      the inter-chunk scan of the states; the same launch also computes the
//                causal 32x32 tiles of G^T = Bmix . Cmix^T from the mixed rows.
//   chunk_state  per (batch, chunk, head): S = (coef * x)^T . Bmix
//   output       per (batch, chunk, head): y = (decay-masked G) (dt x) + exp(cs) Cmix . H + D x
//
// MFMA used: v_mfma_f32_32x32x16_bf16.  Lane l of a wave holds
//   A[row = l%32][k = 8*(l/32) + 0..7],  B[k = 8*(l/32) + 0..7][col = l%32],
//   C[row = 8*(v/4) + 4*(l/32) + v%4][col = l%32] in accumulator register v.
// The k index of a contraction may be permuted freely as long as A and B use
// the same permutation; this is used to read 16 contiguous bytes per operand.
#include "common.hpp"
#include "mfma_util.hpp"

#include <atomic>

namespace swimba {

// Mixed row of one token for MFMA use: lane (row, kg) gets, for ks = 0..7, the 8
// values n = 64*kg + 8*ks + 0..7 of  sum_r w_r * S[e_r][g][n]  as packed bf16.
// `tok` points at S[token][0][g][0]; estride = G*N elements between experts.
// idx / w may live in LDS.  All loads are unconditional (callers clamp the token and
// pass zero weights for tokens past the end of the sequence).
__device__ __forceinline__ void gather_mix_row(uint4 *frag, const uint16_t *tok, int estride,
                                               const int32_t *idx, const float *w, int K, int kg)
{
    float acc[8][8];
#pragma unroll
    for (int ks = 0; ks < 8; ++ks)
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[ks][e] = 0.f;
#pragma unroll 2
    for (int r = 0; r < K; ++r) {
        const uint16_t *row = tok + idx[r] * estride + 64 * kg;
        const float wr = w[r];
        uint4 v[8];
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) v[ks] = *reinterpret_cast<const uint4 *>(row + ks * 8);
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) fma_bf16x8(acc[ks], v[ks], wr);
    }
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) frag[ks] = pack8(acc[ks]);
}

// =========================================================================================
// mix_rows.  Workgroup = (batch, chunk, group, 32-token tile).  Lanes 0..31 route the
// tile's tokens (softmax over all experts, top-k on the raw logits, no renormalisation)
// into LDS and store the routing to topk_idx / topk_w; then wave 0 mixes the C rows,
// wave 1 the B rows (both as MFMA operand registers) and waves 2, 3 the B rows again in
// the token-innermost layout the chunk-state kernel contracts over.  With sep_e >= 0 it
// prepares the streams of ONE expert for the separated-SSM contrast instead:
// Bmix = B^(e), Cmix = gate * C^(e), gate = pi_{t,e} if e is in the active set, else 0.
// With slot >= 0 (one input stream per expert) Bmix keeps only the term of the token's
// slot-th active expert, Bmix = pi_{t,e_slot} B^(e_slot); Cmix is the full mix.  With
// slot == MIX_ALL_SLOTS every slot's term is written, image r of bfrag / bmix_t8 (each
// B*nc*G*Q*MN elements) holding pi_{t,e_r} B^(e_r); the summed B mix is not formed.
//   cmix, bfrag (B, nc, G, NT, 8, 64, 8) bf16, mixed rows of tile I as operand registers:
//           [ks][lane][e] = mix[32I + lane%32][64*(lane/32) + 8ks + e]
//   bmix_t8 (B, nc, G, Q/8, N, 8)    bf16, mixed B with 8 tokens innermost: position 8 o + e of a
//           chunk holds token t8_token(8 o + e) (tokens 4..7 and 8..11 of every 16 swapped), the
//           order in which an accumulator tile hands its rows to the next contraction
// =========================================================================================
__global__ void __launch_bounds__(MTHREADS)
mix_rows_kernel(const uint16_t *__restrict__ Be, const uint16_t *__restrict__ Ce,
                const uint16_t *__restrict__ logits, int32_t *__restrict__ idx_out,
                float *__restrict__ w_out, uint16_t *__restrict__ cmix, uint16_t *__restrict__ bfrag,
                uint16_t *__restrict__ bmix_t8, Shape s, int sep_e, int slot,
                const float *__restrict__ w_sel)
{
    extern __shared__ __align__(16) unsigned char smem_raw[];
    const int Kr = s.K;                                             // experts kept by the router
    int32_t *s_idx = reinterpret_cast<int32_t *>(smem_raw);        // [32][K]
    float *s_w = reinterpret_cast<float *>(s_idx + 32 * Kr);        // [32][K]
    // separated-SSM contrast (sep_e >= 0): expert sep_e alone, B unweighted, C gated
    int32_t *s_idx1 = reinterpret_cast<int32_t *>(s_w + 32 * Kr);   // [32]
    float *s_wb1 = reinterpret_cast<float *>(s_idx1 + 32);          // [32]
    float *s_wc1 = s_wb1 + 32;                                      // [32]
    constexpr int MIXROW = MN + 8;                                  // bf16 elements per padded row
    uint16_t *s_mix = reinterpret_cast<uint16_t *>(s_wc1 + 32);     // [2][32][MIXROW], 16-byte aligned
    float *s_log = reinterpret_cast<float *>(s_mix + 2 * 32 * MIXROW);   // [32][E + 1]
    // expert-specific input streams (slot >= 0): B keeps the weight of active expert `slot` only
    float *s_wslot = s_log + 32 * (s.E + 1);                             // [32][K]
    // every slot's weighted B row on its own (slot == MIX_ALL_SLOTS): [K][32][MIXROW]
    uint16_t *s_slots = reinterpret_cast<uint16_t *>(s_wslot + 32 * Kr);
    const bool all_slots = (slot == MIX_ALL_SLOTS);

    const int NT = s.Q / 32;
    const int tile = blockIdx.x % NT;
    const int g = (blockIdx.x / NT) % s.G;
    const int c = (blockIdx.x / (NT * s.G)) % s.nc;
    const int b = blockIdx.x / (NT * s.G * s.nc);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kg = lane >> 5;
    const int valid = min(s.Q, s.L - c * s.Q) - tile * 32;     // tokens of this tile inside the sequence
    const int64_t tok0 = (int64_t)b * s.L + (int64_t)c * s.Q + tile * 32;
    const int64_t last = (int64_t)b * s.L + min(s.L, (c + 1) * s.Q) - 1 - tok0;   // clamp for padded rows
    const int estride = s.G * s.N;                       // rows of the inputs have the caller's N <= MN
    // Streams of the selected experts only (w_sel != nullptr): Be / Ce are (B,L,k,G,N), row r of
    // a token belongs to its r-th selected expert and w_sel (B,L,k) holds the router weights.
    const bool sel = (w_sel != nullptr);
    const int rowsE = sel ? Kr : s.E;
    const int tokstride = rowsE * estride;               // elements between tokens of B/C_experts
    const int64_t bcg = ((int64_t)b * s.nc + c) * s.G + g;
    const uint16_t *Bg = Be + (tok0 * rowsE * s.G + g) * s.N;  // [token 0 of the tile][expert 0][g][0]
    const uint16_t *Cg = Ce + (tok0 * rowsE * s.G + g) * s.N;

    // ---- routing of the tile's tokens: logits staged through LDS (one coalesced read) ----
    // separated-SSM contrast: the pass of expert 0 routes and stores the routing, the passes of the
    // other experts read it back instead of repeating softmax and top-k E times per token
    const bool reuse = sep_e > 0;
    if (!sel && !reuse) {
        const int nlog = max(0, min(valid, 32)) * s.E;
        const uint16_t *gl = logits + tok0 * s.E;
        for (int i = tid; i < nlog; i += MTHREADS) s_log[(i / s.E) * (s.E + 1) + i % s.E] = to_float(bf16{gl[i]});
    }
    lds_barrier();
    if (tid < 32) {
        const int t = tid;
        if (sel) {
            for (int rr = 0; rr < Kr; ++rr) {
                s_idx[t * Kr + rr] = rr;
                s_w[t * Kr + rr] = (t < valid) ? w_sel[(tok0 + t) * Kr + rr] : 0.f;
            }
        } else if (t < valid && reuse) {
            for (int rr = 0; rr < Kr; ++rr) {
                s_idx[t * Kr + rr] = idx_out[(tok0 + t) * Kr + rr];
                s_w[t * Kr + rr] = w_out[(tok0 + t) * Kr + rr];
            }
        } else if (t < valid) {
            const float *gl = s_log + t * (s.E + 1);
            route_token([&](int e) { return gl[e]; }, s.E, Kr, s_idx + t * Kr, s_w + t * Kr);
            if (g == 0 && sep_e <= 0 && slot <= 0) {
                for (int rr = 0; rr < Kr; ++rr) {
                    idx_out[(tok0 + t) * Kr + rr] = s_idx[t * Kr + rr];
                    w_out[(tok0 + t) * Kr + rr] = s_w[t * Kr + rr];
                }
            }
        } else {
            for (int rr = 0; rr < Kr; ++rr) { s_idx[t * Kr + rr] = 0; s_w[t * Kr + rr] = 0.f; }
        }
        if (slot >= 0)
            for (int rr = 0; rr < Kr; ++rr) s_wslot[t * Kr + rr] = (rr == slot) ? s_w[t * Kr + rr] : 0.f;
        if (sep_e >= 0) {
            // MoE of separated SSMs (paper: separated-SSM equation): expert sep_e keeps its own
            // state, B_t^(e) enters unweighted, the readout weight is pi_{t,e} on the active set
            float gate = 0.f;
            for (int rr = 0; rr < Kr; ++rr)
                if (s_idx[t * Kr + rr] == sep_e) gate += s_w[t * Kr + rr];
            s_idx1[t] = sep_e;
            s_wb1[t] = (t < valid) ? 1.f : 0.f;
            s_wc1[t] = (t < valid) ? gate : 0.f;
        }
    }
    lds_barrier();
    // tables the gathers read: K experts per token, separate weights for the B and C streams
    const int K = (sep_e >= 0) ? 1 : Kr;
    const int32_t *ixt = (sep_e >= 0) ? s_idx1 : s_idx;
    const float *wtB = (sep_e >= 0) ? s_wb1 : (slot >= 0) ? s_wslot : s_w;
    const float *wtC = (sep_e >= 0) ? s_wc1 : s_w;

    // ---- gather and mix: a lane owns one 16-byte piece (8 n) of tokens tg and tg+16, both
    // streams; 16 consecutive lanes read one whole 256-byte expert row.  Experts two at a time.
    const int piece = tid & 15, tg = tid >> 4;
    const bool pin = piece * 8 < s.N;                    // pieces past the caller's N stay zero (padding)
    const int pc = pin ? piece : 0;
    float accB[2][8], accC[2][8];
#pragma unroll
    for (int jj = 0; jj < 2; ++jj)
#pragma unroll
        for (int e = 0; e < 8; ++e) accB[jj][e] = accC[jj][e] = 0.f;
    for (int r0 = 0; r0 < K; r0 += 2) {
        uint4 vb[2][2], vc[2][2];
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int j = tg + 16 * jj;
            const int64_t rowoff = min((int64_t)j, last) * tokstride + pc * 8;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const int eo = ixt[j * K + min(r0 + q, K - 1)] * estride;
                vb[jj][q] = *reinterpret_cast<const uint4 *>(Bg + rowoff + eo);
                vc[jj][q] = *reinterpret_cast<const uint4 *>(Cg + rowoff + eo);
            }
        }
#pragma unroll
        for (int jj = 0; jj < 2; ++jj) {
            const int j = tg + 16 * jj;
#pragma unroll
            for (int q = 0; q < 2; ++q) {
                const bool on = pin && r0 + q < K;
                if (all_slots) {
                    if (r0 + q < K) {
                        float one[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                        fma_bf16x8(one, vb[jj][q], on ? wtB[j * K + r0 + q] : 0.f);
                        *reinterpret_cast<uint4 *>(s_slots + ((r0 + q) * 32 + j) * MIXROW + piece * 8) = pack8(one);
                    }
                } else {
                    fma_bf16x8(accB[jj], vb[jj][q], on ? wtB[j * K + r0 + q] : 0.f);
                }
                fma_bf16x8(accC[jj], vc[jj][q], on ? wtC[j * K + r0 + q] : 0.f);
            }
        }
    }
    // mixed tiles, row-major bf16 with padded rows: [stream][32][MIXROW]
#pragma unroll
    for (int jj = 0; jj < 2; ++jj) {
        const int j = tg + 16 * jj;
        *reinterpret_cast<uint4 *>(s_mix + j * MIXROW + piece * 8) = pack8(accB[jj]);
        *reinterpret_cast<uint4 *>(s_mix + (32 + j) * MIXROW + piece * 8) = pack8(accC[jj]);
    }
    lds_barrier();

    const int nimg = all_slots ? Kr : 1;                 // B images written by this launch
    const int64_t img = (int64_t)s.B * s.nc * s.G * s.Q * MN;   // elements per image
    if (wave == 0) {
        // operand registers: lane (l32, kg) holds n = 64 kg + 8 ks .. + 7 of token l32
        const uint16_t *src = s_mix + (32 + l32) * MIXROW + 64 * kg;
        uint16_t *dst = cmix + (((bcg * NT + tile) * 8) * 64 + lane) * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks)
            *reinterpret_cast<uint4 *>(dst + ks * 64 * 8) = *reinterpret_cast<const uint4 *>(src + ks * 8);
    } else if (wave == 1) {
        for (int r = 0; r < nimg; ++r) {
            const uint16_t *src = (all_slots ? s_slots + r * 32 * MIXROW : s_mix) + l32 * MIXROW + 64 * kg;
            uint16_t *dst = bfrag + r * img + (((bcg * NT + tile) * 8) * 64 + lane) * 8;
#pragma unroll
            for (int ks = 0; ks < 8; ++ks)
                *reinterpret_cast<uint4 *>(dst + ks * 64 * 8) = *reinterpret_cast<const uint4 *>(src + ks * 8);
        }
    } else {
        // mixed B, 8 tokens innermost (in the operand order of t8_token): lane = state index n,
        // one 16-byte store per token octet
        const int n = tid - 128;
        for (int r = 0; r < nimg; ++r) {
            const uint16_t *src = all_slots ? s_slots + r * 32 * MIXROW : s_mix;
#pragma unroll
            for (int jgl = 0; jgl < 4; ++jgl) {
                uint32_t pk[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const uint32_t lo = src[t8_token(jgl * 8 + 2 * q) * MIXROW + n];
                    const uint32_t hi = src[t8_token(jgl * 8 + 2 * q + 1) * MIXROW + n];
                    pk[q] = lo | (hi << 16);
                }
                *reinterpret_cast<uint4 *>(bmix_t8 + r * img + ((bcg * (s.Q / 8) + tile * 4 + jgl) * MN + n) * 8) =
                    make_uint4(pk[0], pk[1], pk[2], pk[3]);
            }
        }
    }
}

// =========================================================================================
// Inter-chunk scan over bf16 chunk states, H_0 = h0, H_{c+1} = exp(cs_c[Q-1]) H_c + S_c,
// states[c] <- H_c in place: the running state is fp32 in registers, 8 state elements per
// lane, the loads of 4 chunks in flight.  The first ncb workgroups of the launch do
// not scan: each of their waves computes one cb tile (see cb_pair), work that only
// depends on the mixed rows and is needed by the output kernel alone, so it rides in
// this launch instead of paying for one of its own.
// With nslots > 1 (one input stream per expert) the chunk states of the slots, images of
// B*nc*H*MP*MN elements behind each other in lp, are summed in fp32 on the way (the state is
// linear in the injection) and the carried states land in image 0; the tiles are computed
// per slot from the slot's B image (cb image r behind image r - 1).  NS >= nslots is the
// number of slot loads kept in flight per chunk.
// =========================================================================================
template <int NS>
__global__ void __launch_bounds__(MTHREADS)
scan_cb_kernel(uint16_t *__restrict__ lp, const float *__restrict__ h0, float *__restrict__ h_final,
               const float *__restrict__ cs, const uint16_t *__restrict__ cmix,
               const uint16_t *__restrict__ bfrag, uint16_t *__restrict__ cb, Shape s, int ncb, int64_t nbcg,
               int nslots)
{
    if ((int)blockIdx.x < ncb) {
        const int NT = s.Q / 32, NPAIR = NT * (NT + 1) / 2, PB = (NPAIR + 3) / 4;
        // consecutive logical ids (the pairs of one (batch, chunk, group)) share an XCD and its L2
        const int64_t id = xcd_logical_id(blockIdx.x, ncb);
        const int64_t sbcg = id / PB;                    // (slot, batch, chunk, group)
        const int64_t bcg = sbcg % nbcg;
        const int slot = (int)(sbcg / nbcg);
        const int p = (int)(id % PB) * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        if (slot < nslots && p < NPAIR)
            cb_pair(cmix, bfrag + slot * (nbcg * s.Q * MN), cb + slot * (nbcg * NPAIR * 1024), NT, bcg, p,
                    threadIdx.x & 63);
        return;
    }
    // chunk states are (MP, MN) tiles; h0 / h_final have the caller's P <= MP rows and N <= MN columns
    // (the padding of the states is zero: the mixed B rows and the staged x are zero there)
    constexpr int64_t per_bh = (int64_t)MP * MN / 8;
    const int64_t gid = (int64_t)(blockIdx.x - ncb) * blockDim.x + threadIdx.x;
    if (gid >= per_bh * s.B * s.H) return;
    const int64_t bh = gid / per_bh;
    const int64_t pn = (gid % per_bh) * 8;
    const int b = (int)(bh / s.H), h = (int)(bh % s.H);
    constexpr int64_t PN = (int64_t)MP * MN;
    const int pp = (int)(pn / MN), nn = (int)(pn % MN);
    const bool real = nn < s.N && pp < s.P;              // 8 consecutive columns: all real or all padding
    const int64_t user = (bh * s.P + pp) * s.N + nn;

    float run[8];
#pragma unroll
    for (int v = 0; v < 8; ++v) run[v] = (h0 && real) ? h0[user + v] : 0.f;

    constexpr int UN = (NS > 2) ? 2 : 4;  // chunks whose loads are issued together
    const int64_t simg = (int64_t)s.B * s.nc * s.H * PN;   // elements per slot image
    for (int c0 = 0; c0 < s.nc; c0 += UN) {
        uint4 S[UN][NS];
        float decay[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int c = min(c0 + u, s.nc - 1);
#pragma unroll
            for (int r = 0; r < NS; ++r)
                S[u][r] = *reinterpret_cast<const uint4 *>(lp + min(r, nslots - 1) * simg +
                                                           (((int64_t)b * s.nc + c) * s.H + h) * PN + pn);
            decay[u] = fast_exp2(cs[(((int64_t)b * s.nc + c) * s.H + h) * s.Q + s.Q - 1] * LOG2E);
        }
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int c = c0 + u;
            if (c < s.nc) {
                *reinterpret_cast<uint4 *>(lp + (((int64_t)b * s.nc + c) * s.H + h) * PN + pn) = pack8(run);
                float sv[8];
                unpack8(sv, S[u][0]);
#pragma unroll
                for (int r = 1; r < NS; ++r) {
                    float sr[8];
                    unpack8(sr, S[u][r]);
                    if (r < nslots) {
#pragma unroll
                        for (int v = 0; v < 8; ++v) sv[v] += sr[v];
                    }
                }
#pragma unroll
                for (int v = 0; v < 8; ++v) run[v] = decay[u] * run[v] + sv[v];
            }
        }
    }
    if (h_final && real) {
#pragma unroll
        for (int v = 0; v < 8; ++v) h_final[user + v] = run[v];
    }
}

swimba_status launch_mix_rows_mfma(const Shape &s, const void *Be, const void *Ce, const void *logits,
                                   int32_t *idx, float *w, void *cmix, void *bfrag, void *bmix_t8,
                                   int sep_e, int slot, const float *w_sel, hipStream_t st)
{
    const int NT = s.Q / 32;
    const int64_t nbcg = (int64_t)s.B * s.nc * s.G;
    if (nbcg == 0) return SWIMBA_OK;
    if (w_sel && (sep_e >= 0 || slot >= 0)) return SWIMBA_ERR_UNSUPPORTED;
    if (slot == MIX_ALL_SLOTS && (sep_e >= 0 || s.K > MIX_ALL_SLOTS_MAX)) return SWIMBA_ERR_UNSUPPORTED;
    const size_t shm = (size_t)32 * s.K * 8 + 32 * 12 + (size_t)2 * 32 * (MN + 8) * 2 + (size_t)32 * (s.E + 1) * 4
                       + (size_t)32 * s.K * 4 + (slot == MIX_ALL_SLOTS ? (size_t)s.K * 32 * (MN + 8) * 2 : 0);
    hipLaunchKernelGGL(mix_rows_kernel, dim3((unsigned)(nbcg * NT)), dim3(MTHREADS), shm, st,
                       (const uint16_t *)Be, (const uint16_t *)Ce, (const uint16_t *)logits, idx, w,
                       (uint16_t *)cmix, (uint16_t *)bfrag, (uint16_t *)bmix_t8, s, sep_e, slot, w_sel);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_scan_cb_mfma(const Shape &s, const float *h0, float *h_final, void *states_lp,
                                  const float *cs, const void *cmix, const void *bfrag, void *cb,
                                  hipStream_t st, int nslots)
{
    const int64_t elems = (int64_t)s.B * s.H * MP * MN;
    const int64_t nbcg = (int64_t)s.B * s.nc * s.G;
    if (elems == 0) return SWIMBA_OK;
    if (nslots < 1 || nslots > MIX_ALL_SLOTS_MAX) return SWIMBA_ERR_UNSUPPORTED;
    const int NT = s.Q / 32;
    const int ncb = xcd_padded(nslots * nbcg * ((NT * (NT + 1) / 2 + 3) / 4));   // 0 for an empty sequence
    const unsigned grid = (unsigned)(ncb + (elems / 8 + MTHREADS - 1) / MTHREADS);
#define SWIMBA_SCAN_LAUNCH(NS)                                                                                    \
    hipLaunchKernelGGL(scan_cb_kernel<NS>, dim3(grid), dim3(MTHREADS), 0, st, (uint16_t *)states_lp, h0, h_final, \
                       cs, (const uint16_t *)cmix, (const uint16_t *)bfrag, (uint16_t *)cb, s, ncb, nbcg, nslots)
    if (nslots == 1) SWIMBA_SCAN_LAUNCH(1);
    else if (nslots == 2) SWIMBA_SCAN_LAUNCH(2);
    else SWIMBA_SCAN_LAUNCH(4);
#undef SWIMBA_SCAN_LAUNCH
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

// =========================================================================================
// Chunk state:  S_c[p][n] = sum_j coef_j x[j][p] Bmix[j][n],  coef_j = dt_j exp(cs_last - cs_j)
// Workgroup = (batch, chunk, group, run of heads of that group).  The mixed B operand
// (shared by the group's heads) is read once from bmix_t8 into registers.  The heads
// are walked in a software pipeline: while the MFMAs and the state stores of head k
// run, the x rows of head k+1 are already in flight, and they are staged into the other
// half of a double-buffered LDS tile.  (Loads two heads ahead, in a second register set,
// measured slower: 24.9 us against 22.6 us on the 130M-shaped workload.)
// Per head the kernel also computes the chunk's inclusive cumsum cs of dt*A (block
// scan) and stores it for the scan and output kernels.
// The coefficient-weighted x tile is staged transposed ([p][j]); wave w owns columns
// n = 32w..32w+31 and both 32-channel halves of p.  The chunk state is stored in bf16.
// With nslots > 1 (one input stream per expert) the grid carries the slot as its slowest
// index: slot r reads x rows r*H*P elements into a token (xts elements between tokens), the
// r-th mixed-B image, and writes the r-th chunk-state image; the scan sums the images.
// =========================================================================================
template <int Q>
__global__ void __launch_bounds__(MTHREADS, 2)   // two waves per SIMD: 256 registers, two workgroups per compute unit
chunk_state_mfma_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dt,
                        const float *__restrict__ A, const uint16_t *__restrict__ bmix_t8,
                        float *__restrict__ cs, uint16_t *__restrict__ states_lp, Shape s, int ipw,
                        int nruns, int total, int nblocks, int xts, int nslots, int ncb,
                        const uint16_t *__restrict__ cmix, const uint16_t *__restrict__ bmix_frag,
                        uint16_t *__restrict__ cb, int nseg, const float *__restrict__ cs2)
{
    if ((int)blockIdx.x < ncb) {
        // The first ncb workgroups compute the causal G^T tiles instead (one wave per tile pair, see
        // cb_pair): on short sequences, where the output kernel carries the states forward itself and
        // no scan launch exists for them to ride in, they ride here.
        const int NT = Q / 32, NPAIR = NT * (NT + 1) / 2, PB = (NPAIR + 3) / 4;
        const int64_t id = xcd_logical_id(blockIdx.x, ncb);
        const int64_t bcg = id / PB;
        const int p = (int)(id % PB) * 4 + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
        if (bcg < (int64_t)s.B * s.nc * s.G && p < NPAIR) cb_pair(cmix, bmix_frag, cb, NT, bcg, p, threadIdx.x & 63);
        return;
    }
    constexpr int STR = Q + 8;                    // row stride of the transposed x tile (elements)
    constexpr int KS = Q / 16;
    constexpr int XU = (Q / 8) * 32 / MTHREADS;   // x staging units per lane
    constexpr int LASTW = (Q - 1) / 64;
    extern __shared__ __align__(16) unsigned char smem_raw[];
    uint16_t *sXt = reinterpret_cast<uint16_t *>(smem_raw);                  // [2][MP][STR]
    float *s_coef = reinterpret_cast<float *>(sXt + 2 * MP * STR);            // [2][Q]
    float *s_part = s_coef + 2 * Q;                                           // [2][4]

    const int lid = xcd_logical_id(blockIdx.x - ncb, nblocks);
    if (lid >= total) return;
    const int run = lid % nruns;
    const int g = (lid / nruns) % s.G;
    // split pass: how much a workgroup has to do depends on its chunk's distance from the boundary (every head
    // counts next to it, further away only the slowly decaying ones).  The XCD-aware ids give each XCD a
    // contiguous range of ids, so consecutive ids take chunks nc/8 apart (every XCD gets all distances), and
    // the chunks next to the boundary come first (the long workgroups are handed out before the short ones).
    const int cidx = (lid / (nruns * s.G)) % s.nc;
    const int cperm = (s.nc % 8 == 0) ? (cidx % 8) * (s.nc / 8) + cidx / 8 : cidx;
    const int c = nseg > 1 ? s.nc - 1 - cperm : cidx;
    // split pass (nseg > 1, one slot): the grid covers the segments in front of a boundary only
    const int bgrid = nseg > 1 ? s.B / nseg * (nseg - 1) : s.B;
    const int bb = (lid / (nruns * s.G * s.nc)) % bgrid;
    const int b = nseg > 1 ? bb / (nseg - 1) * nseg + bb % (nseg - 1) : bb;
    const int slot = lid / (nruns * s.G * s.nc * bgrid);
    x += (int64_t)slot * s.H * s.P;
    bmix_t8 += (int64_t)slot * s.B * s.nc * s.G * Q * MN;
    states_lp += (int64_t)slot * s.B * s.nc * s.H * MP * MN;
    const int hpg = s.H / s.G;
    const int h0 = g * hpg + run * ipw;
    const int count = min(ipw, hpg - run * ipw);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, kg = lane >> 5;
    const int64_t tok0 = (int64_t)b * s.L + (int64_t)c * Q;
    const int valid = min(Q, s.L - c * Q);
    const int64_t bcg = ((int64_t)b * s.nc + c) * s.G + g;
    const int tokstride = xts;                       // elements between tokens of x
    const int tq = min(tid, Q - 1);
    // a lane always stages the same two channels 2 p2, 2 p2 + 1; channels past P are staged as zeros
    const bool pok = 2 * (tid & 31) < s.P;
    const int pclamp = pok ? 2 * (tid & 31) : 0;
    const int valid_x = pok ? valid : 0;

    // The tile is computed transposed, S^T[n][p] = Bmix^T . (coef x): the mixed B is the A
    // operand.  Operand row l32 holds column n = 32*wave + prow, so that accumulator row
    // 8a + 4k + b is n = 32*wave + 16k + 4a + b: a lane ends up with 16 consecutive n of one
    // channel p (two 16-byte bf16 stores).  k-step ks covers tokens 16ks + 8kg + 0..7.
    const int prow = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);
    // Split pass (nseg > 1; the shape is that of the segments, "batch" b is segment b % nseg of its
    // sequence): only the states at the segment boundaries are wanted, and a chunk state reaches the
    // boundary behind it times exp2 of the totals of the chunks in between.  Below 2^-150 nothing of
    // it survives in fp32, and the boundary kernel leaves such a chunk out; this kernel computes the
    // states down to 2^-151 (the two sum the totals in different orders).  The chunks behind the
    // last boundary have no workgroups.
    uint32_t hmask = count >= 32 ? 0xffffffffu : (1u << count) - 1u;
    if (nseg > 1) {
        // wave w sums for the heads w, w + 4, ... of the run (a lane per chunk in between), then the
        // waves put their bits together
        uint32_t bits = 0;
        for (int k = wave; k < count; k += 4) {
            const float *tot = cs2 + (((int64_t)b * s.nc) * s.H + h0 + k) * Q + (Q - 1);
            float suf = 0.f;
            for (int cc = c + 1 + lane; cc < s.nc; cc += 64) suf += tot[(int64_t)cc * s.H * Q];
#pragma unroll
            for (int off = 32; off > 0; off >>= 1) suf += __shfl_xor(suf, off);
            if (suf >= SPLIT_KEEP_LOG2 - 1.f) bits |= 1u << k;
        }
        if (lane == 0) reinterpret_cast<uint32_t *>(s_part)[wave] = bits;
        lds_barrier();
        hmask = reinterpret_cast<uint32_t *>(s_part)[0] | reinterpret_cast<uint32_t *>(s_part)[1] |
                reinterpret_cast<uint32_t *>(s_part)[2] | reinterpret_cast<uint32_t *>(s_part)[3];
        lds_barrier();                                   // s_part is the scan's scratch from here on
        hmask = __builtin_amdgcn_readfirstlane(hmask);
        if (hmask == 0) return;
    }
    uint4 bfrag[KS];
    {
        const uint16_t *src = bmix_t8 + (bcg * (Q / 8) * MN + (wave * 32 + prow)) * 8;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks)
            bfrag[ks] = *reinterpret_cast<const uint4 *>(src + (2 * ks + kg) * MN * 8);
    }

    uint16_t dt_raw;
    uint32_t xv[XU][8];
    // all global loads of one head, clamped and unconditional
    auto issue_loads = [&](int h) {
        const uint16_t *xh = x + tok0 * xts + h * s.P + pclamp;
        dt_raw = dt[(tok0 + min(tq, valid - 1)) * s.H + h];
#pragma unroll
        for (int it = 0; it < XU; ++it) {
            const int u = tid + it * MTHREADS;
            const int p2 = u & 31, jg = u >> 5;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = t8_token(jg * 8 + e);
                // raw value: nothing may consume it here, or the loads would be waited for one by
                // one right after their issue; rows past the sequence end are zeroed when staged
                xv[it][e] = *reinterpret_cast<const uint32_t *>(xh + min(j, valid - 1) * tokstride);
            }
        }
    };
    // cumsum, coefficients and the transposed x tile of head h into buffer `buf`
    auto stage = [&](int buf, int h) {
        const float dtv = (tid < valid) ? to_float(bf16{dt_raw}) : 0.f;
        float incl = (tid < Q) ? dtv * A[h] : 0.f;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float v = __shfl_up(incl, off);
            if (lane >= off) incl += v;
        }
        if (lane == 63) s_part[buf * 4 + wave] = incl;
        lds_barrier();
        {
            float base = 0.f;
#pragma unroll
            for (int ww = 0; ww < 3; ++ww)
                if (ww < wave) base += s_part[buf * 4 + ww];
            incl += base;
        }
        float cs_last = 0.f;
#pragma unroll
        for (int ww = 0; ww <= LASTW; ++ww) cs_last += s_part[buf * 4 + ww];
        if (tid < Q) {
            if (cs) cs[(((int64_t)b * s.nc + c) * s.H + h) * Q + tid] = incl;
            s_coef[buf * Q + tid] = dtv * fast_exp2((cs_last - incl) * LOG2E);
        }
        lds_barrier();
        uint16_t *dstX = sXt + buf * MP * STR;
#pragma unroll
        for (int it = 0; it < XU; ++it) {
            const int u = tid + it * MTHREADS;
            const int p2 = u & 31, jg = u >> 5;
            float xa[8], xb[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = t8_token(jg * 8 + e);
                const float cf = s_coef[buf * Q + j];
                const uint32_t xr = (j < valid_x) ? xv[it][e] : 0u;
                xa[e] = bf_lo(xr) * cf;
                xb[e] = bf_hi(xr) * cf;
            }
            *reinterpret_cast<uint4 *>(dstX + (2 * p2) * STR + jg * 8) = pack8(xa);
            *reinterpret_cast<uint4 *>(dstX + (2 * p2 + 1) * STR + jg * 8) = pack8(xb);
        }
    };

    // the heads of the run that are computed, lowest first
    auto next_head = [&]() {
        const int k = __builtin_ctz(hmask);
        hmask &= hmask - 1;
        return h0 + k;
    };
    int hcur = next_head();
    issue_loads(hcur);
    stage(0, hcur);
    {
        // Touch every mixed-B operand register here: the wait for those loads then sits in front
        // of the head loop.  Left inside it, the (static) wait counts of the first MFMAs would also
        // cover the x loads issued at the top of every later iteration, and each head's prefetch
        // would be waited for before the previous head's MFMAs instead of overlapping them.
        uint32_t touch = 0;
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) touch |= bfrag[ks].x ^ bfrag[ks].y ^ bfrag[ks].z ^ bfrag[ks].w;
        if (touch == 0x7fc07fc1u && count < 0) s_part[0] = 1.f;   // never true
    }
    lds_barrier();
    for (int k = 0;; ++k) {
        const int h = hcur;
        const bool more = hmask != 0;
        if (more) { hcur = next_head(); issue_loads(hcur); }
        const uint16_t *srcX = sXt + (k & 1) * MP * STR;
        f32x16_t acc0 = {0}, acc1 = {0};
#pragma unroll
        for (int ks = 0; ks < KS; ++ks) {
            const int kb = ks * 16 + kg * 8;
            const uint4 a0 = *reinterpret_cast<const uint4 *>(srcX + l32 * STR + kb);
            const uint4 a1 = *reinterpret_cast<const uint4 *>(srcX + (32 + l32) * STR + kb);
            acc0 = mfma32(bfrag[ks], a0, acc0);
            acc1 = mfma32(bfrag[ks], a1, acc1);
        }
        // chunk state as bf16 (it is only ever an MFMA operand or a summand of the fp32 scan)
        uint16_t *out = states_lp + ((((int64_t)b * s.nc + c) * s.H + h) * MP + l32) * MN + wave * 32 + 16 * kg;
        {
            float t0[16], t1[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) { t0[v] = acc0[v]; t1[v] = acc1[v]; }
            *reinterpret_cast<uint4 *>(out) = pack8(t0);
            *reinterpret_cast<uint4 *>(out + 8) = pack8(t0 + 8);
            *reinterpret_cast<uint4 *>(out + 32 * MN) = pack8(t1);
            *reinterpret_cast<uint4 *>(out + 32 * MN + 8) = pack8(t1 + 8);
        }
        if (more) stage((k + 1) & 1, hcur);
        lds_barrier();
        if (!more) break;
    }
}

template <int Q>
static swimba_status launch_cs_q(const Shape &s, const void *x, const void *dt, const float *A,
                                 const void *bmix_t8, float *cs, void *states_lp, hipStream_t st, int xts,
                                 int nslots, const void *cmix, const void *bfrag, void *cb, int nseg, const float *cs2)
{
    const int hpg = s.H / s.G;
    // heads per workgroup: as many as possible while at least ~2 workgroups per CU remain
    int ipw = hpg < 32 ? hpg : 32;               // (the kernel keeps the heads of a run as a 32-bit mask)
    while (ipw > 1 && (int64_t)s.B * s.nc * s.G * ((hpg + ipw - 1) / ipw) < 512) ipw = (ipw + 1) / 2;
    // split pass: which heads of a run are computed depends on the data, so shorter runs balance better
    // (measured on the long-sequence workload, whole launch pair: runs of 1, 2, 4, 8 heads 68, 62, 59, 59 us)
    if (nseg > 1 && ipw > 4) ipw = 4;
    const int nruns = (hpg + ipw - 1) / ipw;
    const int64_t total = (int64_t)(nseg > 1 ? s.B / nseg * (nseg - 1) : s.B) * s.nc * s.G * nruns * nslots;
    if (total == 0) return SWIMBA_OK;
    if (total > (int64_t)1 << 30) return SWIMBA_ERR_UNSUPPORTED;
    const int nblocks = xcd_padded(total);
    const size_t shm = (size_t)2 * MP * (Q + 8) * 2 + 2 * Q * sizeof(float) + 8 * sizeof(float);
    // more than 64 KB of dynamic LDS has to be allowed once per device (a plain attribute call:
    // legal under stream capture, but the first call on a device is best made before capturing)
    static std::atomic<uint64_t> attr_set{0};            // one bit per device ordinal
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
    const uint64_t bit = 1ull << (dev & 63);
    if (!(attr_set.load(std::memory_order_acquire) & bit)) {
        e = hipFuncSetAttribute((const void *)chunk_state_mfma_kernel<Q>,
                                hipFuncAttributeMaxDynamicSharedMemorySize, (int)shm);
        if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
        attr_set.fetch_or(bit, std::memory_order_release);
    }
    // the G^T tiles in front, when the caller wants them from this launch
    const int ncb = cb ? xcd_padded((int64_t)s.B * s.nc * s.G * (((Q / 32) * (Q / 32 + 1) / 2 + 3) / 4)) : 0;
    hipLaunchKernelGGL(chunk_state_mfma_kernel<Q>, dim3(ncb + nblocks), dim3(MTHREADS), shm, st,
                       (const uint16_t *)x, (const uint16_t *)dt, A, (const uint16_t *)bmix_t8, cs,
                       (uint16_t *)states_lp, s, ipw, nruns, (int)total, nblocks, xts, nslots, ncb,
                       (const uint16_t *)cmix, (const uint16_t *)bfrag, (uint16_t *)cb, nseg, cs2);
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

// x is (B, L, nslots, H, P) for nslots > 1 (rows of the selected experts), (B, L, H, P) otherwise;
// with cb != nullptr the same launch also computes the G^T tiles from cmix and bfrag
swimba_status launch_chunk_state_mfma(const Shape &s, const void *x, const void *dt, const float *A,
                                      const void *bmix_t8, float *cs, void *states_lp, hipStream_t st,
                                      int nslots, const void *cmix, const void *bfrag, void *cb, int nseg,
                                      const float *cs2)
{
    if (nseg < 1 || (nseg > 1 && (!cs2 || nslots != 1))) return SWIMBA_ERR_UNSUPPORTED;
    if (nseg == 1 && !cs) return SWIMBA_ERR_NULL;
    const int xts = nslots * s.H * s.P;
    switch (s.Q) {
    case 64: return launch_cs_q<64>(s, x, dt, A, bmix_t8, cs, states_lp, st, xts, nslots, cmix, bfrag, cb, nseg, cs2);
    case 128: return launch_cs_q<128>(s, x, dt, A, bmix_t8, cs, states_lp, st, xts, nslots, cmix, bfrag, cb, nseg, cs2);
    case 256: return launch_cs_q<256>(s, x, dt, A, bmix_t8, cs, states_lp, st, xts, nslots, cmix, bfrag, cb, nseg, cs2);
    }
    return SWIMBA_ERR_UNSUPPORTED;
}

// =========================================================================================
// Output:  y_i = sum_{j<=i} G[i][j] exp(cs_i-cs_j) dt_j x_j + exp(cs_i) Cmix_i.H_c + D x_i
// Workgroup = (batch, chunk, head), one wave per 32-token output tile (Q/32 waves).
// Tile I has I+1 causal tile pairs; waves w and w+4, which share a SIMD, get tiles
// whose pair counts add up to the same number on every SIMD.
//
// Everything is computed transposed, Y^T[p][i] (accumulator rows = channels, columns =
// tokens), so that every per-token factor is a per-lane scalar:
//   Y^T  = H_c . Cmix^T  scaled by exp(cs_i)                       (A = H_c rows, B = Cmix regs)
//   Y^T += x^T . M^T,  M^T[j][i] = G^T[j][i] * decay(i,j) * dt_j    (A = x^T from LDS, B = M^T)
// The G^T tile arrives from `cb` in accumulator layout (rows j, cols i), which is also
// a valid B-operand layout once the k index (j) is permuted; x^T is staged in LDS with
// the same permutation (within 16 tokens: bits 2 and 3 swapped).
// For J < I the decay factors as exp(cs_i - R_J) * exp(R_J - cs_j) with R_J = cs at the
// last token of tile J; both factors are <= 1 (cs is non-increasing), so nothing
// overflows and only one exp per lane and pair is needed; the second factor is
// tabulated per token.  The diagonal tile uses exp(cs_i - cs_j) under the mask i >= j.
// Accumulator row r = 8a + 4k + b holds channel 16k + 4a + b of its 32-channel half, so
// a lane ends up with 16 consecutive channels of one token; the tile is rounded to
// bf16, passed through LDS and stored as full 128-byte rows (D x is added on the way).
// cs is kept multiplied by log2(e): every exponential is one v_exp_f32.
// =========================================================================================
// MODE 1 (one pass per expert or per slot, the results added up in y): the skip term carries the
// per-token factor skip_w[token * skip_stride], and with `accumulate` the result is added to
// what y already holds.
// MODE 2 (one input stream per expert, all slots in one launch): x is (B, L, nslots, H, P); the
// carried state is read out once, then slot after slot the x tile of the slot is staged and its
// tile pairs, taken from the slot's G^T image, go into the same accumulators.  The skip term
// D sum_r pi_r x^(r) is one more contraction per slot, x^T . diag(D pi_{i,r}) with the factor
// split into two bf16 terms, so the epilogue reads no x; pi_{i,r} = skip_w[token * skip_stride + r].
// MODE 3 (short sequences, no scan launch): Hlp holds the chunk states S_c as the chunk-state kernel
// wrote them, and the workgroup of chunk c carries the state forward itself,
// H_c = S_{c-1} + a_{c-1} (S_{c-2} + ... a_0 h0), a_c = exp(cs_c[Q-1]), in fp32 and in the scan
// kernel's order of operations; the workgroups of the last chunk also write h_final.  At most
// OUTPUT_LOOKBACK_MAX_CHUNKS chunks.
template <int Q, int MODE>
__global__ void __launch_bounds__(64 * (Q / 32), (Q == 256 ? 4 : 1))   // Q = 256: two workgroups per compute unit
output_mfma_kernel(const uint16_t *__restrict__ x, const uint16_t *__restrict__ dt,
                   const float *__restrict__ D, const uint16_t *__restrict__ cmix,
                   const uint16_t *__restrict__ cb, const float *__restrict__ cs,
                   const uint16_t *__restrict__ Hlp, uint16_t *__restrict__ y, Shape s, int total,
                   int nblocks, const float *__restrict__ skip_w, int skip_stride, int accumulate,
                   int nslots, const float *__restrict__ h0, float *__restrict__ h_final)
{
    constexpr bool XE = (MODE == 1);
    constexpr bool SLOTS = (MODE == 2);
    constexpr bool LOOKBACK = (MODE == 3);
    constexpr int NT = Q / 32;                 // 32-token tiles in the chunk
    constexpr int NP = NT * (NT + 1) / 2;
    constexpr int NTHR = 64 * NT;              // one wave per output tile
    constexpr int HSTR = MN + 8;               // row stride of the carried-state tile
    constexpr int XSTR = Q + 8;                // row stride of the transposed x tile
    // MODE 2 keeps the x tiles of two slots: the second one takes the place of the carried-state tile,
    // which is dead once the state has been read out, and runs past it (dynamic LDS, more than 64 KB
    // at Q = 256); the other modes keep their fixed layout.
    uint16_t *sX, *sH, *sX1;
    float *s_cs, *s_dt, *s_f;
    if constexpr (SLOTS) {
        extern __shared__ __align__(16) unsigned char smem_slots[];
        sX = reinterpret_cast<uint16_t *>(smem_slots);
        sX1 = sX + MP * XSTR;
        sH = sX1;
        s_cs = reinterpret_cast<float *>(sX1 + MP * (XSTR > HSTR ? XSTR : HSTR));
        s_dt = s_cs + Q;
        s_f = s_dt + Q;
    } else {
        __shared__ __align__(16) uint16_t sX_[MP * XSTR];
        __shared__ __align__(16) uint16_t sH_[MP * HSTR];
        __shared__ float s_cs_[Q], s_dt_[Q], s_f_[Q];
        sX = sX_; sH = sH_; sX1 = sX_;
        s_cs = s_cs_; s_dt = s_dt_; s_f = s_f_;
    }

    const int lid = xcd_logical_id(blockIdx.x, nblocks);
    if (lid >= total) return;
    const int h = lid % s.H;
    const int c = (lid / s.H) % s.nc;
    const int b = lid / (s.H * s.nc);
    const int g = (h * s.G) / s.H;
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // wave-uniform
    const int l32 = lane & 31, kg = lane >> 5;
    const int64_t tok0 = (int64_t)b * s.L + (int64_t)c * Q;
    const int valid = min(Q, s.L - c * Q);
    const int64_t bcg = ((int64_t)b * s.nc + c) * s.G + g;
    const int tokstride = s.H * s.P;                         // elements between tokens of y (P <= MP)
    const int xts = SLOTS ? nslots * tokstride : tokstride;  // ... of x
    const uint16_t *xh = x + tok0 * xts + h * s.P;           // x[token 0 of the chunk][slot 0][h][0]
    uint16_t *yh = y + (tok0 * s.H + h) * s.P;
    // channels past the caller's P: staged as zeros, never stored
    const bool pok = 2 * (tid & 31) < s.P;
    const int pclamp = pok ? 2 * (tid & 31) : 0;
    const int valid_x = pok ? valid : 0;
    // channel held by operand row l32 (see the header comment)
    const int prow = 16 * ((l32 >> 2) & 1) + 4 * (l32 >> 3) + (l32 & 3);

    // Waves w and w + 4 share a SIMD: give them tiles whose causal work adds up to the
    // same amount on every SIMD.
    const int I = (NT == 8 && wave >= 4) ? 11 - wave : wave;

    // ---- issue every global load of the prologue before the first barrier ----
    // (indices are clamped instead of branching, so that all loads go out back to back)
    const int tq = min(tid, Q - 1);
    const float *csr = cs + (((int64_t)b * s.nc + c) * s.H + h) * Q;
    const float cs_raw = csr[tq];
    const float cs_end = csr[tq | 31];           // cs at the last token of this token's tile
    const uint16_t dt_raw = dt[(tok0 + min(tq, valid - 1)) * s.H + h];
    constexpr int HPASS = 64 * 16 / NTHR;      // 16-byte pieces of the state tile per lane
    uint4 hreg[HPASS];
    if constexpr (!LOOKBACK) {
        const uint16_t *Hc = Hlp + (((int64_t)b * s.nc + c) * s.H + h) * MP * MN;
#pragma unroll
        for (int pass = 0; pass < HPASS; ++pass) {
            const int row = (tid >> 4) + (NTHR / 16) * pass, piece = tid & 15;
            hreg[pass] = load_nt(Hc + row * MN + piece * 8);   // the carried state is read once
        }
    }
    // MODE 3: the chunk states before this chunk, four at a time (clamped, unconditional loads)
    uint4 sprev[LOOKBACK ? 4 : 1][HPASS];
    float aprev[LOOKBACK ? 4 : 1];
    auto lb_issue = [&](int c0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const int cp = max(min(c0 + u, c - 1), 0);
            const uint16_t *Sc = Hlp + (((int64_t)b * s.nc + cp) * s.H + h) * MP * MN;
#pragma unroll
            for (int pass = 0; pass < HPASS; ++pass) {
                const int row = (tid >> 4) + (NTHR / 16) * pass, piece = tid & 15;
                sprev[u][pass] = *reinterpret_cast<const uint4 *>(Sc + row * MN + piece * 8);
            }
            aprev[u] = cs[(((int64_t)b * s.nc + cp) * s.H + h) * Q + Q - 1];
        }
    };
    float hacc[LOOKBACK ? HPASS : 1][8];
    auto lb_fold = [&](int c0) __attribute__((always_inline)) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (c0 + u < c) {
                const float a = fast_exp2(aprev[u] * LOG2E);
#pragma unroll
                for (int pass = 0; pass < HPASS; ++pass) {
                    float sv[8];
                    unpack8(sv, sprev[u][pass]);
#pragma unroll
                    for (int v = 0; v < 8; ++v) hacc[pass][v] = a * hacc[pass][v] + sv[v];
                }
            }
        }
    };
    if constexpr (LOOKBACK) {
#pragma unroll
        for (int pass = 0; pass < HPASS; ++pass) {
            const int row = (tid >> 4) + (NTHR / 16) * pass, piece = tid & 15;
            const bool real = h0 && row < s.P && piece * 8 < s.N;      // h0 has the caller's P x N
            const float *hp = h0 + (((int64_t)b * s.H + h) * s.P + (real ? row : 0)) * s.N + (real ? piece * 8 : 0);
            float4 lo = make_float4(0.f, 0.f, 0.f, 0.f), hi = lo;
            if (real) { lo = *reinterpret_cast<const float4 *>(hp); hi = *reinterpret_cast<const float4 *>(hp + 4); }
            hacc[pass][0] = lo.x; hacc[pass][1] = lo.y; hacc[pass][2] = lo.z; hacc[pass][3] = lo.w;
            hacc[pass][4] = hi.x; hacc[pass][5] = hi.y; hacc[pass][6] = hi.z; hacc[pass][7] = hi.w;
        }
        lb_issue(0);
    }
    // x staging: unit = (8 tokens in operand order) x (2 channels)
    constexpr int XU = (Q / 8) * 32 / NTHR;
    uint32_t xv[XU][8], xw[SLOTS ? XU : 1][8];   // xw: the second slot of a pair (MODE 2)
    auto load_x = [&](uint32_t (*xd)[8], const uint16_t *xs, int xts, int vlast) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < XU; ++it) {
            const int u = tid + it * NTHR;
            const int gi = u >> 5;
            const int t16 = gi >> 1, kgx = gi & 1;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = 16 * t16 + 8 * (e >> 2) + 4 * kgx + (e & 3);
                // raw value: rows past the end of the sequence and channels past P are zeroed when staged
                // (a select here would put a wait behind every single load)
                xd[it][e] = *reinterpret_cast<const uint32_t *>(xs + min(j, vlast) * xts + pclamp);
            }
        }
    };
    load_x(xv, xh, xts, valid - 1);
    if constexpr (SLOTS) load_x(xw, xh + min(1, nslots - 1) * tokstride, xts, valid - 1);
    // mixed C rows of the owned tiles (operand registers)
    uint4 cfrag[8];
    {
        const uint16_t *src = cmix + (((bcg * NT + I) * 8) * 64 + lane) * 8;
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) cfrag[ks] = *reinterpret_cast<const uint4 *>(src + ks * 64 * 8);
    }
    if constexpr (LOOKBACK) {
        lb_fold(0);
        if (c > 4) {                               // workgroup-uniform
            lb_issue(4);
            lb_fold(4);
        }
#pragma unroll
        for (int pass = 0; pass < HPASS; ++pass) hreg[pass] = pack8(hacc[pass]);
        if (h_final && c == s.nc - 1) {
            // the state after the last chunk: one more step of the recurrence, on this chunk's own state
            const uint16_t *Sc = Hlp + (((int64_t)b * s.nc + c) * s.H + h) * MP * MN;
            const float a = fast_exp2(csr[Q - 1] * LOG2E);
#pragma unroll
            for (int pass = 0; pass < HPASS; ++pass) {
                const int row = (tid >> 4) + (NTHR / 16) * pass, piece = tid & 15;
                float sv[8];
                unpack8(sv, *reinterpret_cast<const uint4 *>(Sc + row * MN + piece * 8));
                if (row < s.P && piece * 8 < s.N) {
                    float *hp = h_final + (((int64_t)b * s.H + h) * s.P + row) * s.N + piece * 8;
                    *reinterpret_cast<float4 *>(hp) = make_float4(a * hacc[pass][0] + sv[0], a * hacc[pass][1] + sv[1],
                                                                  a * hacc[pass][2] + sv[2], a * hacc[pass][3] + sv[3]);
                    *reinterpret_cast<float4 *>(hp + 4) = make_float4(a * hacc[pass][4] + sv[4], a * hacc[pass][5] + sv[5],
                                                                      a * hacc[pass][6] + sv[6], a * hacc[pass][7] + sv[7]);
                }
            }
        }
    }
    // per-token tables: cs (times log2 e), dt, and dt * exp(R_J - cs_j) for the tiles J < I.
    // dt is applied through these tables (i.e. on the M^T operand), so x itself is staged
    // unscaled: a pure bf16 transpose.
    if (tid < Q) {
        const float dtv = (tid < valid) ? to_float(bf16{dt_raw}) : 0.f;
        s_cs[tid] = cs_raw * LOG2E;
        s_dt[tid] = dtv;
        s_f[tid] = dtv * fast_exp2((cs_end - cs_raw) * LOG2E);
    }
#pragma unroll
    for (int pass = 0; pass < HPASS; ++pass) {
        const int row = (tid >> 4) + (NTHR / 16) * pass, piece = tid & 15;
        *reinterpret_cast<uint4 *>(sH + row * HSTR + piece * 8) = hreg[pass];
    }
    auto stage_x = [&](uint32_t (*xv)[8], uint16_t *sX) __attribute__((always_inline)) {
#pragma unroll
        for (int it = 0; it < XU; ++it) {
            const int u = tid + it * NTHR;
            const int p2 = u & 31, gi = u >> 5;
            const int t16 = gi >> 1, kgx = gi & 1;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int j = 16 * t16 + 8 * (e >> 2) + 4 * kgx + (e & 3);
                xv[it][e] = (j < valid_x) ? xv[it][e] : 0u;
            }
            uint4 lo, hi;   // channel 2*p2 and 2*p2+1 of the unit's 8 tokens
            lo.x = __builtin_amdgcn_perm(xv[it][1], xv[it][0], 0x05040100u);
            lo.y = __builtin_amdgcn_perm(xv[it][3], xv[it][2], 0x05040100u);
            lo.z = __builtin_amdgcn_perm(xv[it][5], xv[it][4], 0x05040100u);
            lo.w = __builtin_amdgcn_perm(xv[it][7], xv[it][6], 0x05040100u);
            hi.x = __builtin_amdgcn_perm(xv[it][1], xv[it][0], 0x07060302u);
            hi.y = __builtin_amdgcn_perm(xv[it][3], xv[it][2], 0x07060302u);
            hi.z = __builtin_amdgcn_perm(xv[it][5], xv[it][4], 0x07060302u);
            hi.w = __builtin_amdgcn_perm(xv[it][7], xv[it][6], 0x07060302u);
            *reinterpret_cast<uint4 *>(sX + (2 * p2) * XSTR + 16 * t16 + 8 * kgx) = lo;
            *reinterpret_cast<uint4 *>(sX + (2 * p2 + 1) * XSTR + 16 * t16 + 8 * kgx) = hi;
        }
    };
    stage_x(xv, sX);
    lds_barrier();

    const float dsk = D ? D[h] : 0.f;
    const uint16_t *sXr0 = sX + prow * XSTR + 8 * kg;          // operand rows of the two channel halves
    const uint16_t *sXr1 = sX + (32 + prow) * XSTR + 8 * kg;

    // G^T tiles are streamed two pairs ahead of their use (tile index clamped to I, so the
    // loads are unconditional and the wait counters stay exact).
    const uint16_t *tile0 = cb + ((bcg * NP + I * (I + 1) / 2) * 2 * 64 + lane) * 8;
    const int64_t cbimg = (int64_t)s.B * s.nc * s.G * NP * 1024;   // elements per slot image of the tiles
    auto load_tile = [&](int J, uint4 &u0, uint4 &u1) {
        const uint16_t *t = tile0 + min(J, I) * (2 * 64 * 8);
        u0 = *reinterpret_cast<const uint4 *>(t);
        u1 = *reinterpret_cast<const uint4 *>(t + 64 * 8);
    };
    uint4 uA0, uA1, uB0, uB1;
    if constexpr (!SLOTS) {
        load_tile(0, uA0, uA1);
        load_tile(1, uB0, uB1);
    }
    {
        // x of the skip term, loaded the way y is stored: lane -> (token row, 16-byte piece)
        const int erow = lane >> 3, epiece = lane & 7;
        const bool epok = epiece * 8 < s.P;
        const int eoff = epok ? epiece * 8 : 0;
        uint4 xe[4];
        if (!SLOTS) {
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const int i = I * 32 + erow + 8 * q4;
                xe[q4] = *reinterpret_cast<const uint4 *>(xh + min(i, valid - 1) * tokstride + eoff);
            }
        }
        // keep these loads (first two G^T tiles, x of the skip term) in front of the MFMAs below:
        // moved behind them, the first tile pair would wait a full memory latency
        __builtin_amdgcn_sched_barrier(0);
        f32x16_t y0 = {0}, y1 = {0};
        // ---- H_c . Cmix^T, then the per-token factor exp(cs_i) ----
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            const uint4 h0 = *reinterpret_cast<const uint4 *>(sH + prow * HSTR + 64 * kg + ks * 8);
            const uint4 h1 = *reinterpret_cast<const uint4 *>(sH + (32 + prow) * HSTR + 64 * kg + ks * 8);
            y0 = mfma32(h0, cfrag[ks], y0);
            y1 = mfma32(h1, cfrag[ks], y1);
        }
        const float csi = s_cs[I * 32 + l32];
        {
            const float sc = fast_exp2(csi);
#pragma unroll
            for (int v = 0; v < 16; ++v) { y0[v] *= sc; y1[v] *= sc; }
        }
        // ---- intra-chunk part ----
        auto pair = [&](int J, uint4 u0, uint4 u1, int xoff) __attribute__((always_inline)) {
            float m[16];
            unpack8(m, u0);
            unpack8(m + 8, u1);
            if (J < I) {
                // dt_j exp(R_J - cs_j) from the table, exp(cs_i - R_J) once per lane
                const float *fj = s_f + J * 32 + 4 * kg;
                const float ei = fast_exp2(csi - s_cs[J * 32 + 31]);
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const float4 f4 = *reinterpret_cast<const float4 *>(fj + 8 * a);
                    m[4 * a + 0] *= ei * f4.x;
                    m[4 * a + 1] *= ei * f4.y;
                    m[4 * a + 2] *= ei * f4.z;
                    m[4 * a + 3] *= ei * f4.w;
                }
            } else {
                const float *cj = s_cs + J * 32 + 4 * kg;
                const float *dj = s_dt + J * 32 + 4 * kg;
#pragma unroll
                for (int a = 0; a < 4; ++a) {
                    const float4 c4 = *reinterpret_cast<const float4 *>(cj + 8 * a);
                    const float4 d4 = *reinterpret_cast<const float4 *>(dj + 8 * a);
                    const float cc[4] = {c4.x, c4.y, c4.z, c4.w};
                    const float dd[4] = {d4.x, d4.y, d4.z, d4.w};
#pragma unroll
                    for (int bb = 0; bb < 4; ++bb) {
                        const int jl = 8 * a + 4 * kg + bb;
                        // masked entries (j > i) get a hugely negative exponent: exp2 -> 0
                        const float arg = (l32 >= jl) ? fminf(csi - cc[bb], 0.f) : -1.0e30f;
                        m[4 * a + bb] *= fast_exp2(arg) * dd[bb];
                    }
                }
            }
#pragma unroll
            for (int t = 0; t < 2; ++t) {
                const uint4 mfrag = pack8(m + 8 * t);
                const uint4 x0 = *reinterpret_cast<const uint4 *>(sXr0 + xoff + J * 32 + 16 * t);
                const uint4 x1 = *reinterpret_cast<const uint4 *>(sXr1 + xoff + J * 32 + 16 * t);
                y0 = mfma32(x0, mfrag, y0);
                y1 = mfma32(x1, mfrag, y1);
            }
        };
        if constexpr (!SLOTS) {
            // three tile buffers rotate by name, so no register moves sit behind the loads
            uint4 uC0, uC1;
            int J = 0;
            while (true) {
                load_tile(J + 2, uC0, uC1);
                pair(J, uA0, uA1, 0);
                if (++J > I) break;
                load_tile(J + 2, uA0, uA1);
                pair(J, uB0, uB1, 0);
                if (++J > I) break;
                load_tile(J + 2, uB0, uB1);
                pair(J, uC0, uC1, 0);
                if (++J > I) break;
            }
        } else {
            // Slots two at a time, their x tiles side by side in LDS.  The first pair's tiles were
            // loaded in the prologue; the second tile of a pair is staged once every wave has read
            // the carried state out of the space it takes.
            const int iw = I * 32 + l32;                       // this lane's token (column of the tile)
            const float *wtok = skip_w + (tok0 + min(iw, valid - 1)) * skip_stride;
            lds_barrier();
            stage_x(xw, sX1);
            lds_barrier();
            for (int g0 = 0; g0 < nslots; g0 += 2) {
                const int ns = min(2, nslots - g0);
                // router weights of the two slots for the skip term
                const float w0 = wtok[g0], w1 = wtok[min(g0 + 1, nslots - 1)];
                if (g0 > 0) {
                    // stride and last row go through opaque copies: the row addresses are rebuilt here instead
                    // of living in registers (or scratch memory) across the whole kernel
                    int xts_r = xts, vlast_r = valid - 1;
                    asm volatile("" : "+s"(xts_r), "+s"(vlast_r));
                    load_x(xv, xh + g0 * tokstride, xts_r, vlast_r);
                    load_x(xw, xh + min(g0 + 1, nslots - 1) * tokstride, xts_r, vlast_r);
                    lds_barrier();                              // every wave is done with the previous pair of slots
                    stage_x(xv, sX);
                    stage_x(xw, sX1);
                    lds_barrier();
                }
                // the (slot, J) steps of the pair of slots as one sequence; three tile buffers rotate by
                // name and the loads run two steps ahead, across the change of slot
                const uint16_t *tileg = tile0 + g0 * cbimg;
                int pj = 0, psl = 0;
                auto fetch = [&](uint4 &u0, uint4 &u1) __attribute__((always_inline)) {
                    const uint16_t *t = tileg + psl * cbimg + pj * (2 * 64 * 8);
                    u0 = *reinterpret_cast<const uint4 *>(t);
                    u1 = *reinterpret_cast<const uint4 *>(t + 64 * 8);
                    // next tile; past the last step the counters stay on the last tile (plain selects: a
                    // conditional store to one of two counters would put both in scratch memory)
                    const bool more = pj < I, wrap = !more && psl + 1 < ns;
                    pj = more ? pj + 1 : (wrap ? 0 : pj);
                    psl = wrap ? psl + 1 : psl;
                };
                int cj = 0, csl = 0;
                auto step = [&](uint4 u0, uint4 u1) __attribute__((always_inline)) {
                    pair(cj, u0, u1, csl * (MP * XSTR));
                    const bool last = (cj == I);
                    const int slot_now = csl;
                    cj = last ? 0 : cj + 1;
                    csl = last ? csl + 1 : csl;
                    if (!last) return;
                    // that was the last tile of the slot; now its skip term: Y^T += x^T . diag(D pi_{i,r}); the B operand
                    // of k-step t holds rows j = 16t + 8(e>>2) + 4kg + (e&3) of column i = l32, non-zero
                    // where j == i
                    const float dv = (iw < valid) ? dsk * (slot_now ? w1 : w0) : 0.f;
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
                        const uint4 mh = make_uint4(wh[0], wh[1], wh[2], wh[3]);
                        const uint4 ml = make_uint4(wl[0], wl[1], wl[2], wl[3]);
                        const uint4 x0 = *reinterpret_cast<const uint4 *>(sXr0 + slot_now * (MP * XSTR) + I * 32 + 16 * t);
                        const uint4 x1 = *reinterpret_cast<const uint4 *>(sXr1 + slot_now * (MP * XSTR) + I * 32 + 16 * t);
                        y0 = mfma32(x0, mh, y0);
                        y1 = mfma32(x1, mh, y1);
                        y0 = mfma32(x0, ml, y0);
                        y1 = mfma32(x1, ml, y1);
                    }
                };
                const int steps = ns * (I + 1);
                uint4 uC0, uC1;
                fetch(uA0, uA1);
                fetch(uB0, uB1);
                int q = 0;
                while (true) {
                    fetch(uC0, uC1);
                    step(uA0, uA1);
                    if (++q >= steps) break;
                    fetch(uA0, uA1);
                    step(uB0, uB1);
                    if (++q >= steps) break;
                    fetch(uB0, uB1);
                    step(uC0, uC1);
                    if (++q >= steps) break;
                }
            }
        }
        // ---- y = acc + D x.  The wave's 32 x 64 tile goes through LDS (the x^T tile is
        // dead by now) so that every global access is a full 128-byte row. ----
        lds_barrier();
        // scratch: 32 rows x 8 pieces of 16 bytes per wave, piece index XOR-swizzled by the row
        static_assert(NT * 32 * MP * 2 <= MP * XSTR * 2, "epilogue scratch must fit in the x^T tile");
        constexpr int YSTR = MP;
        uint16_t *scr = sX + wave * 32 * YSTR;
        {
            float a0[16], a1[16];
#pragma unroll
            for (int v = 0; v < 16; ++v) { a0[v] = y0[v]; a1[v] = y1[v]; }
            uint16_t *dst = scr + l32 * YSTR;              // lane holds channels 16kg..16kg+15 (+32)
            const int sw = l32 & 7;
            *reinterpret_cast<uint4 *>(dst + (((2 * kg) ^ sw) << 3)) = pack8(a0);
            *reinterpret_cast<uint4 *>(dst + (((2 * kg + 1) ^ sw) << 3)) = pack8(a0 + 8);
            *reinterpret_cast<uint4 *>(dst + (((4 + 2 * kg) ^ sw) << 3)) = pack8(a1);
            *reinterpret_cast<uint4 *>(dst + (((5 + 2 * kg) ^ sw) << 3)) = pack8(a1 + 8);
        }
        lds_barrier();
#pragma unroll
        for (int q4 = 0; q4 < 4; ++q4) {
            const int row = erow + 8 * q4, i = I * 32 + row;
            if (i < valid && epok) {
                const uint4 tile_row = *reinterpret_cast<const uint4 *>(scr + row * YSTR + ((epiece ^ (row & 7)) << 3));
                if (SLOTS) {
                    store_nt(yh + i * tokstride + epiece * 8, tile_row);   // the skip term is in the tile already
                } else {
                    float a[8], xf[8];
                    unpack8(a, tile_row);
                    unpack8(xf, xe[q4]);
                    float dski = dsk;
                    if (XE) {
                        if (skip_w) dski *= skip_w[(tok0 + i) * skip_stride];
                        if (accumulate) {
                            float prev[8];
                            unpack8(prev, *reinterpret_cast<const uint4 *>(yh + i * tokstride + epiece * 8));
#pragma unroll
                            for (int e = 0; e < 8; ++e) a[e] += prev[e];
                        }
                    }
#pragma unroll
                    for (int e = 0; e < 8; ++e) a[e] += dski * xf[e];
                    store_nt(yh + i * tokstride + epiece * 8, pack8(a));
                }
            }
        }
    }
}

template <int Q>
static swimba_status launch_out_q(const Shape &s, const void *x, const void *dt, const float *D,
                                  const void *cmix, const void *cb, const float *cs, const void *Hlp,
                                  void *y, const float *skip_w, int skip_stride, int accumulate, int nslots,
                                  hipStream_t st, bool lookback = false, const float *h0 = nullptr,
                                  float *h_final = nullptr)
{
    const int64_t total = (int64_t)s.B * s.nc * s.H;
    if (total == 0) return SWIMBA_OK;
    const int nblocks = xcd_padded(total);
#define SWIMBA_OUT_LAUNCH(MODE, SHM, SW, SS, ACC, NSL)                                                             \
    hipLaunchKernelGGL((output_mfma_kernel<Q, MODE>), dim3(nblocks), dim3(64 * (Q / 32)), SHM, st,                \
                       (const uint16_t *)x, (const uint16_t *)dt, D, (const uint16_t *)cmix, (const uint16_t *)cb, \
                       cs, (const uint16_t *)Hlp, (uint16_t *)y, s, (int)total, nblocks, SW, SS, ACC, NSL, h0,    \
                       h_final)
    if (nslots > 0) {
        // two x tiles (the second in the place of the carried-state tile) and the three tables
        constexpr int XSTR = Q + 8, HSTR = MN + 8;
        constexpr size_t shm = (size_t)(MP * XSTR + MP * (XSTR > HSTR ? XSTR : HSTR)) * 2 + 3 * Q * sizeof(float);
        static std::atomic<uint64_t> attr_set{0};            // one bit per device ordinal
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
        const uint64_t bit = 1ull << (dev & 63);
        if (!(attr_set.load(std::memory_order_acquire) & bit)) {
            e = hipFuncSetAttribute((const void *)output_mfma_kernel<Q, 2>, hipFuncAttributeMaxDynamicSharedMemorySize,
                                    (int)shm);
            if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
            attr_set.fetch_or(bit, std::memory_order_release);
        }
        SWIMBA_OUT_LAUNCH(2, shm, skip_w, skip_stride, 0, nslots);
    } else if (lookback) {
        if (s.nc > OUTPUT_LOOKBACK_MAX_CHUNKS) return SWIMBA_ERR_UNSUPPORTED;
        SWIMBA_OUT_LAUNCH(3, 0, nullptr, 0, 0, 1);
    } else if (skip_w || accumulate) {
        SWIMBA_OUT_LAUNCH(1, 0, skip_w, skip_stride, accumulate, 1);
    } else {
        SWIMBA_OUT_LAUNCH(0, 0, nullptr, 0, 0, 1);
    }
#undef SWIMBA_OUT_LAUNCH
    SWIMBA_CHECK_LAUNCH();
    return SWIMBA_OK;
}

swimba_status launch_output_mfma(const Shape &s, const void *x, const void *dt, const float *D,
                                 const void *cmix, const void *cb, const float *cs,
                                 const void *states_lp, void *y, const float *skip_w, int skip_stride,
                                 int accumulate, hipStream_t st)
{
    switch (s.Q) {
    case 64: return launch_out_q<64>(s, x, dt, D, cmix, cb, cs, states_lp, y, skip_w, skip_stride, accumulate, 0, st);
    case 128: return launch_out_q<128>(s, x, dt, D, cmix, cb, cs, states_lp, y, skip_w, skip_stride, accumulate, 0, st);
    case 256: return launch_out_q<256>(s, x, dt, D, cmix, cb, cs, states_lp, y, skip_w, skip_stride, accumulate, 0, st);
    }
    return SWIMBA_ERR_UNSUPPORTED;
}

// Short sequences (at most OUTPUT_LOOKBACK_MAX_CHUNKS chunks): states_lp holds the chunk states, not the carried ones; every
// workgroup carries the state up to its chunk itself and the last chunk's workgroups write h_final.
swimba_status launch_output_lookback_mfma(const Shape &s, const void *x, const void *dt, const float *D,
                                          const void *cmix, const void *cb, const float *cs, const void *states_lp,
                                          void *y, const float *h0, float *h_final, hipStream_t st)
{
    switch (s.Q) {
    case 64: return launch_out_q<64>(s, x, dt, D, cmix, cb, cs, states_lp, y, nullptr, 0, 0, 0, st, true, h0, h_final);
    case 128: return launch_out_q<128>(s, x, dt, D, cmix, cb, cs, states_lp, y, nullptr, 0, 0, 0, st, true, h0, h_final);
    case 256: return launch_out_q<256>(s, x, dt, D, cmix, cb, cs, states_lp, y, nullptr, 0, 0, 0, st, true, h0, h_final);
    }
    return SWIMBA_ERR_UNSUPPORTED;
}

// all slots of the forward with one input stream per expert in one launch: x (B, L, nslots, H, P),
// cb = nslots images of G^T tiles, w (B, L, nslots) router weights of the slots
swimba_status launch_output_slots_mfma(const Shape &s, const void *x, const void *dt, const float *D,
                                       const void *cmix, const void *cb, const float *cs,
                                       const void *states_lp, void *y, const float *w, int nslots, hipStream_t st)
{
    if (nslots < 1 || !w) return SWIMBA_ERR_UNSUPPORTED;
    switch (s.Q) {
    case 64: return launch_out_q<64>(s, x, dt, D, cmix, cb, cs, states_lp, y, w, nslots, 0, nslots, st);
    case 128: return launch_out_q<128>(s, x, dt, D, cmix, cb, cs, states_lp, y, w, nslots, 0, nslots, st);
    case 256: return launch_out_q<256>(s, x, dt, D, cmix, cb, cs, states_lp, y, w, nslots, 0, nslots, st);
    }
    return SWIMBA_ERR_UNSUPPORTED;
}

}  // namespace swimba
