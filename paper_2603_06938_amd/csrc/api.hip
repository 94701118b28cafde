// C ABI of libswimba: host-side validation, workspace carve-up, kernel dispatch.
#include "common.hpp"

#include <string.h>

#include <atomic>
#include <initializer_list>

namespace swimba {

static thread_local int g_last_hip_error = 0;
void set_last_hip_error(int e) { g_last_hip_error = e; }

static inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// Pointer alignment (NULL passes: whether a pointer may be NULL is checked elsewhere).  The
// large tensors are read and written with 16-byte vector accesses; the small per-token and
// per-head ones element by element.
static swimba_status check_align(int io_dtype, std::initializer_list<const void *> vec16,
                                 std::initializer_list<const void *> io_elems,
                                 std::initializer_list<const void *> words)
{
    const uintptr_t io = io_dtype == SWIMBA_BF16 ? 2 : 4;
    for (const void *q : vec16)
        if ((uintptr_t)q & 15u) return SWIMBA_ERR_ALIGNMENT;
    for (const void *q : io_elems)
        if ((uintptr_t)q & (io - 1)) return SWIMBA_ERR_ALIGNMENT;
    for (const void *q : words)
        if ((uintptr_t)q & 3u) return SWIMBA_ERR_ALIGNMENT;
    return SWIMBA_OK;
}

// Checks that hold for both entry points.
static swimba_status check_common(const swimba_dims *d)
{
    if (!d) return SWIMBA_ERR_NULL;
    if (d->io_dtype != SWIMBA_F32 && d->io_dtype != SWIMBA_BF16) return SWIMBA_ERR_DTYPE;
    if (d->batch < 0 || d->seqlen < 0 || d->nheads < 1 || d->headdim < 1 || d->dstate < 1 ||
        d->ngroups < 1 || d->nexperts < 1 || d->top_k < 1 || d->top_k > d->nexperts ||
        d->nheads % d->ngroups != 0)
        return SWIMBA_ERR_SHAPE;
    if (d->nexperts > SWIMBA_MAX_EXPERTS || d->top_k > SWIMBA_MAX_TOPK ||
        d->dstate > SWIMBA_MAX_DSTATE || d->headdim > SWIMBA_MAX_HEADDIM)
        return SWIMBA_ERR_UNSUPPORTED;
    // 32-bit block indices and 64-bit element offsets are used; keep the grid sizes sane
    if ((int64_t)d->batch * d->nheads > (1 << 30)) return SWIMBA_ERR_UNSUPPORTED;
    return SWIMBA_OK;
}

static swimba_status check_mixer(const swimba_dims *d)
{
    swimba_status st = check_common(d);
    if (st != SWIMBA_OK) return st;
    if (d->chunk < 1) return SWIMBA_ERR_SHAPE;
    if (d->chunk > SWIMBA_MAX_CHUNK) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)d->headdim * d->dstate > 8192) return SWIMBA_ERR_UNSUPPORTED;
    const int64_t nc = ((int64_t)d->seqlen + d->chunk - 1) / d->chunk;
    if ((int64_t)d->batch * nc * d->nheads * ((d->chunk + 15) / 16) > (1ll << 31) - 1)
        return SWIMBA_ERR_UNSUPPORTED;
    return SWIMBA_OK;
}

static void layout_of(const swimba_dims *d, swimba_ws_layout *o)
{
    const Shape s = make_shape(d);
    const size_t T = (size_t)s.B * s.L;
    size_t off = 0;
    o->topk_idx = off; off = align_up(off + T * s.K * sizeof(int32_t), 256);
    o->topk_w = off;   off = align_up(off + T * s.K * sizeof(float), 256);
    o->cs = off;       off = align_up(off + (size_t)s.B * s.nc * s.H * s.Q * sizeof(float), 256);
    const bool mf = use_mfma_path(d);
    const size_t Nk = mf ? 128 : (size_t)s.N;   // the MFMA kernels pad the states to 64 x 128
    const size_t Pk = mf ? 64 : (size_t)s.P;
    const size_t nstate = (size_t)s.B * s.nc * s.H * Pk * Nk;
    o->states = off;
    if (!mf) off = align_up(off + nstate * sizeof(float), 256);
    const size_t mixed = (size_t)s.B * s.nc * s.Q * s.G * Nk * sizeof(uint16_t);
    const size_t nt = (size_t)s.Q / 32;
    o->states_lp = off;
    if (mf) off = align_up(off + nstate * sizeof(uint16_t), 256);
    o->cmix = off;
    if (mf) off = align_up(off + mixed, 256);
    o->bmix_t8 = off;
    if (mf) off = align_up(off + mixed, 256);
    o->bmix_frag = off;
    if (mf) off = align_up(off + mixed, 256);
    o->cb = off;
    if (mf) off = align_up(off + (size_t)s.B * s.nc * s.G * (nt * (nt + 1) / 2) * 2048, 256);
    o->cs2 = off;
    if (mf) off = align_up(off + (size_t)s.B * s.nc * s.H * s.Q * sizeof(float), 256);
    o->fdec = off;
    if (mf) off = align_up(off + (size_t)s.B * s.nc * s.H * s.Q * sizeof(float), 256);
    o->cdec = off;
    if (mf) off = align_up(off + (size_t)s.B * s.nc * s.H * s.Q * sizeof(float), 256);
    o->hmid = off;
    if (mf) off = align_up(off + (size_t)s.B * (PASS_SPLIT_MAX_SEGMENTS - 1) * s.H * s.P * s.N * sizeof(float), 256);
    o->total = off > 0 ? off : 256;
}

// compute units of the current device (0 if the query fails); asked once
static int device_cus()
{
    static std::atomic<int> ncu_cache{0};
    int ncu = ncu_cache.load(std::memory_order_relaxed);
    if (ncu == 0) {
        int dev = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&ncu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || ncu <= 0)
            return 0;
        ncu_cache.store(ncu, std::memory_order_relaxed);
    }
    return ncu;
}

// Which evaluation of the SSD part swimba_mixer_fwd takes on the bf16 MFMA path.  A single pass keeps
// one workgroup (one per compute unit: its LDS) busy for the whole sequence of its chain, so it
// needs chains that fill the rounds they run in, and enough chunks per chain to pay for the ramp;
// the staged kernels also parallelise over chunks and win everywhere else.
//   head64   a chain per (batch, head), all channels: 7.5 us per chunk with every compute unit busy,
//            about 6 us with 5/8 of them (the operands come through the same L2s).  Takes the shapes
//            whose B*H chains fill at least 5/8 of their rounds, from 12 chunks on, and those that fill
//            7/8 from 8 chunks on (B8 L2048 H32: 85 against 99 us staged; H24, workload 1: 86 against 85).
//   head64, split: where B*H leaves the rounds emptier than that but 2, 3 or 4 times as many chains
//            fill 7/8 of them, every sequence is cut into that many equal segments of whole chunks (at
//            least 12 each), each a chain of its own: the state at a segment boundary comes from the
//            chunk states in front of it, of which only those that still count there are computed
//            (launch_boundary_states_mfma).  Ahead of slices32: per channel head64 is the cheaper kernel.
//   slices32 a chain per (batch, head, 32 channels): 5.1 us per chunk, i.e. more per channel (the
//            operands a group shares are read per slice), but twice the chains: for the remaining
//            shapes whose slices number between 7/8 of and all of the compute units, from 16 chunks on.
// Measured on MI355X, staged / slices32 / head64 / head64 split in us (device-random inputs, dt and A
// drawn as in the workloads, one input set; mix and prep in front of every variant):
//   B8 L4096 H32 172/184/138/-      B8 L4096 H40 248/243/230/241(2)  B4 L8192 H40 245/293/226/255(4)
//   B8 L4096 H16 104/101/121/-      B4 L8192 H24 137/163/201/162(2)  B8 L2048 H24  81/ 98/ 79/-
//   with 8 groups and 16 experts:   B2 L16384 H64 544/491/550/465(2) B1 L32768 H128 887/797/944/707(2)
//   B1 L16384 H64 297/367/462/267(4)  B2 L8192 H64 290/253/288/241(2)
enum PassKind { PASS_STAGED = 0, PASS_SLICES32 = 1, PASS_HEAD64 = 2 };
// chains fill at least num/8 of the rounds of workgroups (one per compute unit) they run in
static bool fills_rounds(int64_t chains, int ncu, int num)
{
    const int64_t rounds = (chains + ncu - 1) / ncu;
    return chains > 0 && 8 * chains >= num * rounds * ncu;
}
// segments per sequence of the head64 pass (1: whole sequences; 0: head64 does not take the shape)
static int head64_segments(const swimba_dims *d)
{
    const int ncu = device_cus();
    if (ncu == 0 || !use_mfma_path(d) || d->headdim <= 32) return 0;
    const int64_t heads = (int64_t)d->batch * d->nheads;
    const int64_t nc = ((int64_t)d->seqlen + d->chunk - 1) / d->chunk;
    if ((nc >= 12 && fills_rounds(heads, ncu, 5)) || (nc >= 8 && fills_rounds(heads, ncu, 7))) return 1;
    if (nc * d->chunk != d->seqlen) return 0;
    for (int nseg = 2; nseg <= PASS_SPLIT_MAX_SEGMENTS; ++nseg)
        if (nc % nseg == 0 && nc / nseg >= 12 && nc / nseg <= PASS_SPLIT_MAX_CHUNKS &&
            fills_rounds(heads * nseg, ncu, 7))
            return nseg;
    return 0;
}
static PassKind pass_kind(const swimba_dims *d)
{
    const int ncu = device_cus();
    if (ncu == 0 || !use_mfma_path(d)) return PASS_STAGED;
    const int64_t heads = (int64_t)d->batch * d->nheads;
    const int64_t nc = ((int64_t)d->seqlen + d->chunk - 1) / d->chunk;
    if (head64_segments(d) >= 1) return PASS_HEAD64;
    const int64_t slices = heads * ((d->headdim + 31) / 32);
    if (nc >= 16 && slices <= ncu && fills_rounds(slices, ncu, 7)) return PASS_SLICES32;
    return PASS_STAGED;
}

// Router, mixing and G^T tiles per whole chunk in one persistent kernel (no operand image of the mixed B
// rows, no tile pass) in front of a single pass: taken where every compute unit gets at least two
// (batch, chunk, group) items, so that the gather of the next item overlaps the tiles of the current one.
static bool use_chunk_mix(const swimba_dims *d, bool selected)
{
    if (pass_kind(d) == PASS_STAGED) return false;
    swimba_dims dk = *d;
    const Shape s = make_shape(&dk);
    return mix_chunk_covers(s, selected) && (int64_t)s.B * s.nc * s.G >= 2 * (int64_t)device_cus();
}

struct Ws {
    int32_t *idx;
    float *w;
    float *cs;
    float *states;
    void *states_lp, *cmix, *bmix_t8, *bmix_frag, *cb;
    float *cs2, *fdec, *cdec, *hmid;
};

static swimba_status carve(const swimba_dims *d, void *workspace, size_t bytes, Ws *ws)
{
    swimba_status st = check_mixer(d);
    if (st != SWIMBA_OK) return st;
    swimba_ws_layout lo;
    layout_of(d, &lo);
    if (!workspace || bytes < lo.total || ((uintptr_t)workspace & 255u)) return SWIMBA_ERR_WORKSPACE;
    char *p = (char *)workspace;
    ws->idx = (int32_t *)(p + lo.topk_idx);
    ws->w = (float *)(p + lo.topk_w);
    ws->cs = (float *)(p + lo.cs);
    ws->states = (float *)(p + lo.states);
    const bool mf = use_mfma_path(d);
    ws->states_lp = mf ? (void *)(p + lo.states_lp) : nullptr;
    ws->cmix = mf ? (void *)(p + lo.cmix) : nullptr;
    ws->bmix_t8 = mf ? (void *)(p + lo.bmix_t8) : nullptr;
    ws->bmix_frag = mf ? (void *)(p + lo.bmix_frag) : nullptr;
    ws->cb = mf ? (void *)(p + lo.cb) : nullptr;
    ws->cs2 = mf ? (float *)(p + lo.cs2) : nullptr;
    ws->fdec = mf ? (float *)(p + lo.fdec) : nullptr;
    ws->cdec = mf ? (float *)(p + lo.cdec) : nullptr;
    ws->hmid = mf ? (float *)(p + lo.hmid) : nullptr;
    return SWIMBA_OK;
}

}  // namespace swimba

using namespace swimba;

extern "C" {

size_t swimba_mixer_workspace_bytes(const swimba_dims *dims)
{
    if (check_mixer(dims) != SWIMBA_OK) return 0;
    swimba_ws_layout lo;
    layout_of(dims, &lo);
    return lo.total;
}

swimba_status swimba_mixer_workspace_layout(const swimba_dims *dims, swimba_ws_layout *layout)
{
    if (!layout) return SWIMBA_ERR_NULL;
    swimba_status st = check_mixer(dims);
    if (st != SWIMBA_OK) return st;
    layout_of(dims, layout);
    return SWIMBA_OK;
}

swimba_status swimba_router_topk(int64_t tokens, int32_t nexperts, int32_t top_k, int32_t io_dtype,
                                 const void *logits, int32_t *topk_idx, float *topk_w,
                                 void *hip_stream)
{
    if (io_dtype != SWIMBA_F32 && io_dtype != SWIMBA_BF16) return SWIMBA_ERR_DTYPE;
    if (tokens < 0 || nexperts < 1 || top_k < 1 || top_k > nexperts) return SWIMBA_ERR_SHAPE;
    if (nexperts > SWIMBA_MAX_EXPERTS || top_k > SWIMBA_MAX_TOPK || tokens > (1ll << 38))
        return SWIMBA_ERR_UNSUPPORTED;
    if (tokens == 0) return SWIMBA_OK;
    if (!logits || !topk_idx || !topk_w) return SWIMBA_ERR_NULL;
    if (check_align(io_dtype, {}, {logits}, {topk_idx, topk_w}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_router(tokens, nexperts, top_k, io_dtype, logits, topk_idx, topk_w,
                         (hipStream_t)hip_stream);
}

swimba_status swimba_router_linear(int64_t tokens, int32_t d_model, int32_t nexperts, int32_t io_dtype,
                                   const void *u, const void *W_g, void *router_logits, void *hip_stream)
{
    if (io_dtype != SWIMBA_F32 && io_dtype != SWIMBA_BF16) return SWIMBA_ERR_DTYPE;
    if (tokens < 0 || d_model < 1 || nexperts < 1) return SWIMBA_ERR_SHAPE;
    if (nexperts > SWIMBA_MAX_EXPERTS || d_model > 65536 || tokens > (1ll << 38)) return SWIMBA_ERR_UNSUPPORTED;
    if (tokens == 0) return SWIMBA_OK;
    if (!u || !W_g || !router_logits) return SWIMBA_ERR_NULL;
    if (check_align(io_dtype, {u, W_g}, {router_logits}, {}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_router_linear(tokens, d_model, nexperts, io_dtype, u, W_g, router_logits,
                                (hipStream_t)hip_stream);
}

swimba_status swimba_stage_router(const swimba_dims *dims, const void *router_logits,
                                  void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    if (T == 0) return SWIMBA_OK;
    if (!router_logits) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {}, {router_logits}, {}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_router(T, dims->nexperts, dims->top_k, dims->io_dtype, router_logits, ws.idx, ws.w,
                         (hipStream_t)hip_stream);
}

swimba_status swimba_stage_cumsum(const swimba_dims *dims, const void *dt, const float *A,
                                  void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!dt || !A) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {}, {dt}, {A}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    if (use_mfma_path(dims)) return SWIMBA_OK;   // the MFMA chunk-state kernel computes cs itself
    return launch_cumsum(make_shape(dims), dims->io_dtype, dt, A, ws.cs, (hipStream_t)hip_stream);
}

swimba_status swimba_stage_mix(const swimba_dims *dims, const void *B_experts,
                               const void *C_experts, const void *router_logits, void *workspace,
                               size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!B_experts || !C_experts || !router_logits) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {B_experts, C_experts}, {router_logits}, {}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    if (!use_mfma_path(dims)) return SWIMBA_OK;   // the fp32 chunk kernels mix while staging
    return launch_mix_rows_mfma(make_shape(dims), B_experts, C_experts, router_logits, ws.idx, ws.w,
                                ws.cmix, ws.bmix_frag, ws.bmix_t8, -1, -1, nullptr, (hipStream_t)hip_stream);
}

swimba_status swimba_stage_chunk_state(const swimba_dims *dims, const void *x, const void *dt,
                                       const float *A, const void *B_experts, void *workspace,
                                       size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!x || !dt || !A || !B_experts) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x, B_experts}, {dt}, {A}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    const Shape s = make_shape(dims);
    if (use_mfma_path(dims))
        return launch_chunk_state_mfma(s, x, dt, A, ws.bmix_t8, ws.cs, ws.states_lp,
                                       (hipStream_t)hip_stream);
    return launch_chunk_state_generic(s, dims->io_dtype, x, dt, B_experts, ws.idx, ws.w, ws.cs,
                                      ws.states, (hipStream_t)hip_stream);
}

swimba_status swimba_stage_state_scan(const swimba_dims *dims, const float *h0, float *h_final,
                                      void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if (dims->batch == 0) return SWIMBA_OK;
    if (use_mfma_path(dims))
        return launch_scan_cb_mfma(make_shape(dims), h0, h_final, ws.states_lp, ws.cs, ws.cmix,
                                   ws.bmix_frag, ws.cb, (hipStream_t)hip_stream);
    return launch_state_scan(make_shape(dims), h0, h_final, ws.states, nullptr, ws.cs,
                             (hipStream_t)hip_stream);
}

swimba_status swimba_stage_output(const swimba_dims *dims, const void *x, const void *dt,
                                  const float *D, const void *B_experts, const void *C_experts,
                                  void *y, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!x || !dt || !B_experts || !C_experts || !y) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x, B_experts, C_experts, y}, {dt}, {D}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    const Shape s = make_shape(dims);
    if (use_mfma_path(dims))
        return launch_output_mfma(s, x, dt, D, ws.cmix, ws.cb, ws.cs, ws.states_lp, y, nullptr, 0, 0,
                                  (hipStream_t)hip_stream);
    return launch_output_generic(s, dims->io_dtype, x, dt, D, B_experts, C_experts, ws.idx, ws.w,
                                 ws.w, ws.cs, ws.states, y, nullptr, 0, 0, (hipStream_t)hip_stream);
}

int swimba_prefill_path(const swimba_dims *dims)
{
    swimba_status st = check_mixer(dims);
    if (st != SWIMBA_OK) return -(int)st;
    if (!use_mfma_path(dims)) return SWIMBA_PATH_GENERIC;
    const PassKind pk = pass_kind(dims);
    if (pk == PASS_STAGED) {
        const int64_t nc = ((int64_t)dims->seqlen + dims->chunk - 1) / dims->chunk;
        return nc <= OUTPUT_LOOKBACK_MAX_CHUNKS ? SWIMBA_PATH_STAGED_SHORT : SWIMBA_PATH_STAGED;
    }
    const bool cm = use_chunk_mix(dims, false);
    if (pk == PASS_SLICES32) return cm ? SWIMBA_PATH_SINGLE_PASS_CHUNK_MIX : SWIMBA_PATH_SINGLE_PASS;
    if (head64_segments(dims) > 1)
        return cm ? SWIMBA_PATH_SINGLE_PASS_HEAD_SPLIT_CHUNK_MIX : SWIMBA_PATH_SINGLE_PASS_HEAD_SPLIT;
    return cm ? SWIMBA_PATH_SINGLE_PASS_HEAD_CHUNK_MIX : SWIMBA_PATH_SINGLE_PASS_HEAD;
}

int swimba_pass_segments(const swimba_dims *dims)
{
    swimba_status st = check_mixer(dims);
    if (st != SWIMBA_OK) return -(int)st;
    return pass_kind(dims) == PASS_HEAD64 ? head64_segments(dims) : 1;
}

swimba_status swimba_stage_mix_chunk(const swimba_dims *dims, const void *B_experts, const void *C_experts,
                                     const void *router_logits, void *workspace, size_t workspace_bytes,
                                     void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    const Shape s = make_shape(dims);
    if (!use_mfma_path(dims) || !mix_chunk_covers(s, false)) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!B_experts || !C_experts || !router_logits) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {B_experts, C_experts}, {router_logits}, {}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    const int ncu = device_cus();
    if (ncu == 0) return SWIMBA_ERR_HIP;
    return launch_mix_chunk_mfma(s, B_experts, C_experts, router_logits, ws.idx, ws.w, ws.cmix, ws.bmix_t8, ws.cb,
                                 nullptr, ncu, (hipStream_t)hip_stream);
}

swimba_status swimba_stage_tables(const swimba_dims *dims, const void *dt, const float *A, void *workspace,
                                  size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if (!use_mfma_path(dims)) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!dt || !A) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {}, {dt}, {A}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_prep_mfma(make_shape(dims), dt, A, ws.cmix, ws.bmix_frag, ws.cb, ws.cs2, ws.fdec, ws.cdec,
                            (hipStream_t)hip_stream, false);
}

swimba_status swimba_stage_prep(const swimba_dims *dims, const void *dt, const float *A, void *workspace,
                                size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if (!use_mfma_path(dims)) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!dt || !A) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {}, {dt}, {A}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_prep_mfma(make_shape(dims), dt, A, ws.cmix, ws.bmix_frag, ws.cb, ws.cs2, ws.fdec, ws.cdec,
                            (hipStream_t)hip_stream);
}

swimba_status swimba_stage_pass(const swimba_dims *dims, const void *x, const void *dt, const float *D,
                                const float *h0, void *y, float *h_final, void *workspace,
                                size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if (!use_mfma_path(dims)) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!x || !dt || !y) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x, y, h0, h_final}, {dt}, {D}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_pass_mfma(make_shape(dims), x, dt, D, ws.cmix, ws.bmix_t8, ws.cb, ws.cs2, ws.fdec, ws.cdec, h0, h_final,
                            y, (hipStream_t)hip_stream);
}

swimba_status swimba_stage_chunk_state_tiles(const swimba_dims *dims, const void *x, const void *dt, const float *A,
                                             void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if (!use_mfma_path(dims)) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!x || !dt || !A) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x}, {dt}, {A}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_chunk_state_mfma(make_shape(dims), x, dt, A, ws.bmix_t8, ws.cs, ws.states_lp, (hipStream_t)hip_stream,
                                   1, ws.cmix, ws.bmix_frag, ws.cb);
}

swimba_status swimba_stage_output_carry(const swimba_dims *dims, const void *x, const void *dt, const float *D,
                                        const float *h0, void *y, float *h_final, void *workspace,
                                        size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    const Shape s = make_shape(dims);
    if (!use_mfma_path(dims) || s.nc > OUTPUT_LOOKBACK_MAX_CHUNKS) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!x || !dt || !y) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x, y, h0, h_final}, {dt}, {D}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_output_lookback_mfma(s, x, dt, D, ws.cmix, ws.cb, ws.cs, ws.states_lp, y, h0, h_final,
                                       (hipStream_t)hip_stream);
}

swimba_status swimba_stage_pass64(const swimba_dims *dims, const void *x, const void *dt, const float *D,
                                  const float *h0, void *y, float *h_final, void *workspace,
                                  size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if (!use_mfma_path(dims)) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!x || !dt || !y) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x, y, h0, h_final}, {dt}, {D}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_pass64_mfma(make_shape(dims), x, dt, D, ws.cmix, ws.bmix_t8, ws.cb, ws.cs2, ws.fdec, ws.cdec, h0,
                              h_final, y, (hipStream_t)hip_stream);
}

swimba_status swimba_stage_boundary_states(const swimba_dims *dims, const void *x, const void *dt, const float *A,
                                           const float *h0, int32_t nseg, void *workspace, size_t workspace_bytes,
                                           void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if (!use_mfma_path(dims)) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!x || !dt || !A) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x, h0}, {dt}, {A}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_boundary_states_mfma(make_shape(dims), nseg, x, dt, A, ws.bmix_t8, ws.cs2, ws.states_lp, h0, ws.hmid,
                                       (hipStream_t)hip_stream);
}

swimba_status swimba_stage_pass64_split(const swimba_dims *dims, const void *x, const void *dt, const float *D,
                                        const float *h0, void *y, float *h_final, int32_t nseg, void *workspace,
                                        size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    if (!use_mfma_path(dims)) return SWIMBA_ERR_UNSUPPORTED;
    if ((int64_t)dims->batch * dims->seqlen == 0) return SWIMBA_OK;
    if (!x || !dt || !y) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x, y, h0, h_final}, {dt}, {D}) != SWIMBA_OK) return SWIMBA_ERR_ALIGNMENT;
    return launch_pass64_mfma(make_shape(dims), x, dt, D, ws.cmix, ws.bmix_t8, ws.cb, ws.cs2, ws.fdec, ws.cdec, h0,
                              h_final, y, (hipStream_t)hip_stream, nseg, ws.hmid);
}

swimba_status swimba_mixer_fwd(const swimba_dims *dims, const void *x, const void *dt,
                               const float *A, const float *D, const void *B_experts,
                               const void *C_experts, const void *router_logits, const float *h0,
                               void *y, float *h_final, int32_t *topk_idx, float *topk_w,
                               void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    if (T > 0 && (!x || !dt || !A || !B_experts || !C_experts || !router_logits || !y))
        return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x, B_experts, C_experts, y, h0, h_final}, {dt, router_logits},
                    {A, D, topk_idx, topk_w}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    hipStream_t stream = (hipStream_t)hip_stream;
    const Shape s = make_shape(dims);
    const bool mf = use_mfma_path(dims);
    if (T > 0) {
        // On the bf16 MFMA path the mix kernel routes the tokens itself and the chunk-state
        // kernel computes the cumsum itself: two launches fewer.
        if (!mf) {
            st = swimba_stage_router(dims, router_logits, workspace, workspace_bytes, hip_stream);
            if (st != SWIMBA_OK) return st;
            st = swimba_stage_cumsum(dims, dt, A, workspace, workspace_bytes, hip_stream);
            if (st != SWIMBA_OK) return st;
        }
        const bool chunk_mix = use_chunk_mix(dims, false);
        st = chunk_mix ? swimba_stage_mix_chunk(dims, B_experts, C_experts, router_logits, workspace, workspace_bytes,
                                                hip_stream)
                       : swimba_stage_mix(dims, B_experts, C_experts, router_logits, workspace, workspace_bytes,
                                          hip_stream);
        if (st != SWIMBA_OK) return st;
        if (topk_idx || topk_w) {
            const size_t n = (size_t)T * dims->top_k;
            hipError_t e = hipSuccess;
            if (topk_idx)
                e = hipMemcpyAsync(topk_idx, ws.idx, n * sizeof(int32_t), hipMemcpyDeviceToDevice, stream);
            if (e == hipSuccess && topk_w)
                e = hipMemcpyAsync(topk_w, ws.w, n * sizeof(float), hipMemcpyDeviceToDevice, stream);
            if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
        }
        const PassKind pk = pass_kind(dims);
        const bool slices = pk == PASS_SLICES32;
        if (pk != PASS_STAGED) {
            // single pass: G^T tiles and cumsum tables, then one walk over the chunks per
            // (batch, head, 32 channels) or per (batch, head) with the state in registers
            st = launch_prep_mfma(s, dt, A, ws.cmix, ws.bmix_frag, ws.cb, ws.cs2, ws.fdec, ws.cdec, stream, !chunk_mix);
            if (st != SWIMBA_OK) return st;
            if (slices)
                return launch_pass_mfma(s, x, dt, D, ws.cmix, ws.bmix_t8, ws.cb, ws.cs2, ws.fdec, ws.cdec, h0, h_final,
                                        y, stream);
            const int nseg = head64_segments(dims);
            if (nseg > 1) {
                st = launch_boundary_states_mfma(s, nseg, x, dt, A, ws.bmix_t8, ws.cs2, ws.states_lp, h0, ws.hmid,
                                                 stream);
                if (st != SWIMBA_OK) return st;
            }
            return launch_pass64_mfma(s, x, dt, D, ws.cmix, ws.bmix_t8, ws.cb, ws.cs2, ws.fdec, ws.cdec, h0, h_final, y,
                                      stream, nseg, ws.hmid);
        }
        if (mf && s.nc <= OUTPUT_LOOKBACK_MAX_CHUNKS) {
            // short sequences: no scan launch; the G^T tiles ride in the chunk-state launch and every
            // workgroup of the output kernel carries the state up to its own chunk
            st = launch_chunk_state_mfma(s, x, dt, A, ws.bmix_t8, ws.cs, ws.states_lp, stream, 1, ws.cmix,
                                         ws.bmix_frag, ws.cb);
            if (st != SWIMBA_OK) return st;
            return launch_output_lookback_mfma(s, x, dt, D, ws.cmix, ws.cb, ws.cs, ws.states_lp, y, h0, h_final,
                                               stream);
        }
        st = swimba_stage_chunk_state(dims, x, dt, A, B_experts, workspace, workspace_bytes, hip_stream);
        if (st != SWIMBA_OK) return st;
    }
    // with L == 0 the scan only copies h0 (or zeros) to h_final
    if (dims->batch > 0 && (T > 0 || h_final)) {
        st = mf ? launch_scan_cb_mfma(s, h0, h_final, ws.states_lp, ws.cs, ws.cmix, ws.bmix_frag, ws.cb, stream)
                : launch_state_scan(s, h0, h_final, ws.states, nullptr, ws.cs, stream);
        if (st != SWIMBA_OK) return st;
    }
    if (T > 0) {
        st = swimba_stage_output(dims, x, dt, D, B_experts, C_experts, y, workspace, workspace_bytes,
                                 hip_stream);
        if (st != SWIMBA_OK) return st;
    }
    return SWIMBA_OK;
}

// ---- separated-SSM contrast ---------------------------------------------------------------
struct SepLayout {
    size_t mixer, idx1, wb1, wc1, total;
};
static void sep_layout_of(const swimba_dims *d, SepLayout *o)
{
    swimba_ws_layout lo;
    layout_of(d, &lo);
    const size_t T = (size_t)d->batch * d->seqlen;
    size_t off = 0;
    o->mixer = off; off = align_up(off + lo.total, 256);
    o->idx1 = off;  off = align_up(off + T * sizeof(int32_t), 256);
    o->wb1 = off;   off = align_up(off + T * sizeof(float), 256);
    o->wc1 = off;   off = align_up(off + T * sizeof(float), 256);
    o->total = off;
}

size_t swimba_separated_workspace_bytes(const swimba_dims *dims)
{
    if (check_mixer(dims) != SWIMBA_OK) return 0;
    SepLayout sl;
    sep_layout_of(dims, &sl);
    return sl.total;
}

swimba_status swimba_separated_fwd(const swimba_dims *dims, const void *x, const void *dt,
                                   const float *A, const float *D, const void *B_experts,
                                   const void *C_experts, const void *router_logits, void *y,
                                   int32_t *topk_idx, float *topk_w, void *workspace,
                                   size_t workspace_bytes, void *hip_stream)
{
    swimba_status st = check_mixer(dims);
    if (st != SWIMBA_OK) return st;
    SepLayout sl;
    sep_layout_of(dims, &sl);
    if (!workspace || workspace_bytes < sl.total || ((uintptr_t)workspace & 255u)) return SWIMBA_ERR_WORKSPACE;
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    if (T == 0) return SWIMBA_OK;
    if (!x || !dt || !A || !B_experts || !C_experts || !router_logits || !y) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x, B_experts, C_experts, y}, {dt, router_logits}, {A, D, topk_idx, topk_w}) !=
        SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    char *base = (char *)workspace;
    Ws ws;
    swimba_ws_layout lo;
    layout_of(dims, &lo);
    st = carve(dims, base + sl.mixer, lo.total, &ws);
    if (st != SWIMBA_OK) return st;
    int32_t *idx1 = (int32_t *)(base + sl.idx1);
    float *wb1 = (float *)(base + sl.wb1), *wc1 = (float *)(base + sl.wc1);
    hipStream_t stream = (hipStream_t)hip_stream;
    const Shape s = make_shape(dims);
    const bool mf = use_mfma_path(dims);
    Shape s1 = s;
    s1.K = 1;   // one expert at a time on the fp32 kernels
    if (!mf) {
        st = launch_router(T, s.E, s.K, dims->io_dtype, router_logits, ws.idx, ws.w, stream);
        if (st != SWIMBA_OK) return st;
        st = launch_cumsum(s, dims->io_dtype, dt, A, ws.cs, stream);
        if (st != SWIMBA_OK) return st;
    }
    // Expert e's output is added to y by its own output kernel (in the io dtype).  A token's
    // readout weight is zero outside its active set, where the pass adds exact zeros, so a
    // token's y sees k roundings, not E; the skip term D x enters with the last pass, after the
    // small state terms have been summed.
    for (int e = 0; e < s.E; ++e) {
        const float *D_e = (e == s.E - 1) ? D : nullptr;
        const int acc_e = e > 0;
        if (mf) {
            st = launch_mix_rows_mfma(s, B_experts, C_experts, router_logits, ws.idx, ws.w, ws.cmix,
                                      ws.bmix_frag, ws.bmix_t8, e, -1, nullptr, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_chunk_state_mfma(s, x, dt, A, ws.bmix_t8, ws.cs, ws.states_lp, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_scan_cb_mfma(s, nullptr, nullptr, ws.states_lp, ws.cs, ws.cmix, ws.bmix_frag, ws.cb, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_output_mfma(s, x, dt, D_e, ws.cmix, ws.cb, ws.cs, ws.states_lp, y, nullptr, 0, acc_e,
                                    stream);
            if (st != SWIMBA_OK) return st;
        } else {
            st = launch_sep_prepare(s, e, ws.idx, ws.w, idx1, wb1, wc1, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_chunk_state_generic(s1, dims->io_dtype, x, dt, B_experts, idx1, wb1, ws.cs,
                                            ws.states, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_state_scan(s1, nullptr, nullptr, ws.states, nullptr, ws.cs, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_output_generic(s1, dims->io_dtype, x, dt, D_e, B_experts, C_experts, idx1,
                                       wb1, wc1, ws.cs, ws.states, y, nullptr, 0, acc_e, stream);
            if (st != SWIMBA_OK) return st;
        }
    }
    if (topk_idx || topk_w) {
        const size_t cnt = (size_t)T * dims->top_k;
        hipError_t e = hipSuccess;
        if (topk_idx) e = hipMemcpyAsync(topk_idx, ws.idx, cnt * sizeof(int32_t), hipMemcpyDeviceToDevice, stream);
        if (e == hipSuccess && topk_w)
            e = hipMemcpyAsync(topk_w, ws.w, cnt * sizeof(float), hipMemcpyDeviceToDevice, stream);
        if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
    }
    return SWIMBA_OK;
}

// ---- mixed forward with one input stream per expert -----------------------------------------
// Two evaluations.  bf16 MFMA shapes with top_k <= MIX_ALL_SLOTS_MAX: every kernel handles all
// slots in one launch (the mix writes one weighted B image per slot, the chunk-state grid
// carries the slot, the scan sums the slots' chunk states in fp32, the output kernel reads the
// carried state once and walks the slots).  Anything else: k rank-1 passes through the
// one-stream kernels, pass r adding its output to y.
struct XeLayout {
    size_t mixer, xg, wslot, hf, bfragK, t8K, cbK, statesK, total;
    bool slots;
};
static void xe_layout_of(const swimba_dims *d, XeLayout *o, bool selected)
{
    swimba_ws_layout lo;
    layout_of(d, &lo);
    const size_t T = (size_t)d->batch * d->seqlen;
    const size_t n = T * d->nheads * d->headdim;
    const size_t io = d->io_dtype == SWIMBA_BF16 ? 2 : 4;
    const size_t K = d->top_k;
    o->slots = use_mfma_path(d) && d->top_k <= MIX_ALL_SLOTS_MAX;
    size_t off = 0;
    o->mixer = off; off = align_up(off + lo.total, 256);
    // rows of the selected experts: all slots (B,L,k,H,P) for the slot kernels unless the caller
    // brings them, one slot at a time otherwise
    o->xg = off;    off = align_up(off + (o->slots ? (selected ? 0 : n * K * io) : n * io), 256);
    o->wslot = off; off = align_up(off + T * K * sizeof(float), 256);
    o->hf = off;    off = align_up(off + (size_t)d->batch * d->nheads * d->headdim * d->dstate * sizeof(float), 256);
    o->bfragK = o->t8K = o->cbK = o->statesK = off;
    if (o->slots) {
        const size_t nc = ((size_t)d->seqlen + d->chunk - 1) / d->chunk;
        const size_t nbcg = (size_t)d->batch * nc * d->ngroups;
        const size_t NT = d->chunk / 32, NP = NT * (NT + 1) / 2;
        const size_t image = nbcg * d->chunk * 128 * 2;                       // one mixed-B image, bytes
        o->bfragK = off;  off = align_up(off + K * image, 256);
        o->t8K = off;     off = align_up(off + K * image, 256);
        o->cbK = off;     off = align_up(off + K * nbcg * NP * 2048, 256);
        o->statesK = off; off = align_up(off + K * (size_t)d->batch * nc * d->nheads * 64 * 128 * 2, 256);
    }
    o->total = off;
}

size_t swimba_mixer_xe_workspace_bytes(const swimba_dims *dims)
{
    if (check_mixer(dims) != SWIMBA_OK) return 0;
    XeLayout xl;
    xe_layout_of(dims, &xl, false);
    return xl.total;
}

size_t swimba_mixer_xe_selected_workspace_bytes(const swimba_dims *dims)
{
    if (check_mixer(dims) != SWIMBA_OK) return 0;
    XeLayout xl;
    xe_layout_of(dims, &xl, true);
    return xl.total;
}

// x_src: (B,L,E,H,P) with the routing taken from router_logits, or, with w_sel != nullptr, the
// rows of the selected experts (B,L,k,H,P) beside B_src / C_src (B,L,k,G,N) and their weights
static swimba_status xe_core(const swimba_dims *dims, const void *x_src, const void *dt, const float *A,
                             const float *D, const void *B_src, const void *C_src, const void *router_logits,
                             const float *w_sel, const float *h0, void *y, float *h_final, char *base,
                             const XeLayout &xl, hipStream_t stream)
{
    const bool selected = (w_sel != nullptr);
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    Ws ws;
    swimba_ws_layout lo;
    layout_of(dims, &lo);
    swimba_status st = carve(dims, base + xl.mixer, lo.total, &ws);
    if (st != SWIMBA_OK) return st;
    swimba_dims dk = *dims;
    if (selected) dk.nexperts = dims->top_k;        // the kernels see k "experts" with the identity selection
    const Shape s = make_shape(&dk);
    const bool mf = use_mfma_path(dims);
    if (T == 0) {
        // nothing to inject: the final state is the initial one
        if (dims->batch > 0 && h_final)
            return mf ? launch_scan_cb_mfma(s, h0, h_final, ws.states_lp, ws.cs, ws.cmix, ws.bmix_frag, ws.cb, stream)
                      : launch_state_scan(s, h0, h_final, ws.states, nullptr, ws.cs, stream);
        return SWIMBA_OK;
    }
    void *xg = base + xl.xg;
    if (xl.slots) {
        void *bfragK = base + xl.bfragK, *t8K = base + xl.t8K, *cbK = base + xl.cbK, *statesK = base + xl.statesK;
        st = launch_mix_rows_mfma(s, B_src, C_src, router_logits, ws.idx, ws.w, ws.cmix, bfragK, t8K, -1,
                                  MIX_ALL_SLOTS, w_sel, stream);
        if (st != SWIMBA_OK) return st;
        const void *xs = x_src;
        if (!selected) {
            st = launch_xe_gather(s, dims->io_dtype, -1, x_src, ws.idx, xg, stream);
            if (st != SWIMBA_OK) return st;
            xs = xg;
        }
        st = launch_chunk_state_mfma(s, xs, dt, A, t8K, ws.cs, statesK, stream, s.K);
        if (st != SWIMBA_OK) return st;
        st = launch_scan_cb_mfma(s, h0, h_final, statesK, ws.cs, ws.cmix, bfragK, cbK, stream, s.K);
        if (st != SWIMBA_OK) return st;
        return launch_output_slots_mfma(s, xs, dt, D, ws.cmix, cbK, ws.cs, statesK, y, selected ? w_sel : ws.w,
                                        s.K, stream);
    }
    float *wslot = (float *)(base + xl.wslot), *hf_tmp = (float *)(base + xl.hf);
    const int64_t nstate = (int64_t)dims->batch * dims->nheads * dims->headdim * dims->dstate;
    // the selected form runs on the plain-arithmetic kernels (the per-slot MFMA mix routes by itself)
    const bool mfl = mf && !selected;
    const float *wsrc = selected ? w_sel : ws.w;
    if (!mfl) {
        st = selected ? launch_slot_ids(ws.idx, T, dims->top_k, stream)
                      : launch_router(T, s.E, s.K, dims->io_dtype, router_logits, ws.idx, ws.w, stream);
        if (st != SWIMBA_OK) return st;
        st = launch_cumsum(s, dims->io_dtype, dt, A, ws.cs, stream);
        if (st != SWIMBA_OK) return st;
    }
    for (int r = 0; r < s.K; ++r) {
        const float *h0_r = (r == 0) ? h0 : nullptr;       // the initial state enters the sum once
        float *hf_r = !h_final ? nullptr : (r == 0 ? h_final : hf_tmp);
        // pass r adds its output to y; its skip term is D pi_{t,e_r} x_t^(e_r)
        const float *skip_w = wsrc + r;
        if (mfl) {
            st = launch_mix_rows_mfma(s, B_src, C_src, router_logits, ws.idx, ws.w, ws.cmix,
                                      ws.bmix_frag, ws.bmix_t8, -1, r, nullptr, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_xe_gather(s, dims->io_dtype, r, x_src, ws.idx, xg, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_chunk_state_mfma(s, xg, dt, A, ws.bmix_t8, ws.cs, ws.states_lp, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_scan_cb_mfma(s, h0_r, hf_r, ws.states_lp, ws.cs, ws.cmix, ws.bmix_frag, ws.cb, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_output_mfma(s, xg, dt, D, ws.cmix, ws.cb, ws.cs, ws.states_lp, y, skip_w, s.K, r > 0,
                                    stream);
            if (st != SWIMBA_OK) return st;
        } else {
            st = launch_xe_slot_weights(s, r, wsrc, wslot, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_xe_gather(s, dims->io_dtype, r, x_src, ws.idx, xg, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_chunk_state_generic(s, dims->io_dtype, xg, dt, B_src, ws.idx, wslot, ws.cs,
                                            ws.states, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_state_scan(s, h0_r, hf_r, ws.states, nullptr, ws.cs, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_output_generic(s, dims->io_dtype, xg, dt, D, B_src, C_src, ws.idx, wslot,
                                       wsrc, ws.cs, ws.states, y, skip_w, s.K, r > 0, stream);
            if (st != SWIMBA_OK) return st;
        }
        if (h_final && r > 0) {
            st = launch_sep_accumulate(SWIMBA_F32, nstate, hf_tmp, h_final, 0, stream);
            if (st != SWIMBA_OK) return st;
        }
    }
    return SWIMBA_OK;
}

swimba_status swimba_mixer_fwd_xe(const swimba_dims *dims, const void *x_experts, const void *dt,
                                  const float *A, const float *D, const void *B_experts,
                                  const void *C_experts, const void *router_logits, const float *h0,
                                  void *y, float *h_final, int32_t *topk_idx, float *topk_w,
                                  void *workspace, size_t workspace_bytes, void *hip_stream)
{
    swimba_status st = check_mixer(dims);
    if (st != SWIMBA_OK) return st;
    XeLayout xl;
    xe_layout_of(dims, &xl, false);
    if (!workspace || workspace_bytes < xl.total || ((uintptr_t)workspace & 255u)) return SWIMBA_ERR_WORKSPACE;
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    if (T > 0 && (!x_experts || !dt || !A || !B_experts || !C_experts || !router_logits || !y))
        return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x_experts, B_experts, C_experts, y, h0, h_final}, {dt, router_logits},
                    {A, D, topk_idx, topk_w}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    hipStream_t stream = (hipStream_t)hip_stream;
    char *base = (char *)workspace;
    st = xe_core(dims, x_experts, dt, A, D, B_experts, C_experts, router_logits, nullptr, h0, y, h_final, base, xl,
                 stream);
    if (st != SWIMBA_OK) return st;
    if (T > 0 && (topk_idx || topk_w)) {
        swimba_ws_layout lo;
        layout_of(dims, &lo);
        const size_t cnt = (size_t)T * dims->top_k;
        hipError_t e = hipSuccess;
        if (topk_idx)
            e = hipMemcpyAsync(topk_idx, base + xl.mixer + lo.topk_idx, cnt * sizeof(int32_t), hipMemcpyDeviceToDevice,
                               stream);
        if (e == hipSuccess && topk_w)
            e = hipMemcpyAsync(topk_w, base + xl.mixer + lo.topk_w, cnt * sizeof(float), hipMemcpyDeviceToDevice,
                               stream);
        if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
    }
    return SWIMBA_OK;
}

swimba_status swimba_mixer_fwd_xe_selected(const swimba_dims *dims, const void *x_sel, const void *dt,
                                           const float *A, const float *D, const void *B_sel, const void *C_sel,
                                           const float *topk_w, const float *h0, void *y, float *h_final,
                                           void *workspace, size_t workspace_bytes, void *hip_stream)
{
    swimba_status st = check_mixer(dims);
    if (st != SWIMBA_OK) return st;
    XeLayout xl;
    xe_layout_of(dims, &xl, true);
    if (!workspace || workspace_bytes < xl.total || ((uintptr_t)workspace & 255u)) return SWIMBA_ERR_WORKSPACE;
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    if (T > 0 && (!x_sel || !dt || !A || !B_sel || !C_sel || !topk_w || !y)) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x_sel, B_sel, C_sel, y, h0, h_final}, {dt}, {A, D, topk_w}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    return xe_core(dims, x_sel, dt, A, D, B_sel, C_sel, nullptr, topk_w, h0, y, h_final, (char *)workspace, xl,
                   (hipStream_t)hip_stream);
}

// ---- routed expert in-projection --------------------------------------------------------------
struct ProjLayout {
    size_t idx, w, counts, lists, total;
};
static swimba_status proj_layout_of(const swimba_dims *d, int32_t d_model, ProjLayout *o, bool with_x = false)
{
    swimba_status st = check_common(d);
    if (st != SWIMBA_OK) return st;
    if (d_model < 1) return SWIMBA_ERR_SHAPE;
    const int64_t T = (int64_t)d->batch * d->seqlen;
    if (d_model > 65536 || T * d->top_k > (1ll << 31) - 1 || T * d->nexperts > (1ll << 31) - 1)
        return SWIMBA_ERR_UNSUPPORTED;
    // shapes outside the MFMA GEMM run on a kernel that keeps one token's features in LDS as fp32
    const bool gemm = expert_proj_on_mfma(d->io_dtype, d->ngroups * d->dstate, with_x ? d->nheads * d->headdim : 0,
                                          d_model);
    if (!gemm && d_model > SWIMBA_MAX_DMODEL_GENERIC) return SWIMBA_ERR_UNSUPPORTED;
    size_t off = 0;
    o->idx = off;    off = align_up(off + (size_t)T * d->top_k * sizeof(int32_t), 256);
    o->w = off;      off = align_up(off + (size_t)T * d->top_k * sizeof(float), 256);
    o->counts = off; off = align_up(off + SWIMBA_MAX_EXPERTS * sizeof(int32_t), 256);
    o->lists = off;  off = align_up(off + (size_t)T * d->nexperts * sizeof(int32_t), 256);
    o->total = off;
    return SWIMBA_OK;
}

size_t swimba_expert_proj_workspace_bytes(const swimba_dims *dims, int32_t d_model)
{
    ProjLayout pl;
    return proj_layout_of(dims, d_model, &pl) == SWIMBA_OK ? pl.total : 0;
}

static swimba_status expert_proj_body(const swimba_dims *dims, int32_t d_model, const void *u, const void *W_B,
                                      const void *W_C, const void *router_logits, void *B_experts,
                                      void *C_experts, int32_t *topk_idx, float *topk_w, void *workspace,
                                      size_t workspace_bytes, int compact, void *hip_stream,
                                      bool with_x = false, const void *W_X = nullptr, void *x_out = nullptr)
{
    ProjLayout pl;
    swimba_status st = proj_layout_of(dims, d_model, &pl, with_x);
    if (st != SWIMBA_OK) return st;
    if (!workspace || workspace_bytes < pl.total || ((uintptr_t)workspace & 255u)) return SWIMBA_ERR_WORKSPACE;
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    if (T == 0) return SWIMBA_OK;
    if (!u || !W_B || !W_C || !router_logits || !B_experts || !C_experts) return SWIMBA_ERR_NULL;
    if (with_x && (!W_X || !x_out)) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {u, W_B, W_C, B_experts, C_experts, W_X, x_out}, {router_logits},
                    {topk_idx, topk_w}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    char *base = (char *)workspace;
    int32_t *idx = (int32_t *)(base + pl.idx);
    float *w = (float *)(base + pl.w);
    hipStream_t stream = (hipStream_t)hip_stream;
    st = launch_expert_proj(T, dims->nexperts, dims->top_k, dims->ngroups * dims->dstate, d_model, dims->io_dtype,
                            u, W_B, W_C, router_logits, B_experts, C_experts, idx, w,
                            (int32_t *)(base + pl.counts), (int32_t *)(base + pl.lists), compact, stream,
                            with_x ? W_X : nullptr, with_x ? x_out : nullptr, dims->nheads * dims->headdim);
    if (st != SWIMBA_OK) return st;
    if (topk_idx || topk_w) {
        const size_t cnt = (size_t)T * dims->top_k;
        hipError_t e = hipSuccess;
        if (topk_idx) e = hipMemcpyAsync(topk_idx, idx, cnt * sizeof(int32_t), hipMemcpyDeviceToDevice, stream);
        if (e == hipSuccess && topk_w)
            e = hipMemcpyAsync(topk_w, w, cnt * sizeof(float), hipMemcpyDeviceToDevice, stream);
        if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
    }
    return SWIMBA_OK;
}

swimba_status swimba_expert_proj(const swimba_dims *dims, int32_t d_model, const void *u, const void *W_B,
                                 const void *W_C, const void *router_logits, void *B_experts,
                                 void *C_experts, int32_t *topk_idx, float *topk_w, void *workspace,
                                 size_t workspace_bytes, void *hip_stream)
{
    return expert_proj_body(dims, d_model, u, W_B, W_C, router_logits, B_experts, C_experts, topk_idx, topk_w,
                            workspace, workspace_bytes, 0, hip_stream);
}

swimba_status swimba_expert_proj_selected(const swimba_dims *dims, int32_t d_model, const void *u,
                                          const void *W_B, const void *W_C, const void *router_logits,
                                          void *B_sel, void *C_sel, int32_t *topk_idx, float *topk_w,
                                          void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return expert_proj_body(dims, d_model, u, W_B, W_C, router_logits, B_sel, C_sel, topk_idx, topk_w,
                            workspace, workspace_bytes, 1, hip_stream);
}

size_t swimba_expert_proj_x_workspace_bytes(const swimba_dims *dims, int32_t d_model)
{
    ProjLayout pl;
    return proj_layout_of(dims, d_model, &pl, true) == SWIMBA_OK ? pl.total : 0;
}

swimba_status swimba_expert_proj_x_selected(const swimba_dims *dims, int32_t d_model, const void *u,
                                            const void *W_B, const void *W_C, const void *W_X,
                                            const void *router_logits, void *B_sel, void *C_sel, void *x_sel,
                                            int32_t *topk_idx, float *topk_w, void *workspace,
                                            size_t workspace_bytes, void *hip_stream)
{
    return expert_proj_body(dims, d_model, u, W_B, W_C, router_logits, B_sel, C_sel, topk_idx, topk_w,
                            workspace, workspace_bytes, 1, hip_stream, true, W_X, x_sel);
}

// ---- forward on the streams of the selected experts only ---------------------------------------
// B_sel / C_sel (B,L,k,G,N), w_sel (B,L,k).  The fp32 kernels see them as E = k experts with
// the identity selection; the bf16 mix kernel takes the weights instead of routing.
static swimba_status mixer_selected_core(const swimba_dims *dims, const void *x, const void *dt, const float *A,
                                         const float *D, const void *B_sel, const void *C_sel,
                                         const float *w_sel, const float *h0, void *y, float *h_final,
                                         const Ws &ws, hipStream_t stream)
{
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    swimba_dims dk = *dims;
    dk.nexperts = dims->top_k;
    const Shape s = make_shape(&dk);
    const bool mf = use_mfma_path(dims);
    swimba_status st;
    if (T > 0) {
        if (mf) {
            const bool chunk_mix = use_chunk_mix(dims, true);
            st = chunk_mix ? launch_mix_chunk_mfma(s, B_sel, C_sel, nullptr, nullptr, nullptr, ws.cmix, ws.bmix_t8,
                                                   ws.cb, w_sel, device_cus(), stream)
                           : launch_mix_rows_mfma(s, B_sel, C_sel, nullptr, nullptr, nullptr, ws.cmix, ws.bmix_frag,
                                                  ws.bmix_t8, -1, -1, w_sel, stream);
            if (st != SWIMBA_OK) return st;
            const PassKind pk = pass_kind(dims);
            const bool slices = pk == PASS_SLICES32;
            if (pk != PASS_STAGED) {
                st = launch_prep_mfma(s, dt, A, ws.cmix, ws.bmix_frag, ws.cb, ws.cs2, ws.fdec, ws.cdec, stream,
                                      !chunk_mix);
                if (st != SWIMBA_OK) return st;
                if (slices)
                    return launch_pass_mfma(s, x, dt, D, ws.cmix, ws.bmix_t8, ws.cb, ws.cs2, ws.fdec, ws.cdec, h0,
                                            h_final, y, stream);
                const int nseg = head64_segments(dims);
                if (nseg > 1) {
                    st = launch_boundary_states_mfma(s, nseg, x, dt, A, ws.bmix_t8, ws.cs2, ws.states_lp, h0, ws.hmid,
                                                     stream);
                    if (st != SWIMBA_OK) return st;
                }
                return launch_pass64_mfma(s, x, dt, D, ws.cmix, ws.bmix_t8, ws.cb, ws.cs2, ws.fdec, ws.cdec, h0,
                                          h_final, y, stream, nseg, ws.hmid);
            }
            if (s.nc <= OUTPUT_LOOKBACK_MAX_CHUNKS) {
                st = launch_chunk_state_mfma(s, x, dt, A, ws.bmix_t8, ws.cs, ws.states_lp, stream, 1, ws.cmix,
                                             ws.bmix_frag, ws.cb);
                if (st != SWIMBA_OK) return st;
                return launch_output_lookback_mfma(s, x, dt, D, ws.cmix, ws.cb, ws.cs, ws.states_lp, y, h0, h_final,
                                                   stream);
            }
            st = launch_chunk_state_mfma(s, x, dt, A, ws.bmix_t8, ws.cs, ws.states_lp, stream);
        } else {
            st = launch_slot_ids(ws.idx, T, dims->top_k, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_cumsum(s, dims->io_dtype, dt, A, ws.cs, stream);
            if (st != SWIMBA_OK) return st;
            st = launch_chunk_state_generic(s, dims->io_dtype, x, dt, B_sel, ws.idx, w_sel, ws.cs, ws.states,
                                            stream);
        }
        if (st != SWIMBA_OK) return st;
    }
    if (dims->batch > 0 && (T > 0 || h_final)) {
        st = mf ? launch_scan_cb_mfma(s, h0, h_final, ws.states_lp, ws.cs, ws.cmix, ws.bmix_frag, ws.cb, stream)
                : launch_state_scan(s, h0, h_final, ws.states, nullptr, ws.cs, stream);
        if (st != SWIMBA_OK) return st;
    }
    if (T > 0) {
        st = mf ? launch_output_mfma(s, x, dt, D, ws.cmix, ws.cb, ws.cs, ws.states_lp, y, nullptr, 0, 0, stream)
                : launch_output_generic(s, dims->io_dtype, x, dt, D, B_sel, C_sel, ws.idx, w_sel, w_sel, ws.cs,
                                        ws.states, y, nullptr, 0, 0, stream);
        if (st != SWIMBA_OK) return st;
    }
    return SWIMBA_OK;
}

swimba_status swimba_mixer_fwd_selected(const swimba_dims *dims, const void *x, const void *dt, const float *A,
                                        const float *D, const void *B_sel, const void *C_sel,
                                        const float *topk_w, const float *h0, void *y, float *h_final,
                                        void *workspace, size_t workspace_bytes, void *hip_stream)
{
    Ws ws;
    swimba_status st = carve(dims, workspace, workspace_bytes, &ws);
    if (st != SWIMBA_OK) return st;
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    if (T > 0 && (!x || !dt || !A || !B_sel || !C_sel || !topk_w || !y)) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {x, B_sel, C_sel, y, h0, h_final}, {dt}, {A, D, topk_w}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    return mixer_selected_core(dims, x, dt, A, D, B_sel, C_sel, topk_w, h0, y, h_final, ws,
                               (hipStream_t)hip_stream);
}

// ---- in-projection + forward, no tensor with an expert axis in between --------------------------
struct MixProjLayout {
    size_t mixer, bsel, csel, counts, lists, total;
};
static swimba_status mixproj_layout_of(const swimba_dims *d, int32_t d_model, MixProjLayout *o)
{
    swimba_status st = check_mixer(d);
    if (st != SWIMBA_OK) return st;
    ProjLayout pl;
    st = proj_layout_of(d, d_model, &pl);   // limits on d_model and on the list sizes
    if (st != SWIMBA_OK) return st;
    swimba_ws_layout lo;
    layout_of(d, &lo);
    const size_t T = (size_t)d->batch * d->seqlen;
    const size_t io = d->io_dtype == SWIMBA_BF16 ? 2 : 4;
    const size_t sel = T * d->top_k * d->ngroups * d->dstate * io;
    size_t off = 0;
    o->mixer = off;  off = align_up(off + lo.total, 256);
    o->bsel = off;   off = align_up(off + sel, 256);
    o->csel = off;   off = align_up(off + sel, 256);
    o->counts = off; off = align_up(off + SWIMBA_MAX_EXPERTS * sizeof(int32_t), 256);
    o->lists = off;  off = align_up(off + T * d->nexperts * sizeof(int32_t), 256);
    o->total = off;
    return SWIMBA_OK;
}

size_t swimba_mixer_proj_workspace_bytes(const swimba_dims *dims, int32_t d_model)
{
    MixProjLayout ml;
    return mixproj_layout_of(dims, d_model, &ml) == SWIMBA_OK ? ml.total : 0;
}

swimba_status swimba_mixer_fwd_proj(const swimba_dims *dims, int32_t d_model, const void *u, const void *W_B,
                                    const void *W_C, const void *x, const void *dt, const float *A,
                                    const float *D, const void *router_logits, const float *h0, void *y,
                                    float *h_final, int32_t *topk_idx, float *topk_w, void *workspace,
                                    size_t workspace_bytes, void *hip_stream)
{
    MixProjLayout ml;
    swimba_status st = mixproj_layout_of(dims, d_model, &ml);
    if (st != SWIMBA_OK) return st;
    if (!workspace || workspace_bytes < ml.total || ((uintptr_t)workspace & 255u)) return SWIMBA_ERR_WORKSPACE;
    char *base = (char *)workspace;
    Ws ws;
    st = carve(dims, base + ml.mixer, ml.bsel - ml.mixer, &ws);
    if (st != SWIMBA_OK) return st;
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    if (T > 0 && (!u || !W_B || !W_C || !x || !dt || !A || !router_logits || !y)) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {u, W_B, W_C, x, y, h0, h_final}, {dt, router_logits},
                    {A, D, topk_idx, topk_w}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    hipStream_t stream = (hipStream_t)hip_stream;
    void *bsel = base + ml.bsel, *csel = base + ml.csel;
    if (T > 0) {
        st = launch_expert_proj(T, dims->nexperts, dims->top_k, dims->ngroups * dims->dstate, d_model,
                                dims->io_dtype, u, W_B, W_C, router_logits, bsel, csel, ws.idx, ws.w,
                                (int32_t *)(base + ml.counts), (int32_t *)(base + ml.lists), 1, stream);
        if (st != SWIMBA_OK) return st;
        // the selection leaves the workspace before the fp32 kernels reuse its place for slot ids
        if (topk_idx || topk_w) {
            const size_t cnt = (size_t)T * dims->top_k;
            hipError_t e = hipSuccess;
            if (topk_idx)
                e = hipMemcpyAsync(topk_idx, ws.idx, cnt * sizeof(int32_t), hipMemcpyDeviceToDevice, stream);
            if (e == hipSuccess && topk_w)
                e = hipMemcpyAsync(topk_w, ws.w, cnt * sizeof(float), hipMemcpyDeviceToDevice, stream);
            if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
        }
    }
    return mixer_selected_core(dims, x, dt, A, D, bsel, csel, ws.w, h0, y, h_final, ws, stream);
}

// ---- token features -> y with one projected input stream per expert ------------------------------
struct XeProjLayout {
    size_t xe, bsel, csel, xsel, idx, w, counts, lists, total;
};
static swimba_status xeproj_layout_of(const swimba_dims *d, int32_t d_model, XeProjLayout *o, XeLayout *xl)
{
    ProjLayout pl;
    swimba_status st = proj_layout_of(d, d_model, &pl, true);
    if (st != SWIMBA_OK) return st;
    st = check_mixer(d);
    if (st != SWIMBA_OK) return st;
    xe_layout_of(d, xl, true);
    const size_t T = (size_t)d->batch * d->seqlen;
    const size_t io = d->io_dtype == SWIMBA_BF16 ? 2 : 4;
    const size_t sel = T * d->top_k * d->ngroups * d->dstate * io;
    size_t off = 0;
    o->xe = off;     off = align_up(off + xl->total, 256);
    o->bsel = off;   off = align_up(off + sel, 256);
    o->csel = off;   off = align_up(off + sel, 256);
    o->xsel = off;   off = align_up(off + T * d->top_k * d->nheads * d->headdim * io, 256);
    o->idx = off;    off = align_up(off + T * d->top_k * sizeof(int32_t), 256);
    o->w = off;      off = align_up(off + T * d->top_k * sizeof(float), 256);
    o->counts = off; off = align_up(off + SWIMBA_MAX_EXPERTS * sizeof(int32_t), 256);
    o->lists = off;  off = align_up(off + T * d->nexperts * sizeof(int32_t), 256);
    o->total = off;
    return SWIMBA_OK;
}

size_t swimba_mixer_xe_proj_workspace_bytes(const swimba_dims *dims, int32_t d_model)
{
    XeProjLayout ml;
    XeLayout xl;
    return xeproj_layout_of(dims, d_model, &ml, &xl) == SWIMBA_OK ? ml.total : 0;
}

swimba_status swimba_mixer_fwd_xe_proj(const swimba_dims *dims, int32_t d_model, const void *u, const void *W_B,
                                       const void *W_C, const void *W_X, const void *dt, const float *A,
                                       const float *D, const void *router_logits, const float *h0, void *y,
                                       float *h_final, int32_t *topk_idx, float *topk_w, void *workspace,
                                       size_t workspace_bytes, void *hip_stream)
{
    XeProjLayout ml;
    XeLayout xl;
    swimba_status st = xeproj_layout_of(dims, d_model, &ml, &xl);
    if (st != SWIMBA_OK) return st;
    if (!workspace || workspace_bytes < ml.total || ((uintptr_t)workspace & 255u)) return SWIMBA_ERR_WORKSPACE;
    char *base = (char *)workspace;
    const int64_t T = (int64_t)dims->batch * dims->seqlen;
    if (T > 0 && (!u || !W_B || !W_C || !W_X || !dt || !A || !router_logits || !y)) return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {u, W_B, W_C, W_X, y, h0, h_final}, {dt, router_logits},
                    {A, D, topk_idx, topk_w}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    hipStream_t stream = (hipStream_t)hip_stream;
    void *bsel = base + ml.bsel, *csel = base + ml.csel, *xsel = base + ml.xsel;
    int32_t *idx = (int32_t *)(base + ml.idx);
    float *w = (float *)(base + ml.w);
    if (T > 0) {
        st = launch_expert_proj(T, dims->nexperts, dims->top_k, dims->ngroups * dims->dstate, d_model,
                                dims->io_dtype, u, W_B, W_C, router_logits, bsel, csel, idx, w,
                                (int32_t *)(base + ml.counts), (int32_t *)(base + ml.lists), 1, stream, W_X, xsel,
                                dims->nheads * dims->headdim);
        if (st != SWIMBA_OK) return st;
        if (topk_idx || topk_w) {
            const size_t cnt = (size_t)T * dims->top_k;
            hipError_t e = hipSuccess;
            if (topk_idx) e = hipMemcpyAsync(topk_idx, idx, cnt * sizeof(int32_t), hipMemcpyDeviceToDevice, stream);
            if (e == hipSuccess && topk_w)
                e = hipMemcpyAsync(topk_w, w, cnt * sizeof(float), hipMemcpyDeviceToDevice, stream);
            if (e != hipSuccess) { set_last_hip_error((int)e); return SWIMBA_ERR_HIP; }
        }
    }
    return xe_core(dims, xsel, dt, A, D, bsel, csel, nullptr, w, h0, y, h_final, base + ml.xe, xl, stream);
}

size_t swimba_step_workspace_bytes(const swimba_dims *dims)
{
    if (check_common(dims) != SWIMBA_OK || dims->seqlen != 1) return 0;
    const size_t n = (size_t)dims->batch * dims->ngroups * dims->dstate * 2 * sizeof(float);
    return align_up(n > 0 ? n : 1, 256);
}

swimba_status swimba_step(const swimba_dims *dims, const float *state_in, float *state_out,
                          const void *x, const void *dt, const float *A, const float *D,
                          const void *B_experts, const void *C_experts, const void *router_logits,
                          void *y, int32_t *topk_idx, void *workspace, size_t workspace_bytes,
                          void *hip_stream)
{
    swimba_status st = check_common(dims);
    if (st != SWIMBA_OK) return st;
    if (dims->seqlen != 1) return SWIMBA_ERR_SHAPE;
    if (dims->batch == 0) return SWIMBA_OK;
    if (!workspace || workspace_bytes < swimba_step_workspace_bytes(dims) || ((uintptr_t)workspace & 255u))
        return SWIMBA_ERR_WORKSPACE;
    if (!state_in || !state_out || !x || !dt || !A || !B_experts || !C_experts || !router_logits || !y)
        return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {state_in, state_out, x, B_experts, C_experts, y}, {dt, router_logits},
                    {A, D, topk_idx}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    return launch_step(make_shape(dims), dims->io_dtype, state_in, state_out, x, dt, A, D, B_experts,
                       C_experts, router_logits, y, topk_idx, (float *)workspace,
                       (hipStream_t)hip_stream);
}

swimba_status swimba_step_static(const swimba_dims *dims, const float *state_in, float *state_out,
                                 const void *x, const void *dt, const float *A, const float *D,
                                 const void *B_experts, const void *C_experts, const void *router_logits,
                                 void *y, int32_t *topk_idx, void *hip_stream)
{
    swimba_status st = check_common(dims);
    if (st != SWIMBA_OK) return st;
    if (dims->seqlen != 1) return SWIMBA_ERR_SHAPE;
    if (swimba_step_workspace_bytes(dims) > SWIMBA_STATIC_SCRATCH_BYTES) return SWIMBA_ERR_UNSUPPORTED;
    if (dims->batch == 0) return SWIMBA_OK;
    if (!state_in || !state_out || !x || !dt || !A || !B_experts || !C_experts || !router_logits || !y)
        return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {state_in, state_out, x, B_experts, C_experts, y}, {dt, router_logits},
                    {A, D, topk_idx}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    return launch_step_static(make_shape(dims), dims->io_dtype, state_in, state_out, x, dt, A, D, B_experts,
                              C_experts, router_logits, y, topk_idx, (hipStream_t)hip_stream);
}

size_t swimba_step_multi_workspace_bytes(const swimba_dims *dims)
{
    if (check_common(dims) != SWIMBA_OK || dims->seqlen < 1 || dims->seqlen > SWIMBA_MAX_STEP_TOKENS) return 0;
    const size_t n = (size_t)dims->batch * dims->seqlen * dims->ngroups * dims->dstate * 2 * sizeof(float);
    return align_up(n > 0 ? n : 1, 256);
}

swimba_status swimba_step_multi(const swimba_dims *dims, const float *state_in, float *state_out,
                                const void *x, const void *dt, const float *A, const float *D,
                                const void *B_experts, const void *C_experts, const void *router_logits,
                                void *y, int32_t *topk_idx, void *workspace, size_t workspace_bytes,
                                void *hip_stream)
{
    swimba_status st = check_common(dims);
    if (st != SWIMBA_OK) return st;
    if (dims->seqlen < 1) return SWIMBA_ERR_SHAPE;
    if (dims->seqlen > SWIMBA_MAX_STEP_TOKENS) return SWIMBA_ERR_UNSUPPORTED;
    if (dims->batch == 0) return SWIMBA_OK;
    if (!workspace || workspace_bytes < swimba_step_multi_workspace_bytes(dims) || ((uintptr_t)workspace & 255u))
        return SWIMBA_ERR_WORKSPACE;
    if (!state_in || !state_out || !x || !dt || !A || !B_experts || !C_experts || !router_logits || !y)
        return SWIMBA_ERR_NULL;
    if (check_align(dims->io_dtype, {state_in, state_out, x, B_experts, C_experts, y}, {dt, router_logits},
                    {A, D, topk_idx}) != SWIMBA_OK)
        return SWIMBA_ERR_ALIGNMENT;
    return launch_step_multi(make_shape(dims), dims->io_dtype, state_in, state_out, x, dt, A, D, B_experts,
                             C_experts, router_logits, y, topk_idx, (float *)workspace,
                             (hipStream_t)hip_stream);
}

const char *swimba_status_string(swimba_status s)
{
    switch (s) {
    case SWIMBA_OK: return "ok";
    case SWIMBA_ERR_NULL: return "a required pointer is NULL";
    case SWIMBA_ERR_SHAPE: return "invalid or inconsistent dimensions";
    case SWIMBA_ERR_DTYPE: return "unknown io_dtype";
    case SWIMBA_ERR_UNSUPPORTED: return "problem outside the kernels' limits";
    case SWIMBA_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case SWIMBA_ERR_HIP: return "HIP runtime error";
    case SWIMBA_ERR_ALIGNMENT: return "a tensor pointer is not aligned as the header requires";
    }
    return "unknown status";
}

int swimba_last_hip_error(void) { return g_last_hip_error; }

}  // extern "C"
