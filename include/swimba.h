/*
 * swimba.h - C ABI of the MI355X (gfx950) Swimba token-mixer library.
 *
 * The library evaluates the forward hot path of the MoE-parameterized SSM
 * layer: a token-level router (softmax over E experts, top-k, no
 * renormalisation), parameter-space mixing of the expert-produced injection
 * (B) and readout (C) streams, and ONE Mamba-2 style SSD chunked recurrence
 * over the single mixed state trajectory; plus the single-token recurrent
 * decode step.
 *
 * Conventions that hold for every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller (the dims
 *     struct and the layout struct are HOST pointers).  Tensors are dense,
 *     row-major, last index contiguous.  The large tensors (x, y, x_experts, u, the
 *     B/C streams, projection weights, states) must be 16-byte aligned: they are moved
 *     with 16-byte vector accesses; dt, router logits, A, D, topk_idx and topk_w need the
 *     alignment of their element type only.  A misaligned pointer is refused
 *     (SWIMBA_ERR_ALIGNMENT), never dereferenced.
 *   - "io" tensors have the element type dims->io_dtype (fp32 or bf16);
 *     A, D, states, weights are always fp32, indices int32.
 *   - The library allocates no device memory.  Scratch comes from the
 *     caller's workspace, sized by swimba_mixer_workspace_bytes().
 *   - Calls validate their arguments on the host first (a failed call
 *     enqueues nothing), then only enqueue kernels on `hip_stream` (a
 *     hipStream_t passed as void*, NULL = the default stream).  They never
 *     synchronise.  Inputs are never written; outputs are fully overwritten.
 *   - Results do not depend on launch order or atomics: two calls on the same
 *     inputs give bitwise-identical outputs.
 *   - Errors are returned as swimba_status; nothing throws across the ABI.
 *
 * Symbols:  B batch, L seqlen, H heads, P headdim, N state size, G B/C groups
 * (head h reads group floor(h*G/H), H % G == 0), E experts, k = top_k,
 * Q = chunk, nc = ceil(L/Q).
 */
#ifndef SWIMBA_H
#define SWIMBA_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* every entry point below is exported with default visibility */
#pragma GCC visibility push(default)

typedef enum {
    SWIMBA_OK = 0,
    SWIMBA_ERR_NULL = 1,        /* a required pointer is NULL */
    SWIMBA_ERR_SHAPE = 2,       /* non-positive or inconsistent dimensions */
    SWIMBA_ERR_DTYPE = 3,       /* io_dtype is not a swimba_dtype */
    SWIMBA_ERR_UNSUPPORTED = 4, /* valid problem, but outside the kernels' limits */
    SWIMBA_ERR_WORKSPACE = 5,   /* workspace NULL or smaller than the query says */
    SWIMBA_ERR_HIP = 6,         /* a HIP call failed; see swimba_last_hip_error() */
    SWIMBA_ERR_ALIGNMENT = 7    /* a tensor pointer is misaligned (see the conventions above) */
} swimba_status;

typedef enum { SWIMBA_F32 = 0, SWIMBA_BF16 = 1 } swimba_dtype;

/* Limits of the kernels (anything beyond returns SWIMBA_ERR_UNSUPPORTED). */
#define SWIMBA_MAX_EXPERTS 256
#define SWIMBA_MAX_TOPK 16
#define SWIMBA_MAX_DSTATE 256
#define SWIMBA_MAX_HEADDIM 256
#define SWIMBA_MAX_CHUNK 256
#define SWIMBA_MAX_STEP_TOKENS 64   /* tokens per sequence in one swimba_step_multi call */
#define SWIMBA_STATIC_SCRATCH_BYTES (1u << 20) /* scratch held inside the library for swimba_step_static */
#define SWIMBA_MAX_DMODEL_GENERIC 16384 /* feature width of the projection outside its MFMA shapes */

typedef struct {
    int32_t batch, seqlen, nheads, headdim, dstate, ngroups, nexperts, top_k;
    int32_t chunk;    /* SSD chunk length Q in [1, SWIMBA_MAX_CHUNK]; ignored by swimba_step */
    int32_t io_dtype; /* a swimba_dtype */
} swimba_dims;

/* Byte offsets of the scratch arrays inside the workspace (for tests and
 * profiling of single stages; a plain caller only needs `total`). */
typedef struct {
    size_t topk_idx;  /* (B,L,k) int32 : active experts, router order              */
    size_t topk_w;    /* (B,L,k) fp32  : their un-renormalised softmax weights      */
    size_t cs;        /* (B,nc,H,Q) fp32 : inclusive cumsum of dt*A inside each chunk */
    size_t states;    /* (B,nc,H,P,N) fp32 : chunk states S_c, then (after the scan)
                         the state carried INTO chunk c; fp32 path only (empty on the
                         bf16 MFMA path)                                            */
    /* bf16 MFMA path only (each equals the next offset when unused): */
    size_t states_lp; /* (B,nc,H,P,N) bf16 : chunk states S_c, then the carried states  */
    size_t cmix;      /* (B,nc,G,Q/32,8,64,8) bf16 : mixed C rows, MFMA operand layout   */
    size_t bmix_t8;   /* (B,nc,G,Q/8,N,8) bf16 : mixed B, 8 consecutive tokens innermost */
    size_t bmix_frag; /* (B,nc,G,Q/32,8,64,8) bf16 : mixed B rows, MFMA operand layout   */
    size_t cb;        /* (B,nc,G,NP,2,64,8) bf16 : causal 32x32 tiles of Bmix.Cmix^T in
                         MFMA accumulator layout, NP = (Q/32)(Q/32+1)/2               */
    size_t cs2;       /* (B,nc,H,Q) fp32 : log2(e) * cs, table of the single-pass kernel */
    size_t fdec;      /* (B,nc,H,Q) fp32 : dt_j exp(R_J - cs_j), R_J = cs at the end of j's
                         32-token tile; table of the single-pass kernel                  */
    size_t cdec;      /* (B,nc,H,Q) fp32 : dt_j exp(cs_last - cs_j); table of the single-pass kernel */
    size_t hmid;      /* (B,3,H,P,N) fp32 : states at the segment boundaries of the split single pass
                         (nseg - 1 of the 3 are used, densely: (B,nseg-1,H,P,N)) */
    size_t total;
} swimba_ws_layout;

/* Workspace size in bytes for swimba_mixer_fwd / the stage calls; 0 if the
 * dims are invalid or unsupported.  `dims` is a host pointer. */
size_t swimba_mixer_workspace_bytes(const swimba_dims *dims);

/* Fills *layout (host pointer) with the offsets above. */
swimba_status swimba_mixer_workspace_layout(const swimba_dims *dims, swimba_ws_layout *layout);

/*
 * Router (paper: router softmax equation and the top-k rule that follows it).
 *   pi = softmax(logits) over ALL E experts; the k largest logits form the
 *   active set; their softmax values are kept and NOT renormalised.
 * Selection compares the raw stored logits (never the softmax values); equal
 * logits (including +0/-0) go to the lower expert index; the active set is
 * written in (logit descending, index ascending) order.  NaN or +inf logits, and
 * tokens whose logits are all -inf, are outside the contract: indices and weights are
 * then unspecified, but every index stays inside [0, E), so no call reads out of bounds.
 *   logits   (tokens, E) io   [in]
 *   topk_idx (tokens, k) int32 [out]
 *   topk_w   (tokens, k) fp32  [out]
 */
swimba_status swimba_router_topk(int64_t tokens, int32_t nexperts, int32_t top_k, int32_t io_dtype,
                                 const void *logits, int32_t *topk_idx, float *topk_w,
                                 void *hip_stream);

/*
 * Prefill / training-forward of the token mixer (paper: mixed state update
 * and mixed readout equations, Theorem 1; evaluated in the chunked SSD form of
 * the background section "Mamba-2 and SSD"):
 *
 *   Bmix_t = sum_{e in K_t} pi_{t,e} B_t^(e),  Cmix_t likewise
 *   h_t    = exp(dt_t A_h) h_{t-1} + dt_t Bmix_t x_t^T
 *   y_t    = Cmix_t . h_t + D_h x_t                  (state read after its update)
 *
 *   x             (B,L,H,P)   io    [in]
 *   dt            (B,L,H)     io    [in]  final positive step size (no softplus inside)
 *   A             (H)         fp32  [in]  negative scalar transition per head
 *   D             (H)         fp32  [in]  skip coefficient; NULL = 0
 *   B_experts     (B,L,E,G,N) io    [in]
 *   C_experts     (B,L,E,G,N) io    [in]
 *   router_logits (B,L,E)     io    [in]
 *   h0            (B,H,P,N)   fp32  [in]  initial state; NULL = zeros
 *   y             (B,L,H,P)   io    [out]
 *   h_final       (B,H,P,N)   fp32  [out] state after the last token; NULL = not wanted
 *   topk_idx      (B,L,k)     int32 [out] NULL = not wanted
 *   topk_w        (B,L,k)     fp32  [out] NULL = not wanted
 *   workspace     >= swimba_mixer_workspace_bytes(dims) bytes, 256-byte aligned
 *
 * L need not be a multiple of Q (the last chunk is ragged).  B == 0 or L == 0
 * is valid: nothing is computed (h_final = h0 or zeros when L == 0).
 * Arithmetic: fp32 throughout for io_dtype fp32.  For bf16 io with
 * P <= 64 and N <= 128 (multiples of 8; below 64 x 128 the staged inputs, the mixed rows and the
 * states are zero-padded inside the kernels and the workspace) and Q in {64,128,256} the
 * contractions run on bf16 MFMA
 * with fp32 accumulation (mixed streams, decay-weighted x, the C.B^T block, on the diagonal
 * tiles also after the decay mask, and the state carried into a chunk are rounded to bf16
 * as operands; the recurrence between chunks itself runs in fp32 registers);
 * other bf16 shapes use the fp32 kernels.
 */
swimba_status swimba_mixer_fwd(const swimba_dims *dims, const void *x, const void *dt,
                               const float *A, const float *D, const void *B_experts,
                               const void *C_experts, const void *router_logits, const float *h0,
                               void *y, float *h_final, int32_t *topk_idx, float *topk_w,
                               void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The stages of swimba_mixer_fwd, one call each, on the same workspace (for
 * per-kernel measurement and stage-level tests).  Running router, cumsum, mix,
 * chunk_state, state_scan, output in this order computes what swimba_mixer_fwd computes
 * (on the bf16 MFMA path swimba_mixer_fwd itself runs mix, prep, pass: the single-pass
 * evaluation below, same operands and roundings, another summation order).
 *   router      : logits -> ws.topk_idx, ws.topk_w     (no-op on the bf16 MFMA path: mix routes)
 *   cumsum      : dt, A  -> ws.cs   (per-chunk cumsum of dt*A; no-op on the bf16 MFMA path:
 *                 chunk_state computes it)
 *   mix         : bf16 MFMA path only (no-op otherwise): logits, B/C_experts -> ws.topk_*,
 *                 ws.cmix, ws.bmix_frag, ws.bmix_t8 (router + parameter-space mixing)
 *   chunk_state : x, dt, B_experts, ws.{topk_*,cs} -> ws.states = S_c
 *                 S_c = sum_j exp(cs_last - cs_j) dt_j x_j (x) Bmix_j
 *   state_scan  : ws.states (ws.states_lp on the bf16 MFMA path): S_c -> state carried
 *                 into chunk c, in place; h0, ws.cs -> h_final.  The running state is
 *                 fp32 in registers on both paths.  On the bf16 MFMA path the same launch
 *                 also turns ws.cmix, ws.bmix_frag into ws.cb (tiles of Bmix.Cmix^T).
 *   output      : x, dt, D, B/C_experts, ws.* -> y
 *                 y_i = sum_{j<=i} (Cmix_i.Bmix_j) exp(cs_i - cs_j) dt_j x_j
 *                       + exp(cs_i) Cmix_i . H_c + D x_i
 * bf16 MFMA path only (SWIMBA_ERR_UNSUPPORTED otherwise), after mix:
 *   prep        : dt, A, ws.cmix, ws.bmix_frag ->  ws.cb (tiles of Bmix.Cmix^T), ws.cs2, ws.fdec, ws.cdec
 *   pass        : x, dt, D, h0, ws.{cmix,bmix_t8,cb,cs2,fdec,cdec} -> y, h_final.  One workgroup per
 *                 (batch, head, 32 channels) walks the chunks in order with the running state
 *                 in registers: chunk states never reach memory and x is read once.
 */
swimba_status swimba_stage_prep(const swimba_dims *dims, const void *dt, const float *A, void *workspace,
                                size_t workspace_bytes, void *hip_stream);
swimba_status swimba_stage_pass(const swimba_dims *dims, const void *x, const void *dt, const float *D,
                                const float *h0, void *y, float *h_final, void *workspace,
                                size_t workspace_bytes, void *hip_stream);

/* Which kernels swimba_mixer_fwd (and the _selected/_proj forms) run for these dims on the
 * current device: SWIMBA_PATH_GENERIC (fp32-capable kernels, any shape), SWIMBA_PATH_STAGED
 * (bf16 MFMA: mix, chunk_state, state_scan, output; SWIMBA_PATH_STAGED_SHORT for at most 8 chunks,
 * see below), or a single pass over the chunks with the
 * state in registers: SWIMBA_PATH_SINGLE_PASS_HEAD (mix, prep, pass64: a workgroup per (batch,
 * head), taken for head dimensions above 32 when batch * heads fills at least 5/8 of the rounds
 * of workgroups it runs in - one workgroup per compute unit - and the sequence has at least 12
 * chunks, or 7/8 of them from 8 chunks on), SWIMBA_PATH_SINGLE_PASS_HEAD_SPLIT (the same pass on sequences cut into 2, 3 or 4 equal
 * segments of whole chunks, each a chain of its own, see swimba_stage_boundary_states: taken where
 * batch * heads alone leaves the rounds emptier than that but that many times as many chains fill
 * 7/8 of them, the sequence is a whole number of chunks and every segment has at least 12) or
 * SWIMBA_PATH_SINGLE_PASS (mix, prep, pass: a workgroup per (batch, head, 32 channels), taken for
 * the remaining shapes whose slices number between 7/8 of and all of the compute units when the
 * sequence has at least 16 chunks), each also with the chunk-level mix kernel in front
 * (..._CHUNK_MIX, see below).  The results of the MFMA paths agree to the rounding of their
 * bf16 operands.  Returns minus the swimba_status for invalid dims.  Host only; launches
 * nothing. */
#define SWIMBA_PATH_GENERIC 0
#define SWIMBA_PATH_STAGED 1
#define SWIMBA_PATH_SINGLE_PASS 2
#define SWIMBA_PATH_SINGLE_PASS_CHUNK_MIX 3
#define SWIMBA_PATH_SINGLE_PASS_HEAD 4            /* mix, prep, pass64: one workgroup per (batch, head) */
#define SWIMBA_PATH_SINGLE_PASS_HEAD_CHUNK_MIX 5  /* mix_chunk, tables, pass64 */
#define SWIMBA_PATH_STAGED_SHORT 6                /* mix, chunk_state_tiles, output_carry: at most 8 chunks */
#define SWIMBA_PATH_SINGLE_PASS_HEAD_SPLIT 7      /* mix, prep, boundary_states, pass64 on segments */
#define SWIMBA_PATH_SINGLE_PASS_HEAD_SPLIT_CHUNK_MIX 8   /* mix_chunk, tables, boundary_states, pass64 on segments */
int swimba_prefill_path(const swimba_dims *dims);
/* Segments per sequence of the per-head single pass the forward takes for these dims on the current
 * device (1: whole sequences, also on every other path).  Minus the swimba_status for invalid dims. */
int swimba_pass_segments(const swimba_dims *dims);

/* Single pass with the router, the mixing and the tiles of Bmix.Cmix^T done per whole chunk in one
 * persistent kernel (SWIMBA_PATH_SINGLE_PASS_CHUNK_MIX: mix_chunk, tables, pass).  Taken by the forward
 * on single-pass shapes with at most 16 experts, top_k <= 2 and at least two (batch, chunk, group)
 * triples per compute unit; same results as mix + prep, bit for bit.
 *   mix_chunk : B/C_experts, logits -> ws.topk_*, ws.cmix, ws.bmix_t8, ws.cb   (ws.bmix_frag is not written)
 *   tables    : dt, A -> ws.cs2, ws.fdec, ws.cdec                              (prep without the tiles)
 * swimba_stage_mix_chunk runs for any bf16 MFMA shape with nexperts <= 16 and top_k <= 2
 * (SWIMBA_ERR_UNSUPPORTED otherwise). */
swimba_status swimba_stage_mix_chunk(const swimba_dims *dims, const void *B_experts, const void *C_experts,
                                     const void *router_logits, void *workspace, size_t workspace_bytes,
                                     void *hip_stream);
swimba_status swimba_stage_tables(const swimba_dims *dims, const void *dt, const float *A, void *workspace,
                                  size_t workspace_bytes, void *hip_stream);

/* Staged kernels for sequences of at most 8 chunks (SWIMBA_PATH_STAGED_SHORT), without a scan launch:
 *   chunk_state_tiles : chunk_state, and in the same launch ws.cmix, ws.bmix_frag -> ws.cb
 *   output_carry      : output on the CHUNK states in ws.states_lp: the workgroups of chunk c carry the
 *                       state up to c themselves (h0, S_0 .. S_{c-1}, fp32, the scan's order of
 *                       operations); those of the last chunk write h_final.  SWIMBA_ERR_UNSUPPORTED for
 *                       more than 8 chunks. */
swimba_status swimba_stage_chunk_state_tiles(const swimba_dims *dims, const void *x, const void *dt, const float *A,
                                             void *workspace, size_t workspace_bytes, void *hip_stream);
swimba_status swimba_stage_output_carry(const swimba_dims *dims, const void *x, const void *dt, const float *D,
                                        const float *h0, void *y, float *h_final, void *workspace,
                                        size_t workspace_bytes, void *hip_stream);
/* pass with one workgroup per (batch, head) and all channels of the head (up to 64) instead of 32-channel
 * slices: same inputs and outputs as swimba_stage_pass. */
swimba_status swimba_stage_pass64(const swimba_dims *dims, const void *x, const void *dt, const float *D,
                                  const float *h0, void *y, float *h_final, void *workspace,
                                  size_t workspace_bytes, void *hip_stream);
/* Split per-head pass (SWIMBA_PATH_SINGLE_PASS_HEAD_SPLIT): every sequence as nseg (2..4) equal segments
 * of whole chunks (seqlen = nseg * m * chunk, else SWIMBA_ERR_UNSUPPORTED), each walked by a workgroup
 * of its own.  The recurrence of S3.2 is linear in the state, so the state at a segment boundary is
 * sum_c (prod_{c' > c} a_c') S_c over the chunks c in front of it, with S_c the chunk state and a_c =
 * exp(sum of dt*A over chunk c), plus the decayed h0.
 *   boundary_states : x, dt, A, h0, ws.bmix_t8, ws.cs2 -> ws.states_lp (chunk states, bf16, of the
 *                     chunks in front of the last boundary whose factor up to the boundary behind them
 *                     is not exactly zero in fp32; the others are neither computed nor read), then
 *                     ws.hmid (B,nseg-1,H,P,N) fp32.  Two launches.  Needs mix (or mix_chunk) and prep
 *                     (or tables) before it.
 *   pass64_split    : pass64 with batch * nseg * heads workgroups; segment 0 starts from h0, the
 *                     others from ws.hmid; the last segment writes h_final.
 * Both take nseg = 1..4 (boundary_states: 2..4).  Results agree with pass64 to the rounding of the
 * bf16 chunk states (the same rounding the staged path has). */
swimba_status swimba_stage_boundary_states(const swimba_dims *dims, const void *x, const void *dt, const float *A,
                                           const float *h0, int32_t nseg, void *workspace, size_t workspace_bytes,
                                           void *hip_stream);
swimba_status swimba_stage_pass64_split(const swimba_dims *dims, const void *x, const void *dt, const float *D,
                                        const float *h0, void *y, float *h_final, int32_t nseg, void *workspace,
                                        size_t workspace_bytes, void *hip_stream);
swimba_status swimba_stage_router(const swimba_dims *dims, const void *router_logits,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);
swimba_status swimba_stage_cumsum(const swimba_dims *dims, const void *dt, const float *A,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);
swimba_status swimba_stage_mix(const swimba_dims *dims, const void *B_experts,
                               const void *C_experts, const void *router_logits, void *workspace,
                               size_t workspace_bytes, void *hip_stream);
swimba_status swimba_stage_chunk_state(const swimba_dims *dims, const void *x, const void *dt,
                                       const float *A, const void *B_experts, void *workspace,
                                       size_t workspace_bytes, void *hip_stream);
swimba_status swimba_stage_state_scan(const swimba_dims *dims, const float *h0, float *h_final,
                                      void *workspace, size_t workspace_bytes, void *hip_stream);
swimba_status swimba_stage_output(const swimba_dims *dims, const void *x, const void *dt,
                                  const float *D, const void *B_experts, const void *C_experts,
                                  void *y, void *workspace, size_t workspace_bytes,
                                  void *hip_stream);

/*
 * Contrast path: MoE of separated SSMs (paper: section "Alternative: MoE of separated
 * SSMs"): every expert keeps its own state trajectory, all E of them advance on every
 * token with their own un-weighted B stream, and the readout sums the active experts,
 *   h_t^(e) = exp(dt_t A_h) h_{t-1}^(e) + dt_t B_t^(e) x_t^T,
 *   y_t = sum_{e in K_t} pi_{t,e} C_t^(e) . h_t^(e) + D_h x_t          (zero initial states).
 * Same tensors as swimba_mixer_fwd (no h0 / h_final).  It is E plain SSM passes through
 * the mixer's own kernels (one per expert); every pass adds its output to y in the io dtype
 * (outside a token's active set a pass adds exact zeros, so a token's y sees top_k roundings;
 * the skip term enters with the last pass): a measure of what replicating the recurrence
 * costs, not a tuned path.
 *   workspace >= swimba_separated_workspace_bytes(dims), 256-byte aligned.
 */
size_t swimba_separated_workspace_bytes(const swimba_dims *dims);
swimba_status swimba_separated_fwd(const swimba_dims *dims, const void *x, const void *dt,
                                   const float *A, const float *D, const void *B_experts,
                                   const void *C_experts, const void *router_logits, void *y,
                                   int32_t *topk_idx, float *topk_w, void *workspace,
                                   size_t workspace_bytes, void *hip_stream);

/*
 * Mixed forward with one input stream per expert (paper: mixed state update equation as
 * printed, the injection mixes the products B^(e) X^(e)):
 *   h_t = exp(dt_t A_h) h_{t-1} + dt_t sum_{e in K_t} pi_{t,e} x_t^(e) (x) B_t^(e)
 *   y_t = Cmix_t . h_t + D_h xbar_t,   xbar_t = sum_{e in K_t} pi_{t,e} x_t^(e)
 * x_experts (B,L,E,H,P) io; every other argument as in swimba_mixer_fwd.  One state
 * trajectory (the state is linear in the injection).  On the bf16 MFMA shapes with
 * top_k <= 4 the selected rows x^(e_r) are gathered once into (B,L,k,H,P) and every kernel
 * takes all k slots in one launch: one weighted B image per slot, the chunk states of the
 * slots summed in fp32 by the scan, one readout of the carried state and one store of y, the
 * skip term as a contraction with diag(D pi) in two bf16 terms.  Other shapes: k rank-1
 * passes through the one-stream kernels, pass r adding its output to y (in the io dtype) and
 * its final state to h_final (fp32), about k times the time of swimba_mixer_fwd.
 *   workspace >= swimba_mixer_xe_workspace_bytes(dims), 256-byte aligned.
 *
 * swimba_mixer_fwd_xe_selected: the same forward on the rows of the selected experts only, as
 * a projection restricted to the active set produces them (no tensor with an expert axis):
 *   x_sel (B,L,k,H,P) io, B_sel / C_sel (B,L,k,G,N) io, topk_w (B,L,k) fp32 [in]: row r of a
 *   token belongs to its r-th selected expert, topk_w holds the router weights pi_{t,e_r}.
 * No gather; otherwise as above (bf16 MFMA shapes with top_k > 4 run on the plain-arithmetic
 * kernels).  workspace >= swimba_mixer_xe_selected_workspace_bytes(dims), 256-byte aligned.
 */
size_t swimba_mixer_xe_workspace_bytes(const swimba_dims *dims);
swimba_status swimba_mixer_fwd_xe(const swimba_dims *dims, const void *x_experts, const void *dt,
                                  const float *A, const float *D, const void *B_experts,
                                  const void *C_experts, const void *router_logits, const float *h0,
                                  void *y, float *h_final, int32_t *topk_idx, float *topk_w,
                                  void *workspace, size_t workspace_bytes, void *hip_stream);
size_t swimba_mixer_xe_selected_workspace_bytes(const swimba_dims *dims);
swimba_status swimba_mixer_fwd_xe_selected(const swimba_dims *dims, const void *x_sel, const void *dt,
                                           const float *A, const float *D, const void *B_sel, const void *C_sel,
                                           const float *topk_w, const float *h0, void *y, float *h_final,
                                           void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Routing logits as a linear function of the token features (paper: the expressivity theorem
 * takes g a linear function of the features; the Swimba layer's router chooses among the
 * in-projection experts from the token's hidden state):
 *   g_t[e] = sum_d W_g[e][d] u_t[d]                    no bias, fp32 accumulation
 *   u (tokens, d_model) io [in]   W_g (nexperts, d_model) io [in]   router_logits (tokens, nexperts) io [out]
 * The logits are rounded to the io dtype when stored; routing (swimba_router_topk, the mixer,
 * the projection) is defined on those stored values.  With d_model % 8 != 0 and bf16 io the rows
 * of u and W_g are not 16-byte aligned past the first: only the base pointers are checked, the
 * kernel then reads element by element.
 */
swimba_status swimba_router_linear(int64_t tokens, int32_t d_model, int32_t nexperts, int32_t io_dtype,
                                   const void *u, const void *W_g, void *router_logits, void *hip_stream);

/*
 * Routed expert in-projection, the step upstream of the mixer (paper, MoE-parameterized
 * SSM: the expert streams are expert-specific linear projections of the token features;
 * only the active set K_t enters the mix).  For every token t and every e in K_t:
 *   B_t^(e)[g][n] = sum_d W_B[e][g][n][d] u_t[d],   C_t^(e) likewise with W_C.
 *   u             (B,L,d_model) io  token features
 *   W_B, W_C      (E,G,N,d_model) io  projection weights, input index d contiguous
 *   router_logits (B,L,E) io
 *   B_experts, C_experts (B,L,E,G,N) io [out]: the rows of each token's top_k experts are
 *                 written; rows of inactive experts are NOT touched (swimba_mixer_fwd with the
 *                 same logits and top_k never reads them).
 *   topk_idx, topk_w (B,L,k) [out, nullable]
 * Uses dims->batch, seqlen, dstate, ngroups, nexperts, top_k, io_dtype.  bf16 io with
 * d_model % 16 == 0 and (G*N) % 64 == 0 runs as a grouped GEMM on bf16 MFMA (fp32
 * accumulation); anything else on plain fp32 arithmetic, for d_model up to
 * SWIMBA_MAX_DMODEL_GENERIC (the GEMM takes d_model up to 65536; beyond either limit the
 * workspace query returns 0 and the call SWIMBA_ERR_UNSUPPORTED).  The router's linear layer is not
 * part of this call: the logits are an input, so that the routing decision is the caller's.
 *   workspace >= swimba_expert_proj_workspace_bytes(dims, d_model), 256-byte aligned.
 */
size_t swimba_expert_proj_workspace_bytes(const swimba_dims *dims, int32_t d_model);
swimba_status swimba_expert_proj(const swimba_dims *dims, int32_t d_model, const void *u, const void *W_B,
                                 const void *W_C, const void *router_logits, void *B_experts,
                                 void *C_experts, int32_t *topk_idx, float *topk_w, void *workspace,
                                 size_t workspace_bytes, void *hip_stream);

/*
 * The same projection written per selected slot, so that no tensor with an expert axis is
 * ever materialised (paper, MoE-parameterized SSM: only the active set K_t contributes):
 *   B_sel, C_sel (B,L,k,G,N) io [out]: row r of token t is the stream of expert topk_idx[t][r].
 * Every other argument, the arithmetic and the workspace are those of swimba_expert_proj.
 */
swimba_status swimba_expert_proj_selected(const swimba_dims *dims, int32_t d_model, const void *u,
                                          const void *W_B, const void *W_C, const void *router_logits,
                                          void *B_sel, void *C_sel, int32_t *topk_idx, float *topk_w,
                                          void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * The projection with the experts' input streams as a third block of output columns (paper,
 * MoE-parameterized SSM: every expert emits X^(e), B^(e), C^(e) from the token features; the
 * mixed state update as printed injects sum_{e in K_t} pi_{t,e} B^(e) X^(e)):
 *   x_t^(e)[h][p] = sum_d W_X[e][h][p][d] u_t[d]
 *   W_X   (E,H,P,d_model) io [in]    input index d contiguous
 *   x_sel (B,L,k,H,P) io [out]       row r of token t is the stream of expert topk_idx[t][r]
 * B_sel, C_sel and every other argument as in swimba_expert_proj_selected; the three blocks are
 * columns of one grouped GEMM.  The GEMM path additionally needs (H*P) % 64 == 0; dims->nheads
 * and headdim are used.  The outputs feed swimba_mixer_fwd_xe_selected.
 *   workspace >= swimba_expert_proj_x_workspace_bytes(dims, d_model), 256-byte aligned.
 *
 * swimba_mixer_fwd_xe_proj: this projection into the workspace and swimba_mixer_fwd_xe_selected
 * on its outputs in one call, token features -> y with nothing that has an expert axis except
 * the weights.  dt, A, D, h0, y, h_final, topk_idx, topk_w as in swimba_mixer_fwd.
 *   workspace >= swimba_mixer_xe_proj_workspace_bytes(dims, d_model), 256-byte aligned.
 */
size_t swimba_expert_proj_x_workspace_bytes(const swimba_dims *dims, int32_t d_model);
swimba_status swimba_expert_proj_x_selected(const swimba_dims *dims, int32_t d_model, const void *u,
                                            const void *W_B, const void *W_C, const void *W_X,
                                            const void *router_logits, void *B_sel, void *C_sel, void *x_sel,
                                            int32_t *topk_idx, float *topk_w, void *workspace,
                                            size_t workspace_bytes, void *hip_stream);
size_t swimba_mixer_xe_proj_workspace_bytes(const swimba_dims *dims, int32_t d_model);
swimba_status swimba_mixer_fwd_xe_proj(const swimba_dims *dims, int32_t d_model, const void *u, const void *W_B,
                                       const void *W_C, const void *W_X, const void *dt, const float *A,
                                       const float *D, const void *router_logits, const float *h0, void *y,
                                       float *h_final, int32_t *topk_idx, float *topk_w, void *workspace,
                                       size_t workspace_bytes, void *hip_stream);

/*
 * swimba_mixer_fwd on the streams of the selected experts only (paper: parameter-space
 * mixing, Bmix_t = sum_{e in K_t} pi_{t,e} B_t^(e), likewise Cmix; one SSD recurrence):
 *   B_sel, C_sel (B,L,k,G,N) io [in]  row r of a token = stream of its r-th selected expert
 *   topk_w       (B,L,k) fp32  [in]  the router weights pi of those experts (softmax over all
 *                                    E experts, not renormalised); no routing happens here
 * x, dt, A, D, h0, y, h_final as in swimba_mixer_fwd; dims->nexperts only has to be >= top_k.
 *   workspace >= swimba_mixer_workspace_bytes(dims), 256-byte aligned.
 */
swimba_status swimba_mixer_fwd_selected(const swimba_dims *dims, const void *x, const void *dt, const float *A,
                                        const float *D, const void *B_sel, const void *C_sel,
                                        const float *topk_w, const float *h0, void *y, float *h_final,
                                        void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * In-projection and forward in one call (paper, MoE-parameterized SSM followed by the mixed
 * state update): swimba_expert_proj_selected into the workspace, then
 * swimba_mixer_fwd_selected on it.  Arguments as in those two calls; u, W_B, W_C,
 * router_logits, x, dt, A are inputs, y / h_final / topk_idx / topk_w outputs (the last three
 * nullable).  Selected streams are rounded to the io dtype between the two steps.
 *   workspace >= swimba_mixer_proj_workspace_bytes(dims, d_model), 256-byte aligned.
 */
size_t swimba_mixer_proj_workspace_bytes(const swimba_dims *dims, int32_t d_model);
swimba_status swimba_mixer_fwd_proj(const swimba_dims *dims, int32_t d_model, const void *u, const void *W_B,
                                    const void *W_C, const void *x, const void *dt, const float *A,
                                    const float *D, const void *router_logits, const float *h0, void *y,
                                    float *h_final, int32_t *topk_idx, float *topk_w, void *workspace,
                                    size_t workspace_bytes, void *hip_stream);

/*
 * Single-token recurrent decode step (paper: selective SSM recurrence, per
 * channel, with the mixed injection and readout of Theorem 1): for every
 * (b,h)
 *   route and mix token b once;  h' = exp(dt A_h) h + dt x (x) Bmix;
 *   y = h' . Cmix + D_h x.
 * dims->seqlen must be 1; dims->chunk is ignored.
 *   state_in  (B,H,P,N) fp32 [in]   state_out (B,H,P,N) fp32 [out]; they may be
 *             the same buffer (each element is read once, then written, by one lane)
 *   x (B,H,P) io, dt (B,H) io, A (H), D (H)|NULL, B/C_experts (B,E,G,N) io,
 *   router_logits (B,E) io  [in]
 *   y (B,H,P) io [out];  topk_idx (B,k) int32 [out] NULL = not wanted
 *   workspace: >= swimba_step_workspace_bytes(dims) bytes (the mixed streams of the
 *             step, B*G*N*2 fp32), 256-byte aligned; 0 from the query = invalid dims
 * Two kernels are enqueued (routing + mixing, then the state update).  Arithmetic is fp32.
 */
size_t swimba_step_workspace_bytes(const swimba_dims *dims);
swimba_status swimba_step(const swimba_dims *dims, const float *state_in, float *state_out,
                          const void *x, const void *dt, const float *A, const float *D,
                          const void *B_experts, const void *C_experts, const void *router_logits,
                          void *y, int32_t *topk_idx, void *workspace, size_t workspace_bytes,
                          void *hip_stream);

/*
 * swimba_step for callers that cannot allocate or pass a workspace: code under HIP graph
 * capture set up elsewhere, tight serving loops, harnesses that forbid hipMalloc.  Same
 * arguments, kernels and results (bitwise) as swimba_step, without the workspace pair: the
 * step's mixed streams (B*G*N*2 fp32) live in a device array inside the library, of
 * SWIMBA_STATIC_SCRATCH_BYTES bytes per GPU the library runs on (held until the process ends).
 * A step that needs more (swimba_step_workspace_bytes(dims) > SWIMBA_STATIC_SCRATCH_BYTES, i.e.
 * B*G*N > 131072) is refused with SWIMBA_ERR_UNSUPPORTED and enqueues nothing.  The call
 * allocates and frees nothing; the first call on a device looks the array's address up once.
 * Every call on a GPU uses that GPU's one array (each call overwrites all of what it reads, so
 * nothing carries over from the previous call): calls that overlap on one GPU - different
 * streams, or different host threads without ordering between them - race; calls on one
 * stream are ordered and safe.
 */
swimba_status swimba_step_static(const swimba_dims *dims, const float *state_in, float *state_out,
                                 const void *x, const void *dt, const float *A, const float *D,
                                 const void *B_experts, const void *C_experts, const void *router_logits,
                                 void *y, int32_t *topk_idx, void *hip_stream);

/*
 * Several decode tokens per call (the same recurrence as swimba_step, paper: selective SSM
 * recurrence with the router-mixed injection and readout, applied to L = dims->seqlen tokens
 * of every sequence in order): for speculative or short-chunk decoding.  The fp32 state is
 * read once, kept in registers over the L tokens, and written once, so a call moves the same
 * state bytes as a single swimba_step.
 *   state_in/out (B,H,P,N) fp32 (may alias); x (B,L,H,P), dt (B,L,H), B/C_experts (B,L,E,G,N),
 *   router_logits (B,L,E), y (B,L,H,P) [out], topk_idx (B,L,k) [out, nullable]
 *   1 <= L <= SWIMBA_MAX_STEP_TOKENS; workspace >= swimba_step_multi_workspace_bytes(dims).
 * Arithmetic is fp32 like swimba_step.  From about 16 tokens per call on, swimba_mixer_fwd with
 * h0 = the state, h_final = the new state and a chunk of 64 is the faster way to the same result
 * where its bf16 MFMA path applies (at B = H = P = 64, N = 128: 150-160 us for any L up to 64,
 * against 146 / 254 / 450 us here for L = 16 / 32 / 64), at that path's bf16-operand accuracy.
 */
size_t swimba_step_multi_workspace_bytes(const swimba_dims *dims);
swimba_status swimba_step_multi(const swimba_dims *dims, const float *state_in, float *state_out,
                                const void *x, const void *dt, const float *A, const float *D,
                                const void *B_experts, const void *C_experts, const void *router_logits,
                                void *y, int32_t *topk_idx, void *workspace, size_t workspace_bytes,
                                void *hip_stream);

/*
 * Measurement helpers (no paper operation): a plain device copy of `bytes`
 * bytes (multiple of 16) used to calibrate bandwidth figures and profiler
 * counters, and a register-resident bf16 MFMA loop that runs `iters`
 * 32x32x16 MFMAs per wave on `blocks` workgroups of 256 lanes and writes one
 * float per lane to `sink` (blocks*256 floats).
 */
swimba_status swimba_probe_copy(void *dst, const void *src, size_t bytes, void *hip_stream);
swimba_status swimba_probe_mfma(float *sink, int32_t blocks, int32_t iters, void *hip_stream);

const char *swimba_status_string(swimba_status s);
/* hipError_t (as int) of the last SWIMBA_ERR_HIP returned on the calling thread, 0 if none. */
int swimba_last_hip_error(void);

#pragma GCC visibility pop

#ifdef __cplusplus
}
#endif
#endif /* SWIMBA_H */
