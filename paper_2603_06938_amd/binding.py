"""Thin ctypes binding of libswimba.so: argument marshalling only.

Every function has the name and the argument order of the C entry point it
calls (include/swimba.h); torch is used for device memory, dtypes and the
current HIP stream, nothing else.  There is no CPU fallback: if the library
has not been built, or a tensor is not on the GPU, the call raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import NamedTuple, Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libswimba.so")

SWIMBA_F32, SWIMBA_BF16 = 0, 1
MAX_TOPK = 16

_lib = None


class SwimbaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = _load().swimba_status_string(status).decode()
        if status == 6:
            msg += " (hipError %d)" % _load().swimba_last_hip_error()
        super().__init__("%s: %s [status %d]" % (where, msg, status))


class swimba_dims(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("batch", "seqlen", "nheads", "headdim", "dstate", "ngroups", "nexperts", "top_k",
                 "chunk", "io_dtype")]


class swimba_ws_layout(ctypes.Structure):
    _fields_ = [(n, ctypes.c_size_t) for n in
                ("topk_idx", "topk_w", "cs", "states", "states_lp", "cmix", "bmix_t8", "bmix_frag", "cb", "cs2", "fdec", "cdec", "hmid", "total")]


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                "libswimba.so is not built (%s); run `python -c 'import __graft_entry__ as g; g.build()'`"
                % LIB_PATH)
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
        dp = ctypes.POINTER(swimba_dims)
        lib.swimba_mixer_workspace_bytes.restype = sz
        lib.swimba_mixer_workspace_bytes.argtypes = [dp]
        lib.swimba_mixer_workspace_layout.restype = i32
        lib.swimba_mixer_workspace_layout.argtypes = [dp, ctypes.POINTER(swimba_ws_layout)]
        lib.swimba_router_topk.restype = i32
        lib.swimba_router_topk.argtypes = [i64, i32, i32, i32, vp, vp, vp, vp]
        lib.swimba_mixer_fwd.restype = i32
        lib.swimba_mixer_fwd.argtypes = [dp] + [vp] * 12 + [vp, sz, vp]
        lib.swimba_stage_router.restype = i32
        lib.swimba_stage_router.argtypes = [dp, vp, vp, sz, vp]
        lib.swimba_stage_cumsum.restype = i32
        lib.swimba_stage_cumsum.argtypes = [dp, vp, vp, vp, sz, vp]
        lib.swimba_stage_mix.restype = i32
        lib.swimba_stage_mix.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        lib.swimba_stage_chunk_state.restype = i32
        lib.swimba_stage_chunk_state.argtypes = [dp, vp, vp, vp, vp, vp, sz, vp]
        lib.swimba_stage_state_scan.restype = i32
        lib.swimba_stage_state_scan.argtypes = [dp, vp, vp, vp, sz, vp]
        lib.swimba_stage_output.restype = i32
        lib.swimba_stage_output.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.swimba_stage_prep.restype = i32
        lib.swimba_stage_prep.argtypes = [dp, vp, vp, vp, sz, vp]
        lib.swimba_prefill_path.restype = ctypes.c_int
        lib.swimba_prefill_path.argtypes = [dp]
        lib.swimba_stage_mix_chunk.restype = i32
        lib.swimba_stage_mix_chunk.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        lib.swimba_stage_tables.restype = i32
        lib.swimba_stage_tables.argtypes = [dp, vp, vp, vp, sz, vp]
        lib.swimba_stage_pass.restype = i32
        lib.swimba_stage_pass.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.swimba_stage_chunk_state_tiles.restype = i32
        lib.swimba_stage_chunk_state_tiles.argtypes = [dp, vp, vp, vp, vp, sz, vp]
        lib.swimba_stage_output_carry.restype = i32
        lib.swimba_stage_output_carry.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.swimba_stage_pass64.restype = i32
        lib.swimba_stage_pass64.argtypes = [dp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        lib.swimba_pass_segments.restype = ctypes.c_int
        lib.swimba_pass_segments.argtypes = [dp]
        lib.swimba_stage_boundary_states.restype = i32
        lib.swimba_stage_boundary_states.argtypes = [dp, vp, vp, vp, vp, i32, vp, sz, vp]
        lib.swimba_stage_pass64_split.restype = i32
        lib.swimba_stage_pass64_split.argtypes = [dp, vp, vp, vp, vp, vp, vp, i32, vp, sz, vp]
        lib.swimba_separated_workspace_bytes.restype = sz
        lib.swimba_separated_workspace_bytes.argtypes = [dp]
        lib.swimba_separated_fwd.restype = i32
        lib.swimba_separated_fwd.argtypes = [dp] + [vp] * 10 + [vp, sz, vp]
        lib.swimba_step_multi_workspace_bytes.restype = sz
        lib.swimba_step_multi_workspace_bytes.argtypes = [dp]
        lib.swimba_step_multi.restype = i32
        lib.swimba_step_multi.argtypes = [dp] + [vp] * 11 + [vp, sz, vp]
        lib.swimba_expert_proj_workspace_bytes.restype = sz
        lib.swimba_expert_proj_workspace_bytes.argtypes = [dp, i32]
        lib.swimba_expert_proj.restype = i32
        lib.swimba_expert_proj.argtypes = [dp, i32] + [vp] * 8 + [vp, sz, vp]
        lib.swimba_mixer_xe_workspace_bytes.restype = sz
        lib.swimba_router_linear.restype = i32
        lib.swimba_router_linear.argtypes = [i64, i32, i32, i32, vp, vp, vp, vp]
        lib.swimba_expert_proj_selected.restype = i32
        lib.swimba_expert_proj_selected.argtypes = [dp, i32] + [vp] * 8 + [vp, sz, vp]
        lib.swimba_mixer_fwd_selected.restype = i32
        lib.swimba_mixer_fwd_selected.argtypes = [dp] + [vp] * 10 + [vp, sz, vp]
        lib.swimba_mixer_proj_workspace_bytes.restype = sz
        lib.swimba_mixer_proj_workspace_bytes.argtypes = [dp, i32]
        lib.swimba_expert_proj_x_workspace_bytes.restype = sz
        lib.swimba_expert_proj_x_workspace_bytes.argtypes = [dp, i32]
        lib.swimba_expert_proj_x_selected.restype = i32
        lib.swimba_expert_proj_x_selected.argtypes = [dp, i32] + [vp] * 10 + [vp, sz, vp]
        lib.swimba_mixer_xe_proj_workspace_bytes.restype = sz
        lib.swimba_mixer_xe_proj_workspace_bytes.argtypes = [dp, i32]
        lib.swimba_mixer_fwd_xe_proj.restype = i32
        lib.swimba_mixer_fwd_xe_proj.argtypes = [dp, i32] + [vp] * 13 + [vp, sz, vp]
        lib.swimba_mixer_fwd_proj.restype = i32
        lib.swimba_mixer_fwd_proj.argtypes = [dp, i32] + [vp] * 13 + [vp, sz, vp]
        lib.swimba_mixer_xe_workspace_bytes.argtypes = [dp]
        lib.swimba_mixer_fwd_xe.restype = i32
        lib.swimba_mixer_fwd_xe.argtypes = [dp] + [vp] * 12 + [vp, sz, vp]
        lib.swimba_mixer_xe_selected_workspace_bytes.restype = sz
        lib.swimba_mixer_xe_selected_workspace_bytes.argtypes = [dp]
        lib.swimba_mixer_fwd_xe_selected.restype = i32
        lib.swimba_mixer_fwd_xe_selected.argtypes = [dp] + [vp] * 10 + [vp, sz, vp]
        lib.swimba_step_workspace_bytes.restype = sz
        lib.swimba_step_workspace_bytes.argtypes = [dp]
        lib.swimba_step.restype = i32
        lib.swimba_step.argtypes = [dp] + [vp] * 11 + [vp, sz, vp]
        lib.swimba_step_static.restype = i32
        lib.swimba_step_static.argtypes = [dp] + [vp] * 11 + [vp]
        lib.swimba_probe_copy.restype = i32
        lib.swimba_probe_copy.argtypes = [vp, vp, sz, vp]
        lib.swimba_probe_mfma.restype = i32
        lib.swimba_probe_mfma.argtypes = [vp, i32, i32, vp]
        lib.swimba_status_string.restype = ctypes.c_char_p
        lib.swimba_status_string.argtypes = [i32]
        lib.swimba_last_hip_error.restype = i32
        lib.swimba_last_hip_error.argtypes = []
        _lib = lib
    return _lib


def library_loaded() -> bool:
    return _lib is not None


# ---- marshalling helpers -------------------------------------------------------------------

def _io_code(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return SWIMBA_F32
    if t.dtype == torch.bfloat16:
        return SWIMBA_BF16
    raise TypeError("io tensors must be float32 or bfloat16, got %s" % t.dtype)


def _ptr(t: Optional[torch.Tensor], name: str, dtype=None, shape=None) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise ValueError("%s must be a GPU tensor (this library has no CPU path)" % name)
    if not t.is_contiguous():
        raise ValueError("%s must be contiguous" % name)
    if dtype is not None and t.dtype != dtype:
        raise TypeError("%s must have dtype %s, got %s" % (name, dtype, t.dtype))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s must have shape %s, got %s" % (name, tuple(shape), tuple(t.shape)))
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(status: int, where: str) -> None:
    if status != 0:
        raise SwimbaError(status, where)


def make_dims(batch, seqlen, nheads, headdim, dstate, ngroups, nexperts, top_k, chunk, io_dtype) -> swimba_dims:
    if isinstance(io_dtype, torch.dtype):
        io_dtype = {torch.float32: SWIMBA_F32, torch.bfloat16: SWIMBA_BF16}[io_dtype]
    return swimba_dims(batch, seqlen, nheads, headdim, dstate, ngroups, nexperts, top_k, chunk, io_dtype)


def dims_of(x: torch.Tensor, B_experts: torch.Tensor, top_k: int, chunk: int) -> swimba_dims:
    B, L, H, P = x.shape
    _, _, E, G, N = B_experts.shape
    return make_dims(B, L, H, P, N, G, E, top_k, chunk, _io_code(x))


# ---- entry points ----------------------------------------------------------------------

def swimba_mixer_workspace_bytes(dims: swimba_dims) -> int:
    return int(_load().swimba_mixer_workspace_bytes(ctypes.byref(dims)))


def swimba_mixer_workspace_layout(dims: swimba_dims) -> swimba_ws_layout:
    lo = swimba_ws_layout()
    _check(_load().swimba_mixer_workspace_layout(ctypes.byref(dims), ctypes.byref(lo)),
           "swimba_mixer_workspace_layout")
    return lo


def alloc_workspace(dims: swimba_dims, device) -> torch.Tensor:
    n = swimba_mixer_workspace_bytes(dims)
    if n == 0:
        raise SwimbaError(_load().swimba_mixer_workspace_layout(ctypes.byref(dims),
                                                                ctypes.byref(swimba_ws_layout())),
                          "swimba_mixer_workspace_bytes")
    return torch.empty(n, dtype=torch.uint8, device=device)


def swimba_router_topk(router_logits: torch.Tensor, top_k: int, topk_idx=None, topk_w=None):
    E = router_logits.shape[-1]
    tokens = router_logits.numel() // E if E else 0
    lead = tuple(router_logits.shape[:-1])
    if topk_idx is None:
        topk_idx = torch.empty(lead + (top_k,), dtype=torch.int32, device=router_logits.device)
    if topk_w is None:
        topk_w = torch.empty(lead + (top_k,), dtype=torch.float32, device=router_logits.device)
    _check(_load().swimba_router_topk(tokens, E, top_k, _io_code(router_logits),
                                      _ptr(router_logits, "router_logits"),
                                      _ptr(topk_idx, "topk_idx", torch.int32, lead + (top_k,)),
                                      _ptr(topk_w, "topk_w", torch.float32, lead + (top_k,)), _stream()),
           "swimba_router_topk")
    return topk_idx, topk_w


class MixerOut(NamedTuple):
    y: torch.Tensor
    h_final: Optional[torch.Tensor]
    topk_idx: Optional[torch.Tensor]
    topk_w: Optional[torch.Tensor]


def swimba_mixer_fwd(x, dt, A, D, B_experts, C_experts, router_logits, top_k: int, chunk: int,
                     h0=None, *, y=None, h_final=None, topk_idx=None, topk_w=None, workspace=None,
                     want_h_final: bool = True, want_topk: bool = False) -> MixerOut:
    d = dims_of(x, B_experts, top_k, chunk)
    B, L, H, P, N, G, E = d.batch, d.seqlen, d.nheads, d.headdim, d.dstate, d.ngroups, d.nexperts
    io = x.dtype
    dev = x.device
    if workspace is None:
        workspace = alloc_workspace(d, dev)
    if y is None:
        y = torch.empty_like(x)
    if h_final is None and want_h_final:
        h_final = torch.empty((B, H, P, N), dtype=torch.float32, device=dev)
    if want_topk and topk_idx is None:
        topk_idx = torch.empty((B, L, top_k), dtype=torch.int32, device=dev)
    if want_topk and topk_w is None:
        topk_w = torch.empty((B, L, top_k), dtype=torch.float32, device=dev)
    st = _load().swimba_mixer_fwd(
        ctypes.byref(d), _ptr(x, "x", io, (B, L, H, P)), _ptr(dt, "dt", io, (B, L, H)),
        _ptr(A, "A", torch.float32, (H,)), _ptr(D, "D", torch.float32, (H,)),
        _ptr(B_experts, "B_experts", io, (B, L, E, G, N)),
        _ptr(C_experts, "C_experts", io, (B, L, E, G, N)),
        _ptr(router_logits, "router_logits", io, (B, L, E)),
        _ptr(h0, "h0", torch.float32, (B, H, P, N)), _ptr(y, "y", io, (B, L, H, P)),
        _ptr(h_final, "h_final", torch.float32, (B, H, P, N)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, L, top_k)),
        _ptr(topk_w, "topk_w", torch.float32, (B, L, top_k)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_mixer_fwd")
    return MixerOut(y, h_final, topk_idx, topk_w)


def swimba_router_linear(u, W_g, router_logits=None) -> torch.Tensor:
    """u (..., Dm), W_g (E, Dm) -> routing logits (..., E) in the io dtype."""
    Dm = u.shape[-1]
    E = W_g.shape[0]
    tokens = u.numel() // Dm if Dm else 0
    if router_logits is None:
        router_logits = torch.empty(tuple(u.shape[:-1]) + (E,), dtype=u.dtype, device=u.device)
    st = _load().swimba_router_linear(tokens, Dm, E, _io_code(u), _ptr(u, "u"), _ptr(W_g, "W_g", u.dtype, (E, Dm)),
                                      _ptr(router_logits, "router_logits", u.dtype, tuple(u.shape[:-1]) + (E,)),
                                      _stream())
    _check(st, "swimba_router_linear")
    return router_logits


def swimba_expert_proj_workspace_bytes(dims: swimba_dims, d_model: int) -> int:
    return int(_load().swimba_expert_proj_workspace_bytes(ctypes.byref(dims), d_model))


class ProjOut(NamedTuple):
    B_experts: torch.Tensor
    C_experts: torch.Tensor
    topk_idx: Optional[torch.Tensor]
    topk_w: Optional[torch.Tensor]


def swimba_expert_proj(u, W_B, W_C, router_logits, top_k: int, *, B_experts=None, C_experts=None,
                       workspace=None, want_topk: bool = False) -> ProjOut:
    """u (B,L,Dm), W_B/W_C (E,G,N,Dm), router_logits (B,L,E) -> B_experts, C_experts (B,L,E,G,N) with
    the rows of the active experts written (new outputs start as zeros)."""
    B, L, Dm = u.shape
    E, G, N, _ = W_B.shape
    io, dev = u.dtype, u.device
    d = make_dims(B, L, G, 1, N, G, E, top_k, 1, _io_code(u))
    if workspace is None:
        n = swimba_expert_proj_workspace_bytes(d, Dm)
        if n == 0:
            raise SwimbaError(2, "swimba_expert_proj_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    if B_experts is None:
        B_experts = torch.zeros((B, L, E, G, N), dtype=io, device=dev)
    if C_experts is None:
        C_experts = torch.zeros((B, L, E, G, N), dtype=io, device=dev)
    topk_idx = torch.empty((B, L, top_k), dtype=torch.int32, device=dev) if want_topk else None
    topk_w = torch.empty((B, L, top_k), dtype=torch.float32, device=dev) if want_topk else None
    st = _load().swimba_expert_proj(
        ctypes.byref(d), Dm, _ptr(u, "u", io, (B, L, Dm)), _ptr(W_B, "W_B", io, (E, G, N, Dm)),
        _ptr(W_C, "W_C", io, (E, G, N, Dm)), _ptr(router_logits, "router_logits", io, (B, L, E)),
        _ptr(B_experts, "B_experts", io, (B, L, E, G, N)), _ptr(C_experts, "C_experts", io, (B, L, E, G, N)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, L, top_k)), _ptr(topk_w, "topk_w", torch.float32, (B, L, top_k)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_expert_proj")
    return ProjOut(B_experts, C_experts, topk_idx, topk_w)


def swimba_expert_proj_selected(u, W_B, W_C, router_logits, top_k: int, *, B_sel=None, C_sel=None,
                                workspace=None, want_topk: bool = True) -> ProjOut:
    """Like swimba_expert_proj, but the outputs are (B,L,k,G,N): row r = stream of the r-th selected expert."""
    B, L, Dm = u.shape
    E, G, N, _ = W_B.shape
    io, dev = u.dtype, u.device
    d = make_dims(B, L, G, 1, N, G, E, top_k, 1, _io_code(u))
    if workspace is None:
        n = swimba_expert_proj_workspace_bytes(d, Dm)
        if n == 0:
            raise SwimbaError(2, "swimba_expert_proj_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    if B_sel is None:
        B_sel = torch.empty((B, L, top_k, G, N), dtype=io, device=dev)
    if C_sel is None:
        C_sel = torch.empty((B, L, top_k, G, N), dtype=io, device=dev)
    topk_idx = torch.empty((B, L, top_k), dtype=torch.int32, device=dev) if want_topk else None
    topk_w = torch.empty((B, L, top_k), dtype=torch.float32, device=dev) if want_topk else None
    st = _load().swimba_expert_proj_selected(
        ctypes.byref(d), Dm, _ptr(u, "u", io, (B, L, Dm)), _ptr(W_B, "W_B", io, (E, G, N, Dm)),
        _ptr(W_C, "W_C", io, (E, G, N, Dm)), _ptr(router_logits, "router_logits", io, (B, L, E)),
        _ptr(B_sel, "B_sel", io, (B, L, top_k, G, N)), _ptr(C_sel, "C_sel", io, (B, L, top_k, G, N)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, L, top_k)), _ptr(topk_w, "topk_w", torch.float32, (B, L, top_k)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_expert_proj_selected")
    return ProjOut(B_sel, C_sel, topk_idx, topk_w)


def swimba_expert_proj_x_workspace_bytes(dims: swimba_dims, d_model: int) -> int:
    return int(_load().swimba_expert_proj_x_workspace_bytes(ctypes.byref(dims), d_model))


def swimba_expert_proj_x_selected(u, W_B, W_C, W_X, router_logits, top_k: int, *, workspace=None,
                                  want_topk: bool = True):
    """Routed projection of the B, C and input streams of the selected experts:
    u (B,L,Dm), W_B/W_C (E,G,N,Dm), W_X (E,H,P,Dm) -> B_sel, C_sel (B,L,k,G,N), x_sel (B,L,k,H,P), topk_idx, topk_w."""
    B, L, Dm = u.shape
    E, G, N, _ = W_B.shape
    _, H, P, _ = W_X.shape
    io, dev = u.dtype, u.device
    d = make_dims(B, L, H, P, N, G, E, top_k, 1, _io_code(u))
    if workspace is None:
        n = swimba_expert_proj_x_workspace_bytes(d, Dm)
        if n == 0:
            raise SwimbaError(2, "swimba_expert_proj_x_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    B_sel = torch.empty((B, L, top_k, G, N), dtype=io, device=dev)
    C_sel = torch.empty((B, L, top_k, G, N), dtype=io, device=dev)
    x_sel = torch.empty((B, L, top_k, H, P), dtype=io, device=dev)
    topk_idx = torch.empty((B, L, top_k), dtype=torch.int32, device=dev) if want_topk else None
    topk_w = torch.empty((B, L, top_k), dtype=torch.float32, device=dev) if want_topk else None
    st = _load().swimba_expert_proj_x_selected(
        ctypes.byref(d), Dm, _ptr(u, "u", io, (B, L, Dm)), _ptr(W_B, "W_B", io, (E, G, N, Dm)),
        _ptr(W_C, "W_C", io, (E, G, N, Dm)), _ptr(W_X, "W_X", io, (E, H, P, Dm)),
        _ptr(router_logits, "router_logits", io, (B, L, E)),
        _ptr(B_sel, "B_sel", io, (B, L, top_k, G, N)), _ptr(C_sel, "C_sel", io, (B, L, top_k, G, N)),
        _ptr(x_sel, "x_sel", io, (B, L, top_k, H, P)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, L, top_k)), _ptr(topk_w, "topk_w", torch.float32, (B, L, top_k)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_expert_proj_x_selected")
    return B_sel, C_sel, x_sel, topk_idx, topk_w


def swimba_mixer_xe_proj_workspace_bytes(dims: swimba_dims, d_model: int) -> int:
    return int(_load().swimba_mixer_xe_proj_workspace_bytes(ctypes.byref(dims), d_model))


def swimba_mixer_fwd_xe_proj(u, W_B, W_C, W_X, dt, A, D, router_logits, top_k: int, chunk: int, h0=None, *, y=None,
                             h_final=None, workspace=None, want_h_final: bool = True,
                             want_topk: bool = False) -> MixerOut:
    """Token features -> y with one projected input stream per expert (projection + expert-X forward in one call)."""
    B, L, Dm = u.shape
    E, G, N, _ = W_B.shape
    _, H, P, _ = W_X.shape
    io, dev = u.dtype, u.device
    d = make_dims(B, L, H, P, N, G, E, top_k, chunk, _io_code(u))
    if workspace is None:
        n = swimba_mixer_xe_proj_workspace_bytes(d, Dm)
        if n == 0:
            raise SwimbaError(2, "swimba_mixer_xe_proj_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    if y is None:
        y = torch.empty((B, L, H, P), dtype=io, device=dev)
    if h_final is None and want_h_final:
        h_final = torch.empty((B, H, P, N), dtype=torch.float32, device=dev)
    topk_idx = torch.empty((B, L, top_k), dtype=torch.int32, device=dev) if want_topk else None
    topk_w = torch.empty((B, L, top_k), dtype=torch.float32, device=dev) if want_topk else None
    st = _load().swimba_mixer_fwd_xe_proj(
        ctypes.byref(d), Dm, _ptr(u, "u", io, (B, L, Dm)), _ptr(W_B, "W_B", io, (E, G, N, Dm)),
        _ptr(W_C, "W_C", io, (E, G, N, Dm)), _ptr(W_X, "W_X", io, (E, H, P, Dm)), _ptr(dt, "dt", io, (B, L, H)),
        _ptr(A, "A", torch.float32, (H,)), _ptr(D, "D", torch.float32, (H,)),
        _ptr(router_logits, "router_logits", io, (B, L, E)), _ptr(h0, "h0", torch.float32, (B, H, P, N)),
        _ptr(y, "y", io, (B, L, H, P)), _ptr(h_final, "h_final", torch.float32, (B, H, P, N)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, L, top_k)), _ptr(topk_w, "topk_w", torch.float32, (B, L, top_k)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_mixer_fwd_xe_proj")
    return MixerOut(y, h_final, topk_idx, topk_w)


def swimba_mixer_fwd_selected(x, dt, A, D, B_sel, C_sel, topk_w, chunk: int, h0=None, *, y=None, h_final=None,
                              workspace=None, want_h_final: bool = True) -> MixerOut:
    """Mixer forward on the selected experts' streams B_sel/C_sel (B,L,k,G,N) with given weights (B,L,k)."""
    B, L, H, P = x.shape
    _, _, K, G, N = B_sel.shape
    io, dev = x.dtype, x.device
    d = make_dims(B, L, H, P, N, G, K, K, chunk, _io_code(x))
    if workspace is None:
        workspace = alloc_workspace(d, dev)
    if y is None:
        y = torch.empty_like(x)
    if h_final is None and want_h_final:
        h_final = torch.empty((B, H, P, N), dtype=torch.float32, device=dev)
    st = _load().swimba_mixer_fwd_selected(
        ctypes.byref(d), _ptr(x, "x", io, (B, L, H, P)), _ptr(dt, "dt", io, (B, L, H)),
        _ptr(A, "A", torch.float32, (H,)), _ptr(D, "D", torch.float32, (H,)),
        _ptr(B_sel, "B_sel", io, (B, L, K, G, N)), _ptr(C_sel, "C_sel", io, (B, L, K, G, N)),
        _ptr(topk_w, "topk_w", torch.float32, (B, L, K)), _ptr(h0, "h0", torch.float32, (B, H, P, N)),
        _ptr(y, "y", io, (B, L, H, P)), _ptr(h_final, "h_final", torch.float32, (B, H, P, N)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_mixer_fwd_selected")
    return MixerOut(y, h_final, None, None)


def swimba_mixer_proj_workspace_bytes(dims: swimba_dims, d_model: int) -> int:
    return int(_load().swimba_mixer_proj_workspace_bytes(ctypes.byref(dims), d_model))


def swimba_mixer_fwd_proj(u, W_B, W_C, x, dt, A, D, router_logits, top_k: int, chunk: int, h0=None, *, y=None,
                          h_final=None, workspace=None, want_h_final: bool = True,
                          want_topk: bool = False) -> MixerOut:
    """In-projection of the selected experts and the mixer forward in one call; u (B,L,Dm), W (E,G,N,Dm)."""
    B, L, H, P = x.shape
    E, G, N, Dm = W_B.shape
    io, dev = x.dtype, x.device
    d = make_dims(B, L, H, P, N, G, E, top_k, chunk, _io_code(x))
    if workspace is None:
        n = swimba_mixer_proj_workspace_bytes(d, Dm)
        if n == 0:
            alloc_workspace(d, dev)   # raises with the status of the dims
            raise SwimbaError(2, "swimba_mixer_proj_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    if y is None:
        y = torch.empty_like(x)
    if h_final is None and want_h_final:
        h_final = torch.empty((B, H, P, N), dtype=torch.float32, device=dev)
    topk_idx = torch.empty((B, L, top_k), dtype=torch.int32, device=dev) if want_topk else None
    topk_w = torch.empty((B, L, top_k), dtype=torch.float32, device=dev) if want_topk else None
    st = _load().swimba_mixer_fwd_proj(
        ctypes.byref(d), Dm, _ptr(u, "u", io, (B, L, Dm)), _ptr(W_B, "W_B", io, (E, G, N, Dm)),
        _ptr(W_C, "W_C", io, (E, G, N, Dm)), _ptr(x, "x", io, (B, L, H, P)), _ptr(dt, "dt", io, (B, L, H)),
        _ptr(A, "A", torch.float32, (H,)), _ptr(D, "D", torch.float32, (H,)),
        _ptr(router_logits, "router_logits", io, (B, L, E)), _ptr(h0, "h0", torch.float32, (B, H, P, N)),
        _ptr(y, "y", io, (B, L, H, P)), _ptr(h_final, "h_final", torch.float32, (B, H, P, N)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, L, top_k)), _ptr(topk_w, "topk_w", torch.float32, (B, L, top_k)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_mixer_fwd_proj")
    return MixerOut(y, h_final, topk_idx, topk_w)


def swimba_mixer_xe_workspace_bytes(dims: swimba_dims) -> int:
    return int(_load().swimba_mixer_xe_workspace_bytes(ctypes.byref(dims)))


def swimba_mixer_fwd_xe(x_experts, dt, A, D, B_experts, C_experts, router_logits, top_k: int, chunk: int,
                        h0=None, *, y=None, h_final=None, topk_idx=None, topk_w=None, workspace=None,
                        want_h_final: bool = True, want_topk: bool = False) -> MixerOut:
    """Mixed forward with one input stream per expert, x_experts (B,L,E,H,P)."""
    B, L, E, H, P = x_experts.shape
    io, dev = x_experts.dtype, x_experts.device
    _, _, _, G, N = B_experts.shape
    d = make_dims(B, L, H, P, N, G, E, top_k, chunk, _io_code(x_experts))
    if workspace is None:
        n = swimba_mixer_xe_workspace_bytes(d)
        if n == 0:
            alloc_workspace(d, dev)   # raises with the status of the dims
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    if y is None:
        y = torch.empty((B, L, H, P), dtype=io, device=dev)
    if h_final is None and want_h_final:
        h_final = torch.empty((B, H, P, N), dtype=torch.float32, device=dev)
    if want_topk and topk_idx is None:
        topk_idx = torch.empty((B, L, top_k), dtype=torch.int32, device=dev)
    if want_topk and topk_w is None:
        topk_w = torch.empty((B, L, top_k), dtype=torch.float32, device=dev)
    st = _load().swimba_mixer_fwd_xe(
        ctypes.byref(d), _ptr(x_experts, "x_experts", io, (B, L, E, H, P)), _ptr(dt, "dt", io, (B, L, H)),
        _ptr(A, "A", torch.float32, (H,)), _ptr(D, "D", torch.float32, (H,)),
        _ptr(B_experts, "B_experts", io, (B, L, E, G, N)),
        _ptr(C_experts, "C_experts", io, (B, L, E, G, N)),
        _ptr(router_logits, "router_logits", io, (B, L, E)),
        _ptr(h0, "h0", torch.float32, (B, H, P, N)), _ptr(y, "y", io, (B, L, H, P)),
        _ptr(h_final, "h_final", torch.float32, (B, H, P, N)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, L, top_k)),
        _ptr(topk_w, "topk_w", torch.float32, (B, L, top_k)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_mixer_fwd_xe")
    return MixerOut(y, h_final, topk_idx, topk_w)


def swimba_mixer_xe_selected_workspace_bytes(dims: swimba_dims) -> int:
    return int(_load().swimba_mixer_xe_selected_workspace_bytes(ctypes.byref(dims)))


def swimba_mixer_fwd_xe_selected(x_sel, dt, A, D, B_sel, C_sel, topk_w, chunk: int, h0=None, *, y=None,
                                 h_final=None, workspace=None, want_h_final: bool = True) -> MixerOut:
    """Expert-X forward on the selected experts' rows: x_sel (B,L,k,H,P), B_sel/C_sel (B,L,k,G,N), topk_w (B,L,k)."""
    B, L, K, H, P = x_sel.shape
    _, _, _, G, N = B_sel.shape
    io, dev = x_sel.dtype, x_sel.device
    d = make_dims(B, L, H, P, N, G, K, K, chunk, _io_code(x_sel))
    if workspace is None:
        n = swimba_mixer_xe_selected_workspace_bytes(d)
        if n == 0:
            alloc_workspace(d, dev)   # raises with the status of the dims
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    if y is None:
        y = torch.empty((B, L, H, P), dtype=io, device=dev)
    if h_final is None and want_h_final:
        h_final = torch.empty((B, H, P, N), dtype=torch.float32, device=dev)
    st = _load().swimba_mixer_fwd_xe_selected(
        ctypes.byref(d), _ptr(x_sel, "x_sel", io, (B, L, K, H, P)), _ptr(dt, "dt", io, (B, L, H)),
        _ptr(A, "A", torch.float32, (H,)), _ptr(D, "D", torch.float32, (H,)),
        _ptr(B_sel, "B_sel", io, (B, L, K, G, N)), _ptr(C_sel, "C_sel", io, (B, L, K, G, N)),
        _ptr(topk_w, "topk_w", torch.float32, (B, L, K)), _ptr(h0, "h0", torch.float32, (B, H, P, N)),
        _ptr(y, "y", io, (B, L, H, P)), _ptr(h_final, "h_final", torch.float32, (B, H, P, N)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_mixer_fwd_xe_selected")
    return MixerOut(y, h_final, None, None)


def swimba_separated_workspace_bytes(dims: swimba_dims) -> int:
    return int(_load().swimba_separated_workspace_bytes(ctypes.byref(dims)))


def swimba_separated_fwd(x, dt, A, D, B_experts, C_experts, router_logits, top_k: int, chunk: int, *,
                         y=None, topk_idx=None, topk_w=None, workspace=None, want_topk: bool = False) -> MixerOut:
    """MoE of separated SSMs (contrast path); same tensors as swimba_mixer_fwd, zero initial states."""
    d = dims_of(x, B_experts, top_k, chunk)
    B, L, H, P, N, G, E = d.batch, d.seqlen, d.nheads, d.headdim, d.dstate, d.ngroups, d.nexperts
    io, dev = x.dtype, x.device
    if workspace is None:
        n = swimba_separated_workspace_bytes(d)
        if n == 0:
            alloc_workspace(d, dev)   # raises with the status of the dims
        workspace = torch.empty(n, dtype=torch.uint8, device=dev)
    if y is None:
        y = torch.empty_like(x)
    if want_topk and topk_idx is None:
        topk_idx = torch.empty((B, L, top_k), dtype=torch.int32, device=dev)
    if want_topk and topk_w is None:
        topk_w = torch.empty((B, L, top_k), dtype=torch.float32, device=dev)
    st = _load().swimba_separated_fwd(
        ctypes.byref(d), _ptr(x, "x", io, (B, L, H, P)), _ptr(dt, "dt", io, (B, L, H)),
        _ptr(A, "A", torch.float32, (H,)), _ptr(D, "D", torch.float32, (H,)),
        _ptr(B_experts, "B_experts", io, (B, L, E, G, N)), _ptr(C_experts, "C_experts", io, (B, L, E, G, N)),
        _ptr(router_logits, "router_logits", io, (B, L, E)), _ptr(y, "y", io, (B, L, H, P)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, L, top_k)),
        _ptr(topk_w, "topk_w", torch.float32, (B, L, top_k)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_separated_fwd")
    return MixerOut(y, None, topk_idx, topk_w)


def swimba_stage_router(dims, router_logits, workspace):
    _check(_load().swimba_stage_router(ctypes.byref(dims), _ptr(router_logits, "router_logits"),
                                       _ptr(workspace, "workspace", torch.uint8), workspace.numel(),
                                       _stream()), "swimba_stage_router")


def swimba_stage_cumsum(dims, dt, A, workspace):
    _check(_load().swimba_stage_cumsum(ctypes.byref(dims), _ptr(dt, "dt"), _ptr(A, "A", torch.float32),
                                       _ptr(workspace, "workspace", torch.uint8), workspace.numel(),
                                       _stream()), "swimba_stage_cumsum")


def swimba_stage_mix(dims, B_experts, C_experts, router_logits, workspace):
    _check(_load().swimba_stage_mix(ctypes.byref(dims), _ptr(B_experts, "B_experts"),
                                    _ptr(C_experts, "C_experts"), _ptr(router_logits, "router_logits"),
                                    _ptr(workspace, "workspace", torch.uint8), workspace.numel(),
                                    _stream()), "swimba_stage_mix")


def swimba_stage_chunk_state(dims, x, dt, A, B_experts, workspace):
    _check(_load().swimba_stage_chunk_state(ctypes.byref(dims), _ptr(x, "x"), _ptr(dt, "dt"),
                                            _ptr(A, "A", torch.float32), _ptr(B_experts, "B_experts"),
                                            _ptr(workspace, "workspace", torch.uint8),
                                            workspace.numel(), _stream()), "swimba_stage_chunk_state")


def swimba_stage_state_scan(dims, h0, h_final, workspace):
    _check(_load().swimba_stage_state_scan(ctypes.byref(dims), _ptr(h0, "h0", torch.float32),
                                           _ptr(h_final, "h_final", torch.float32),
                                           _ptr(workspace, "workspace", torch.uint8),
                                           workspace.numel(), _stream()), "swimba_stage_state_scan")


def swimba_stage_output(dims, x, dt, D, B_experts, C_experts, y, workspace):
    _check(_load().swimba_stage_output(ctypes.byref(dims), _ptr(x, "x"), _ptr(dt, "dt"),
                                       _ptr(D, "D", torch.float32), _ptr(B_experts, "B_experts"),
                                       _ptr(C_experts, "C_experts"), _ptr(y, "y"),
                                       _ptr(workspace, "workspace", torch.uint8), workspace.numel(),
                                       _stream()), "swimba_stage_output")


PATH_GENERIC, PATH_STAGED, PATH_SINGLE_PASS, PATH_SINGLE_PASS_CHUNK_MIX, PATH_SINGLE_PASS_HEAD = 0, 1, 2, 3, 4
PATH_SINGLE_PASS_HEAD_CHUNK_MIX, PATH_STAGED_SHORT = 5, 6
PATH_SINGLE_PASS_HEAD_SPLIT, PATH_SINGLE_PASS_HEAD_SPLIT_CHUNK_MIX = 7, 8


def swimba_prefill_path(dims) -> int:
    """Kernels the forward runs for these dims on the current device (PATH_* values)."""
    r = _load().swimba_prefill_path(ctypes.byref(dims))
    if r < 0:
        _check(-r, "swimba_prefill_path")
    return r


def swimba_stage_mix_chunk(dims, B_experts, C_experts, router_logits, workspace):
    _check(_load().swimba_stage_mix_chunk(ctypes.byref(dims), _ptr(B_experts, "B_experts"), _ptr(C_experts, "C_experts"),
                                          _ptr(router_logits, "router_logits"),
                                          _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream()),
           "swimba_stage_mix_chunk")


def swimba_stage_tables(dims, dt, A, workspace):
    _check(_load().swimba_stage_tables(ctypes.byref(dims), _ptr(dt, "dt"), _ptr(A, "A", torch.float32),
                                       _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream()),
           "swimba_stage_tables")


def swimba_stage_prep(dims, dt, A, workspace):
    _check(_load().swimba_stage_prep(ctypes.byref(dims), _ptr(dt, "dt"), _ptr(A, "A", torch.float32),
                                     _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream()),
           "swimba_stage_prep")


def swimba_stage_pass(dims, x, dt, D, h0, y, h_final, workspace):
    _check(_load().swimba_stage_pass(ctypes.byref(dims), _ptr(x, "x"), _ptr(dt, "dt"), _ptr(D, "D", torch.float32),
                                     _ptr(h0, "h0", torch.float32), _ptr(y, "y"),
                                     _ptr(h_final, "h_final", torch.float32),
                                     _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream()),
           "swimba_stage_pass")


def swimba_stage_chunk_state_tiles(dims, x, dt, A, workspace):
    _check(_load().swimba_stage_chunk_state_tiles(ctypes.byref(dims), _ptr(x, "x"), _ptr(dt, "dt"),
                                                  _ptr(A, "A", torch.float32),
                                                  _ptr(workspace, "workspace", torch.uint8), workspace.numel(),
                                                  _stream()), "swimba_stage_chunk_state_tiles")


def swimba_stage_output_carry(dims, x, dt, D, h0, y, h_final, workspace):
    _check(_load().swimba_stage_output_carry(ctypes.byref(dims), _ptr(x, "x"), _ptr(dt, "dt"),
                                             _ptr(D, "D", torch.float32), _ptr(h0, "h0", torch.float32), _ptr(y, "y"),
                                             _ptr(h_final, "h_final", torch.float32),
                                             _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream()),
           "swimba_stage_output_carry")


def swimba_stage_pass64(dims, x, dt, D, h0, y, h_final, workspace):
    _check(_load().swimba_stage_pass64(ctypes.byref(dims), _ptr(x, "x"), _ptr(dt, "dt"), _ptr(D, "D", torch.float32),
                                       _ptr(h0, "h0", torch.float32), _ptr(y, "y"),
                                       _ptr(h_final, "h_final", torch.float32),
                                       _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream()),
           "swimba_stage_pass64")


def swimba_pass_segments(dims) -> int:
    """Segments per sequence of the per-head single pass the forward takes for these dims (1: none)."""
    r = _load().swimba_pass_segments(ctypes.byref(dims))
    if r < 0:
        _check(-r, "swimba_pass_segments")
    return r


def swimba_stage_boundary_states(dims, x, dt, A, h0, nseg, workspace):
    _check(_load().swimba_stage_boundary_states(ctypes.byref(dims), _ptr(x, "x"), _ptr(dt, "dt"),
                                                _ptr(A, "A", torch.float32), _ptr(h0, "h0", torch.float32), int(nseg),
                                                _ptr(workspace, "workspace", torch.uint8), workspace.numel(),
                                                _stream()),
           "swimba_stage_boundary_states")


def swimba_stage_pass64_split(dims, x, dt, D, h0, y, h_final, nseg, workspace):
    _check(_load().swimba_stage_pass64_split(ctypes.byref(dims), _ptr(x, "x"), _ptr(dt, "dt"),
                                             _ptr(D, "D", torch.float32), _ptr(h0, "h0", torch.float32), _ptr(y, "y"),
                                             _ptr(h_final, "h_final", torch.float32), int(nseg),
                                             _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream()),
           "swimba_stage_pass64_split")


def workspace_views(dims: swimba_dims, workspace: torch.Tensor):
    """Typed views of the scratch arrays inside a workspace (for tests/profiling)."""
    lo = swimba_mixer_workspace_layout(dims)
    B, L, H, P, N, K, Q = (dims.batch, dims.seqlen, dims.nheads, dims.headdim, dims.dstate,
                           dims.top_k, dims.chunk)
    nc = (L + Q - 1) // Q

    def view(off, count, dtype, shape):
        nbytes = count * torch.empty((), dtype=dtype).element_size()
        return workspace[off:off + nbytes].view(dtype).view(shape)

    out = {
        "topk_idx": view(lo.topk_idx, B * L * K, torch.int32, (B, L, K)),
        "topk_w": view(lo.topk_w, B * L * K, torch.float32, (B, L, K)),
        "cs": view(lo.cs, B * nc * H * Q, torch.float32, (B, nc, H, Q)),
    }
    # chunk / carried states: fp32 on the fp32 path, bf16 on the bf16 MFMA path
    if lo.states_lp != lo.cmix:
        # stored as 64 x 128 tiles whatever P <= 64 and N <= 128 are; the view shows the caller's part
        out["states"] = view(lo.states_lp, B * nc * H * 64 * 128, torch.bfloat16, (B, nc, H, 64, 128))[..., :P, :N]
    else:
        out["states"] = view(lo.states, B * nc * H * P * N, torch.float32, (B, nc, H, P, N))
    return out


class StepOut(NamedTuple):
    y: torch.Tensor
    state: torch.Tensor
    topk_idx: Optional[torch.Tensor]


def swimba_step_workspace_bytes(dims: swimba_dims) -> int:
    return int(_load().swimba_step_workspace_bytes(ctypes.byref(dims)))


def swimba_step(state, x, dt, A, D, B_experts, C_experts, router_logits, top_k: int, *,
                state_out=None, y=None, topk_idx=None, workspace=None, want_topk: bool = False) -> StepOut:
    """state (B,H,P,N) fp32, x (B,H,P), dt (B,H), B/C_experts (B,E,G,N), router_logits (B,E).
    state_out defaults to `state` (in place)."""
    B, H, P = x.shape
    _, E, G, N = B_experts.shape
    io = x.dtype
    d = make_dims(B, 1, H, P, N, G, E, top_k, 0, _io_code(x))
    if state_out is None:
        state_out = state
    if y is None:
        y = torch.empty_like(x)
    if want_topk and topk_idx is None:
        topk_idx = torch.empty((B, top_k), dtype=torch.int32, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(swimba_step_workspace_bytes(d), 256), dtype=torch.uint8, device=x.device)
    st = _load().swimba_step(
        ctypes.byref(d), _ptr(state, "state", torch.float32, (B, H, P, N)),
        _ptr(state_out, "state_out", torch.float32, (B, H, P, N)), _ptr(x, "x", io, (B, H, P)),
        _ptr(dt, "dt", io, (B, H)), _ptr(A, "A", torch.float32, (H,)), _ptr(D, "D", torch.float32, (H,)),
        _ptr(B_experts, "B_experts", io, (B, E, G, N)), _ptr(C_experts, "C_experts", io, (B, E, G, N)),
        _ptr(router_logits, "router_logits", io, (B, E)), _ptr(y, "y", io, (B, H, P)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, top_k)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_step")
    return StepOut(y, state_out, topk_idx)


def swimba_step_static(state, x, dt, A, D, B_experts, C_experts, router_logits, top_k: int, y, *,
                       state_out=None, topk_idx=None) -> StepOut:
    """swimba_step on the library's own scratch array: no workspace, and nothing is allocated here
    either (y, and topk_idx / state_out when wanted, are the caller's tensors)."""
    B, H, P = x.shape
    _, E, G, N = B_experts.shape
    io = x.dtype
    d = make_dims(B, 1, H, P, N, G, E, top_k, 0, _io_code(x))
    if state_out is None:
        state_out = state
    st = _load().swimba_step_static(
        ctypes.byref(d), _ptr(state, "state", torch.float32, (B, H, P, N)),
        _ptr(state_out, "state_out", torch.float32, (B, H, P, N)), _ptr(x, "x", io, (B, H, P)),
        _ptr(dt, "dt", io, (B, H)), _ptr(A, "A", torch.float32, (H,)), _ptr(D, "D", torch.float32, (H,)),
        _ptr(B_experts, "B_experts", io, (B, E, G, N)), _ptr(C_experts, "C_experts", io, (B, E, G, N)),
        _ptr(router_logits, "router_logits", io, (B, E)), _ptr(y, "y", io, (B, H, P)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, top_k)), _stream())
    _check(st, "swimba_step_static")
    return StepOut(y, state_out, topk_idx)


def swimba_probe_copy(dst: torch.Tensor, src: torch.Tensor) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes
    _check(_load().swimba_probe_copy(_ptr(dst, "dst"), _ptr(src, "src"), nbytes, _stream()),
           "swimba_probe_copy")


def swimba_probe_mfma(sink: torch.Tensor, blocks: int, iters: int) -> None:
    assert sink.numel() >= blocks * 256
    _check(_load().swimba_probe_mfma(_ptr(sink, "sink", torch.float32), blocks, iters, _stream()),
           "swimba_probe_mfma")


def swimba_step_multi_workspace_bytes(dims: swimba_dims) -> int:
    return int(_load().swimba_step_multi_workspace_bytes(ctypes.byref(dims)))


def swimba_step_multi(state, x, dt, A, D, B_experts, C_experts, router_logits, top_k: int, *,
                      state_out=None, y=None, topk_idx=None, workspace=None, want_topk: bool = False) -> StepOut:
    """L decode tokens per sequence in one call: state (B,H,P,N) fp32, x (B,L,H,P), dt (B,L,H),
    B/C_experts (B,L,E,G,N), router_logits (B,L,E).  state_out defaults to `state` (in place)."""
    B, L, H, P = x.shape
    _, _, E, G, N = B_experts.shape
    io = x.dtype
    d = make_dims(B, L, H, P, N, G, E, top_k, 0, _io_code(x))
    if state_out is None:
        state_out = state
    if y is None:
        y = torch.empty_like(x)
    if want_topk and topk_idx is None:
        topk_idx = torch.empty((B, L, top_k), dtype=torch.int32, device=x.device)
    if workspace is None:
        n = swimba_step_multi_workspace_bytes(d)
        if n == 0:
            raise SwimbaError(4 if L > 0 else 2, "swimba_step_multi_workspace_bytes")
        workspace = torch.empty(n, dtype=torch.uint8, device=x.device)
    st = _load().swimba_step_multi(
        ctypes.byref(d), _ptr(state, "state", torch.float32, (B, H, P, N)),
        _ptr(state_out, "state_out", torch.float32, (B, H, P, N)), _ptr(x, "x", io, (B, L, H, P)),
        _ptr(dt, "dt", io, (B, L, H)), _ptr(A, "A", torch.float32, (H,)), _ptr(D, "D", torch.float32, (H,)),
        _ptr(B_experts, "B_experts", io, (B, L, E, G, N)), _ptr(C_experts, "C_experts", io, (B, L, E, G, N)),
        _ptr(router_logits, "router_logits", io, (B, L, E)), _ptr(y, "y", io, (B, L, H, P)),
        _ptr(topk_idx, "topk_idx", torch.int32, (B, L, top_k)),
        _ptr(workspace, "workspace", torch.uint8), workspace.numel(), _stream())
    _check(st, "swimba_step_multi")
    return StepOut(y, state_out, topk_idx)
