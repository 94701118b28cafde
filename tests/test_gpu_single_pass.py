"""The single-pass evaluation (mix, prep, pass through the C ABI) against the oracle on shapes the
forward's own heuristic would send to the staged kernels: every chunk size, ragged lengths, head
dimensions and state sizes below the kernels' 64 x 128, groups, initial state, with and without
the skip term; and against the staged evaluation of the same inputs."""
import numpy as np
import pytest
import torch

from oracle import swimba_oracle as orc
from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import TOL, abs_inputs, comp_tol, componentwise_excess, host, rel_errors, to_device

pytestmark = pytest.mark.gpu

CASES = [
    # B, L, H, P, N, G, E, k, Q, h0, D
    (2, 600, 4, 64, 128, 2, 8, 2, 256, True, True),
    (1, 1100, 6, 64, 128, 1, 8, 2, 256, False, False),     # several chunks, ragged tail
    (2, 300, 4, 64, 128, 2, 8, 2, 128, True, False),
    (2, 257, 2, 64, 128, 1, 8, 3, 64, False, True),
    (1, 31, 2, 64, 128, 1, 4, 2, 256, True, True),          # one short chunk
    (1, 1, 2, 64, 128, 1, 4, 1, 64, False, True),           # one token
    (2, 520, 3, 32, 64, 3, 4, 4, 256, True, True),          # one 32-channel slice, padded state
    (1, 400, 4, 40, 96, 2, 16, 1, 128, False, True),        # second slice partly past P
    (2, 700, 2, 8, 16, 1, 5, 5, 256, True, False),
    (1, 2100, 8, 64, 128, 8, 16, 2, 256, False, True),      # the long-sequence layer's grouping, 9 chunks
]


def single_pass(d, dims, D, h0, k, Q, whole_head=False):
    """mix, prep and the pass: a workgroup per (batch, head, 32 channels), or per (batch, head) with all
    channels of the head (whole_head)"""
    ws = sw.alloc_workspace(dims, "cuda:0")
    y = torch.full_like(d["x"], float("nan"))
    hf = torch.full((dims.batch, dims.nheads, dims.headdim, dims.dstate), float("nan"), device="cuda:0")
    sw.swimba_stage_mix(dims, d["B_experts"], d["C_experts"], d["router_logits"], ws)
    sw.swimba_stage_prep(dims, d["dt"], d["A"], ws)
    (sw.swimba_stage_pass64 if whole_head else sw.swimba_stage_pass)(dims, d["x"], d["dt"], D, h0, y, hf, ws)
    torch.cuda.synchronize()
    return y, hf, ws


@pytest.mark.parametrize("whole_head", [False, True], ids=["slices32", "head64"])
@pytest.mark.parametrize("case", CASES, ids=lambda c: "B%dL%dH%dP%dN%dG%dE%dk%dQ%d_h0%d_D%d" % c)
def test_single_pass_matches_oracle(case, whole_head):
    B, L, H, P, N, G, E, k, Q, with_h0, with_D = case
    w = synth.Workload("sp", B, L, H, P, N, G, E, k, Q, "bf16", 7)
    p = synth.make_inputs(w, seed=hash(case) % 100000)
    rng = np.random.default_rng(11)
    p["D"] = rng.standard_normal(H).astype(np.float32)
    h0 = (0.1 * rng.standard_normal((B, H, P, N))).astype(np.float32) if with_h0 else None
    D = p["D"] if with_D else None
    d = to_device(p, "bf16")
    dims = sw.dims_of(d["x"], d["B_experts"], k, Q)
    y, hf, ws = single_pass(d, dims, d["D"] if with_D else None,
                            None if h0 is None else torch.from_numpy(h0).to("cuda:0"), k, Q, whole_head)
    ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], D, p["B_experts"], p["C_experts"], p["router_logits"], k, h0=h0)
    idx = sw.workspace_views(dims, ws)["topk_idx"]
    np.testing.assert_array_equal(idx.cpu().numpy(), ref["topk_idx"])
    assert torch.isfinite(y).all() and torch.isfinite(hf).all()
    q = abs_inputs(p)
    aref = orc.mixer_fwd(q["x"], q["dt"], q["A"], None if D is None else np.abs(D), q["B_experts"], q["C_experts"],
                         q["router_logits"], k, h0=None if h0 is None else np.abs(h0))
    ey = componentwise_excess(host(y), ref["y"], aref["y"])
    eh = componentwise_excess(host(hf), ref["h_final"], aref["h_final"])
    l2, linf = rel_errors(host(y), ref["y"], (0, 2))
    hl2, hlinf = rel_errors(host(hf), ref["h_final"], (0, 1))
    print(case, "y l2 %.2e linf %.2e  h_final l2 %.2e  componentwise %.2e %.2e" % (l2, linf, hl2, ey, eh), flush=True)
    assert ey <= comp_tol("bf16") and eh <= comp_tol("bf16"), (ey, eh)
    if L >= 16:
        assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)
    assert hl2 <= TOL["bf16"] and hlinf <= TOL["bf16"], (hl2, hlinf)
    # the staged evaluation of the same inputs (the same operands and roundings, another order of
    # summation): far closer to each other than either is to the exact result
    out = torch.empty_like(d["x"])
    hf2 = torch.empty_like(hf)
    ws2 = sw.alloc_workspace(dims, "cuda:0")
    sw.swimba_stage_mix(dims, d["B_experts"], d["C_experts"], d["router_logits"], ws2)
    sw.swimba_stage_chunk_state(dims, d["x"], d["dt"], d["A"], d["B_experts"], ws2)
    sw.swimba_stage_state_scan(dims, None if h0 is None else torch.from_numpy(h0).to("cuda:0"), hf2, ws2)
    sw.swimba_stage_output(dims, d["x"], d["dt"], d["D"] if with_D else None, d["B_experts"], d["C_experts"], out, ws2)
    torch.cuda.synchronize()
    if L >= 16:
        l2, linf = rel_errors(host(y), host(out), (0, 2))
        assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], ("staged", l2, linf)
    l2, linf = rel_errors(host(hf), host(hf2), (0, 1))
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], ("staged h_final", l2, linf)


@pytest.mark.parametrize("whole_head", [False, True], ids=["slices32", "head64"])
def test_single_pass_is_deterministic_and_causal(whole_head):
    w = synth.Workload("sp", 2, 600, 4, 64, 128, 2, 8, 2, 256, "bf16", 7)
    p = synth.make_inputs(w, seed=5)
    q = synth.make_inputs(w, seed=6)
    d = to_device(p, "bf16")
    dims = sw.dims_of(d["x"], d["B_experts"], 2, 256)
    y1, h1, _ = single_pass(d, dims, d["D"], None, 2, 256, whole_head)
    y2, h2, _ = single_pass(d, dims, d["D"], None, 2, 256, whole_head)
    assert torch.equal(y1, y2) and torch.equal(h1, h2)
    for s in (37, 256, 300, 599):
        mod = {kk: (np.concatenate([v[:, :s], q[kk][:, s:]], axis=1) if kk in ("x", "dt", "B_experts", "C_experts",
                                                                                 "router_logits") else v)
               for kk, v in p.items()}
        dm = to_device(mod, "bf16")
        ym, _, _ = single_pass(dm, dims, dm["D"], None, 2, 256, whole_head)
        assert torch.equal(ym[:, :s], y1[:, :s]), s


def test_stage_calls_refuse_the_fp32_path():
    dev = "cuda:0"
    x = torch.zeros((1, 64, 2, 16), device=dev)
    Be = torch.zeros((1, 64, 3, 1, 16), device=dev)
    dims = sw.dims_of(x, Be, 2, 32)
    ws = sw.alloc_workspace(dims, dev)
    with pytest.raises(sw.SwimbaError) as e:
        sw.swimba_stage_prep(dims, torch.ones((1, 64, 2), device=dev), -torch.ones(2, device=dev), ws)
    assert e.value.status == 4


CHUNK_MIX_CASES = [
    # B, L, H, P, N, G, E, k, Q
    (2, 600, 4, 64, 128, 2, 8, 2, 256),
    (1, 1100, 6, 64, 128, 1, 16, 2, 256),      # 16 experts (two 16-byte loads of logits), ragged tail
    (2, 300, 4, 64, 128, 2, 5, 2, 128),        # odd expert count: element loads of the logits
    (2, 257, 2, 64, 128, 1, 8, 1, 64),         # top-1
    (1, 31, 2, 64, 128, 1, 4, 2, 256),         # one short chunk
    (1, 400, 4, 40, 96, 2, 16, 1, 128),        # padded state size
    (3, 2100, 8, 64, 128, 8, 16, 2, 256),      # 216 items: several per workgroup on a small grid, too
]


@pytest.mark.parametrize("case", CHUNK_MIX_CASES, ids=lambda c: "B%dL%dH%dP%dN%dG%dE%dk%dQ%d" % c)
def test_chunk_level_mix_writes_what_mix_and_prep_write(case):
    """Router + mixing + tiles per whole chunk in one persistent kernel, and the tables alone, against
    the per-tile mix and the prep kernel: every byte of the workspace except the operand image of
    the mixed B rows, which the chunk-level kernel does not need; then the pass on both."""
    B, L, H, P, N, G, E, k, Q = case
    w = synth.Workload("cm", B, L, H, P, N, G, E, k, Q, "bf16", 9)
    p = synth.make_inputs(w, seed=hash(case) % 100000)
    d = to_device(p, "bf16")
    dims = sw.dims_of(d["x"], d["B_experts"], k, Q)
    lo = sw.swimba_mixer_workspace_layout(dims)
    offs = sorted(getattr(lo, f[0]) for f in lo._fields_)
    frag_end = min(o for o in offs if o > lo.bmix_frag)
    out = []
    for chunked in (False, True):
        ws = sw.alloc_workspace(dims, "cuda:0")
        ws.zero_()
        if chunked:
            sw.swimba_stage_mix_chunk(dims, d["B_experts"], d["C_experts"], d["router_logits"], ws)
            sw.swimba_stage_tables(dims, d["dt"], d["A"], ws)
        else:
            sw.swimba_stage_mix(dims, d["B_experts"], d["C_experts"], d["router_logits"], ws)
            sw.swimba_stage_prep(dims, d["dt"], d["A"], ws)
        y = torch.empty_like(d["x"])
        hf = torch.empty((B, H, P, N), device="cuda:0")
        sw.swimba_stage_pass(dims, d["x"], d["dt"], d["D"], None, y, hf, ws)
        torch.cuda.synchronize()
        out.append((ws, y, hf))
    (wa, ya, ha), (wb, yb, hb) = out
    assert torch.equal(wa[:lo.bmix_frag], wb[:lo.bmix_frag])
    assert torch.equal(wa[frag_end:], wb[frag_end:])
    assert (wb[lo.bmix_frag:frag_end] == 0).all()
    assert torch.equal(ya, yb) and torch.equal(ha, hb)


def test_chunk_level_mix_refuses_what_it_does_not_take():
    dev = "cuda:0"
    for E, k in ((17, 2), (8, 3)):
        x = torch.zeros((1, 64, 2, 64), dtype=torch.bfloat16, device=dev)
        Be = torch.zeros((1, 64, E, 1, 128), dtype=torch.bfloat16, device=dev)
        dims = sw.dims_of(x, Be, k, 64)
        ws = sw.alloc_workspace(dims, dev)
        with pytest.raises(RuntimeError):
            sw.swimba_stage_mix_chunk(dims, Be, Be, torch.zeros((1, 64, E), dtype=torch.bfloat16, device=dev), ws)


@pytest.mark.parametrize("case", [(2, 2048, 4, 64, 128, 2, 8, 2, 256, True), (1, 500, 3, 64, 128, 1, 4, 2, 64, True),
                                  (2, 300, 4, 40, 96, 2, 8, 3, 128, False), (1, 31, 2, 64, 128, 1, 4, 1, 256, True)],
                         ids=lambda c: "B%dL%dH%dP%dN%dG%dE%dk%dQ%d_h0%d" % c)
def test_short_sequence_kernels_equal_the_scan_path(case):
    """At most 8 chunks: the tiles ride in the chunk-state launch and the output kernel carries the state
    forward itself (h0, S_0 .. S_{c-1} in fp32, the scan's order of operations), against chunk state,
    scan and output on the same inputs: the same bits."""
    B, L, H, P, N, G, E, k, Q, with_h0 = case
    w = synth.Workload("lb", B, L, H, P, N, G, E, k, Q, "bf16", 5)
    p = synth.make_inputs(w, seed=hash(case) % 100000)
    d = to_device(p, "bf16")
    dims = sw.dims_of(d["x"], d["B_experts"], k, Q)
    h0 = (0.1 * torch.randn((B, H, P, N), device="cuda:0")) if with_h0 else None
    res = []
    for short in (False, True):
        ws = sw.alloc_workspace(dims, "cuda:0")
        ws.zero_()
        y = torch.empty_like(d["x"])
        hf = torch.empty((B, H, P, N), device="cuda:0")
        sw.swimba_stage_mix(dims, d["B_experts"], d["C_experts"], d["router_logits"], ws)
        if short:
            sw.swimba_stage_chunk_state_tiles(dims, d["x"], d["dt"], d["A"], ws)
            sw.swimba_stage_output_carry(dims, d["x"], d["dt"], d["D"], h0, y, hf, ws)
        else:
            sw.swimba_stage_chunk_state(dims, d["x"], d["dt"], d["A"], d["B_experts"], ws)
            sw.swimba_stage_state_scan(dims, h0, hf, ws)
            sw.swimba_stage_output(dims, d["x"], d["dt"], d["D"], d["B_experts"], d["C_experts"], y, ws)
        torch.cuda.synchronize()
        res.append((y, hf))
    assert torch.equal(res[0][0], res[1][0])
    assert torch.equal(res[0][1], res[1][1])
    assert sw.swimba_prefill_path(dims) in (sw.PATH_STAGED_SHORT, sw.PATH_SINGLE_PASS_HEAD, sw.PATH_SINGLE_PASS)


def test_long_sequence_on_the_scan_path_matches_oracle():
    """More than 8 chunks and too few chains for a single pass: mix, chunk state, scan, output from the forward."""
    w = synth.Workload("sc", 2, 700, 4, 64, 128, 2, 8, 2, 64, "bf16", 6)
    p = synth.make_inputs(w, seed=77)
    d = to_device(p, "bf16")
    dims = sw.dims_of(d["x"], d["B_experts"], 2, 64)
    assert sw.swimba_prefill_path(dims) == sw.PATH_STAGED
    h0 = (0.1 * np.random.default_rng(3).standard_normal((2, 4, 64, 128))).astype(np.float32)
    out = sw.swimba_mixer_fwd(d["x"], d["dt"], d["A"], d["D"], d["B_experts"], d["C_experts"], d["router_logits"], 2, 64,
                              torch.from_numpy(h0).to("cuda:0"))
    torch.cuda.synchronize()
    ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], p["D"], p["B_experts"], p["C_experts"], p["router_logits"], 2, h0=h0)
    l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)
    l2, linf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)


SPLIT_CASES = [
    # B, L, H, P, N, G, E, k, Q, h0, D, segments, factor on dt
    (2, 1024, 4, 64, 128, 2, 8, 2, 256, True, True, 2, 1.0),
    (1, 1536, 3, 64, 128, 1, 8, 2, 128, False, True, 3, 1.0),
    (1, 1024, 2, 48, 96, 1, 4, 1, 64, True, False, 4, 1.0),
    (2, 2048, 4, 64, 128, 4, 8, 2, 256, True, True, 2, 0.05),   # hardly any decay: every chunk state counts
    (1, 3072, 4, 64, 128, 1, 8, 2, 256, True, True, 2, 12.0),   # strong decay: most chunk states are left out
    (1, 2048, 2, 64, 128, 1, 4, 2, 128, True, True, 4, 12.0),
    (1, 10240, 2, 64, 128, 1, 4, 2, 64, True, True, 2, 0.02),   # 80 chunks per segment, nearly all of them count
    (2, 4096, 8, 64, 128, 8, 4, 2, 128, False, True, 2, 1.0),   # a group per head
]


@pytest.mark.parametrize("case", SPLIT_CASES, ids=lambda c: "B%dL%dH%dP%dN%dG%dE%dk%dQ%d_h0%d_D%d_seg%d_dt%g" % c)
def test_split_pass_matches_oracle_and_the_whole_pass(case):
    """Every sequence as 2..4 segments, each walked by a workgroup of its own from the state at its boundary
    (chunk states in front of the boundary, those with a factor of exactly zero left out): against the
    oracle, and against the same kernel walking whole sequences."""
    B, L, H, P, N, G, E, k, Q, with_h0, with_D, nseg, dt_scale = case
    w = synth.Workload("split", B, L, H, P, N, G, E, k, Q, "bf16", 9)
    p = synth.make_inputs(w, seed=hash(case[:12]) % 100000)
    # scaled step sizes, rounded to bf16 here so that both sides see the same values
    p["dt"] = torch.from_numpy(p["dt"] * np.float32(dt_scale)).to(torch.bfloat16).to(torch.float32).numpy()
    rng = np.random.default_rng(13)
    p["D"] = rng.standard_normal(H).astype(np.float32)
    h0 = (0.1 * rng.standard_normal((B, H, P, N))).astype(np.float32) if with_h0 else None
    D = p["D"] if with_D else None
    d = to_device(p, "bf16")
    dims = sw.dims_of(d["x"], d["B_experts"], k, Q)
    h0d = None if h0 is None else torch.from_numpy(h0).to("cuda:0")
    Dd = d["D"] if with_D else None
    ws = sw.alloc_workspace(dims, "cuda:0")
    ws.fill_(0xff)                              # chunk states that are left out must not be read either
    y = torch.full_like(d["x"], float("nan"))
    hf = torch.full((B, H, P, N), float("nan"), device="cuda:0")
    sw.swimba_stage_mix(dims, d["B_experts"], d["C_experts"], d["router_logits"], ws)
    sw.swimba_stage_prep(dims, d["dt"], d["A"], ws)
    sw.swimba_stage_boundary_states(dims, d["x"], d["dt"], d["A"], h0d, nseg, ws)
    sw.swimba_stage_pass64_split(dims, d["x"], d["dt"], Dd, h0d, y, hf, nseg, ws)
    torch.cuda.synchronize()
    assert torch.isfinite(y).all() and torch.isfinite(hf).all()
    ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], D, p["B_experts"], p["C_experts"], p["router_logits"], k, h0=h0)
    q = abs_inputs(p)
    aref = orc.mixer_fwd(q["x"], q["dt"], q["A"], None if D is None else np.abs(D), q["B_experts"], q["C_experts"],
                         q["router_logits"], k, h0=None if h0 is None else np.abs(h0))
    ey = componentwise_excess(host(y), ref["y"], aref["y"])
    eh = componentwise_excess(host(hf), ref["h_final"], aref["h_final"])
    l2, linf = rel_errors(host(y), ref["y"], (0, 2))
    hl2, hlinf = rel_errors(host(hf), ref["h_final"], (0, 1))
    print(case, "y l2 %.2e linf %.2e  h_final l2 %.2e  componentwise %.2e %.2e" % (l2, linf, hl2, ey, eh), flush=True)
    assert ey <= comp_tol("bf16") and eh <= comp_tol("bf16"), (ey, eh)
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)
    assert hl2 <= TOL["bf16"] and hlinf <= TOL["bf16"], (hl2, hlinf)
    # whole sequences: identical in the first segment, within the operands' rounding behind it
    y1 = torch.empty_like(y)
    hf1 = torch.empty_like(hf)
    sw.swimba_stage_pass64(dims, d["x"], d["dt"], Dd, h0d, y1, hf1, ws)
    torch.cuda.synchronize()
    assert torch.equal(y[:, :L // nseg], y1[:, :L // nseg])
    l2, linf = rel_errors(host(y), host(y1), (0, 2))
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], ("whole", l2, linf)
    l2, linf = rel_errors(host(hf), host(hf1), (0, 1))
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], ("whole h_final", l2, linf)


def test_split_pass_refuses_what_it_does_not_take():
    dev = "cuda:0"
    for L, Q, nseg in ((1000, 256, 2), (1536, 256, 4), (1024, 256, 5), (1024, 256, 0)):
        x = torch.zeros((1, L, 2, 64), dtype=torch.bfloat16, device=dev)
        Be = torch.zeros((1, L, 4, 1, 128), dtype=torch.bfloat16, device=dev)
        dt = torch.zeros((1, L, 2), dtype=torch.bfloat16, device=dev)
        A = -torch.ones(2, device=dev)
        dims = sw.dims_of(x, Be, 2, Q)
        ws = sw.alloc_workspace(dims, dev)
        hf = torch.zeros((1, 2, 64, 128), device=dev)
        with pytest.raises(RuntimeError):
            sw.swimba_stage_boundary_states(dims, x, dt, A, None, nseg, ws)
        with pytest.raises(RuntimeError):
            sw.swimba_stage_pass64_split(dims, x, dt, None, None, torch.empty_like(x), hf, nseg, ws)


def test_forward_paths_of_the_workloads():
    """Which evaluation the forward picks for the benchmark shapes (a choice made from the shape and the number
    of compute units; the figures hold for the 256 units of an MI355X)."""
    if torch.cuda.get_device_properties(0).multi_processor_count != 256:
        pytest.skip("the expected choices are those of a device with 256 compute units")
    want = {1: (sw.PATH_STAGED_SHORT, 1), 2: (sw.PATH_SINGLE_PASS_HEAD, 1), 3: (sw.PATH_SINGLE_PASS_HEAD_SPLIT_CHUNK_MIX, 2)}
    for idx, (path, nseg) in want.items():
        w = synth.workload(idx)
        dims = sw.make_dims(w.batch, w.seqlen, w.nheads, w.headdim, w.dstate, w.ngroups, w.nexperts, w.top_k, w.chunk,
                            torch.bfloat16)
        assert sw.swimba_prefill_path(dims) == path, idx
        assert sw.swimba_pass_segments(dims) == nseg, idx
    # a ragged sequence is not split, 96 chains do not fill two segments' worth of compute units
    for shape in ((2, 16384 - 100, 64, 64, 128, 8, 16, 2, 256), (4, 8192, 24, 64, 128, 1, 8, 2, 256)):
        assert sw.swimba_pass_segments(sw.make_dims(*shape, torch.bfloat16)) == 1, shape
