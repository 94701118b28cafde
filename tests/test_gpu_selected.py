"""GPU parity of the paths that never hold a tensor with an expert axis: the projection written
per selected slot, the mixer forward on such streams, and both in one call.  The oracle has no
function of its own for them: they are its dense projection and its mixer forward, composed
here (selected rows gathered / scattered with the oracle's own selection)."""
import numpy as np
import pytest
import torch

from oracle import swimba_oracle as orc
from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import IO, TOL, host, rel_errors, to_device
from test_gpu_proj import dev, make_problem

pytestmark = pytest.mark.gpu


def gather_selected(dense, idx):
    """dense (B,L,E,G,N), idx (B,L,k) -> (B,L,k,G,N)"""
    return np.take_along_axis(dense, idx.astype(np.int64)[..., None, None], axis=2)


PROJ_SHAPES = [
    # B, L, Dm, E, G, N, k, io
    (2, 37, 24, 4, 2, 8, 2, "f32"),
    (1, 50, 33, 5, 1, 20, 5, "f32"),
    (2, 40, 48, 4, 1, 24, 2, "bf16"),
    (2, 300, 256, 8, 1, 128, 2, "bf16"),
    (1, 130, 80, 8, 2, 64, 1, "bf16"),
    (1, 70, 64, 16, 8, 128, 3, "bf16"),
    (1, 5, 32, 16, 1, 64, 2, "bf16"),
]


@pytest.mark.parametrize("cfg", PROJ_SHAPES, ids=lambda c: "B%dL%dD%dE%dG%dN%dk%d%s" % c)
def test_expert_proj_selected_matches_oracle(cfg):
    B, L, Dm, E, G, N, k, io = cfg
    u, WB, WC, g = make_problem(B, L, Dm, E, G, N, io, seed=hash(cfg[:7]) % 100000 + 3)
    ref = orc.expert_proj(u, WB, WC, g, k, fill=0.0)
    out = sw.swimba_expert_proj_selected(dev(u, io), dev(WB, io), dev(WC, io), dev(g, io), k)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
    np.testing.assert_allclose(host(out.topk_w), ref["topk_w"], rtol=1e-5, atol=1e-30)
    for name, got, dense in (("B", host(out.B_experts), ref["B_experts"]), ("C", host(out.C_experts), ref["C_experts"])):
        want = gather_selected(dense, ref["topk_idx"])
        assert got.shape == want.shape == (B, L, k, G, N)
        l2 = np.linalg.norm(got - want) / np.linalg.norm(want)
        linf = np.abs(got - want).max() / np.abs(want).max()
        print(cfg, name, "rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
        assert l2 <= TOL[io] and linf <= TOL[io], (name, l2, linf)


@pytest.mark.parametrize("case", ["many_passes_8_column_blocks", "one_hot_expert", "long_lists"])
def test_expert_proj_selected_list_shapes(case):
    """The GEMM shares one round of workgroups out among the experts by list length and walks a
    share in passes of up to 192 entries: cases with several passes per workgroup, with one expert
    holding every token, and with lists far longer than a pass."""
    if case == "many_passes_8_column_blocks":
        B, L, Dm, E, G, N, k = 1, 4100, 64, 4, 8, 128, 2        # 2048 columns: few workgroups per column block
    elif case == "one_hot_expert":
        B, L, Dm, E, G, N, k = 2, 3000, 48, 8, 1, 128, 2
    else:
        B, L, Dm, E, G, N, k = 4, 8192, 32, 4, 1, 64, 2         # 65536 entries for 256 workgroups
    u, WB, WC, g = make_problem(B, L, Dm, E, G, N, "bf16", seed=len(case))
    if case == "one_hot_expert":
        g[..., 3] = 8.0                                         # expert 3 is in every active set
    ref = orc.expert_proj(u, WB, WC, g, k, fill=0.0)
    out = sw.swimba_expert_proj_selected(dev(u, "bf16"), dev(WB, "bf16"), dev(WC, "bf16"), dev(g, "bf16"), k)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
    for name, got, dense in (("B", host(out.B_experts), ref["B_experts"]), ("C", host(out.C_experts), ref["C_experts"])):
        want = gather_selected(dense, ref["topk_idx"])
        l2 = np.linalg.norm(got - want) / np.linalg.norm(want)
        linf = np.abs(got - want).max() / np.abs(want).max()
        print(case, name, "rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
        assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (name, l2, linf)


MIX_SHAPES = [
    # B, L, H, P, N, G, E, k, Q, io
    (2, 96, 4, 16, 16, 2, 4, 2, 32, "f32"),
    (1, 77, 6, 8, 24, 3, 5, 5, 16, "f32"),        # ragged, dense routing
    (2, 130, 2, 32, 64, 1, 6, 1, 64, "f32"),      # top-1
    (2, 96, 4, 16, 16, 2, 4, 2, 32, "bf16"),      # bf16 io on the fp32 kernels
    (2, 300, 4, 64, 128, 2, 8, 2, 128, "bf16"),   # MFMA kernels, ragged tail, groups
    (1, 257, 2, 64, 128, 1, 4, 3, 64, "bf16"),
    (1, 520, 4, 64, 128, 2, 16, 1, 256, "bf16"),
    (1, 300, 2, 64, 128, 1, 32, 16, 256, "bf16"), # the largest active set
]


@pytest.mark.parametrize("cfg", MIX_SHAPES, ids=lambda c: "B%dL%dH%dP%dN%dG%dE%dk%dQ%d%s" % c)
def test_mixer_fwd_selected_matches_oracle(cfg):
    """Streams of the selected experts + their weights in, against the oracle's forward on the
    dense streams and the logits; an initial state and D != 1 are part of the case."""
    B, L, H, P, N, G, E, k, Q, io = cfg
    w = synth.Workload("sel", B, L, H, P, N, G, E, k, Q, io, 7)
    p = synth.make_inputs(w, seed=hash(cfg[:9]) % 100000 + 11)
    rng = np.random.default_rng(3)
    p["D"] = rng.standard_normal(H).astype(np.float32)
    h0 = (0.1 * rng.standard_normal((B, H, P, N))).astype(np.float32)
    ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], p["D"], p["B_experts"], p["C_experts"], p["router_logits"], k, h0=h0)
    idx = ref["topk_idx"]
    d = to_device(p, io)
    Bs = dev(gather_selected(p["B_experts"], idx), io)
    Cs = dev(gather_selected(p["C_experts"], idx), io)
    wsel = torch.from_numpy(ref["topk_w"].astype(np.float32)).to("cuda:0")
    out = sw.swimba_mixer_fwd_selected(d["x"], d["dt"], d["A"], d["D"], Bs, Cs, wsel, Q,
                                       torch.from_numpy(h0).to("cuda:0"))
    torch.cuda.synchronize()
    l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
    hl2, hlinf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
    print(cfg, "y rel l2 %.3e linf %.3e  h_final l2 %.3e" % (l2, linf, hl2), flush=True)
    assert l2 <= TOL[io] and linf <= TOL[io], (l2, linf)
    assert hl2 <= TOL[io] and hlinf <= TOL[io], (hl2, hlinf)


@pytest.mark.parametrize("shape", [(2, 600, 4, 64, 128, 2, 8, 2, 256), (2, 1536, 64, 64, 128, 8, 4, 2, 64),
                                   (4, 1024, 64, 64, 128, 8, 4, 2, 64)],
                         ids=["staged", "split_pass", "pass_per_head"])
def test_mixer_fwd_selected_equals_mixer_fwd_bitwise(shape):
    """Same kernels behind both entry points: gathering the selected rows on the host and
    passing the weights the router kernel produced gives the same bits as the dense call, on the
    staged kernels, on the per-head single pass behind the chunk-level mix kernel and on the split pass
    behind the per-tile one (the paths these shapes take on a device with 256 compute units)."""
    w = synth.Workload("selbit", *shape, "bf16", 5)
    p = synth.make_inputs(w, seed=41)
    d = to_device(p, "bf16")
    dims = sw.dims_of(d["x"], d["B_experts"], w.top_k, w.chunk)
    if torch.cuda.get_device_properties(0).multi_processor_count == 256:
        want = {256: (sw.PATH_STAGED_SHORT,), 64: (sw.PATH_SINGLE_PASS_HEAD_SPLIT, sw.PATH_SINGLE_PASS_HEAD_CHUNK_MIX)}[w.chunk]
        assert sw.swimba_prefill_path(dims) in want
        assert sw.swimba_pass_segments(dims) == (2 if shape[1] == 1536 else 1)
    dense = sw.swimba_mixer_fwd(d["x"], d["dt"], d["A"], d["D"], d["B_experts"], d["C_experts"],
                                d["router_logits"], w.top_k, w.chunk, want_topk=True)
    idx = dense.topk_idx.to(torch.int64)[..., None, None].expand(-1, -1, -1, w.ngroups, w.dstate)
    Bs = torch.gather(d["B_experts"], 2, idx).contiguous()
    Cs = torch.gather(d["C_experts"], 2, idx).contiguous()
    sel = sw.swimba_mixer_fwd_selected(d["x"], d["dt"], d["A"], d["D"], Bs, Cs, dense.topk_w, w.chunk)
    torch.cuda.synchronize()
    assert torch.equal(sel.y, dense.y)
    assert torch.equal(sel.h_final, dense.h_final)
    if w.chunk == 64:
        # the forward on these paths against the oracle as well (the staged case is covered above)
        ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], p["D"], p["B_experts"], p["C_experts"], p["router_logits"], w.top_k)
        l2, linf = rel_errors(host(dense.y), ref["y"], (0, 2))
        hl2, hlinf = rel_errors(host(dense.h_final), ref["h_final"], (0, 1))
        print(shape, "y rel l2 %.3e linf %.3e  h_final l2 %.3e" % (l2, linf, hl2), flush=True)
        assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)
        assert hl2 <= TOL["bf16"] and hlinf <= TOL["bf16"], (hl2, hlinf)


FUSED_SHAPES = [
    # B, L, Dm, H, P, N, G, E, k, Q, io
    (2, 90, 24, 4, 16, 16, 2, 4, 2, 32, "f32"),
    (1, 77, 40, 6, 8, 24, 3, 5, 5, 16, "f32"),
    (2, 64, 48, 2, 16, 24, 1, 4, 2, 32, "bf16"),       # bf16 on the fp32 kernels
    (2, 300, 128, 4, 64, 128, 1, 8, 2, 128, "bf16"),   # MFMA GEMM + MFMA chunk kernels
    (1, 520, 80, 4, 64, 128, 2, 16, 3, 256, "bf16"),
    (1, 300, 64, 2, 64, 128, 1, 8, 1, 64, "bf16"),     # top-1
]


@pytest.mark.parametrize("cfg", FUSED_SHAPES, ids=lambda c: "B%dL%dD%dH%dP%dN%dG%dE%dk%dQ%d%s" % c)
def test_mixer_fwd_proj_matches_oracle_chain(cfg):
    """Token features in, y out.  The oracle chain hands the projected streams on in fp32; the
    GPU rounds them to the io dtype between projection and mix (as a caller holding B/C tensors
    would), which stays far inside the bars."""
    B, L, Dm, H, P, N, G, E, k, Q, io = cfg
    u, WB, WC, g = make_problem(B, L, Dm, E, G, N, io, seed=hash(cfg[:10]) % 100000 + 5)
    w = synth.Workload("fused", B, L, H, P, N, G, E, k, Q, io, 7)
    p = synth.make_inputs(w, seed=hash(cfg[:10]) % 100000 + 6)
    rng = np.random.default_rng(8)
    D = rng.standard_normal(H).astype(np.float32)
    h0 = (0.1 * rng.standard_normal((B, H, P, N))).astype(np.float32)
    rp = orc.expert_proj(u, WB, WC, g, k, fill=0.0)
    ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], D, rp["B_experts"].astype(np.float32),
                        rp["C_experts"].astype(np.float32), g, k, h0=h0)
    out = sw.swimba_mixer_fwd_proj(dev(u, io), dev(WB, io), dev(WC, io), dev(p["x"], io), dev(p["dt"], io),
                                   torch.from_numpy(p["A"]).to("cuda:0"), torch.from_numpy(D).to("cuda:0"),
                                   dev(g, io), k, Q, torch.from_numpy(h0).to("cuda:0"), want_topk=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
    np.testing.assert_allclose(host(out.topk_w), ref["topk_w"], rtol=1e-5, atol=1e-30)
    l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
    hl2, hlinf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
    print(cfg, "y rel l2 %.3e linf %.3e  h_final l2 %.3e" % (l2, linf, hl2), flush=True)
    assert l2 <= TOL[io] and linf <= TOL[io], (l2, linf)
    assert hl2 <= TOL[io] and hlinf <= TOL[io], (hl2, hlinf)


def test_selected_paths_empty_and_workspace_errors():
    d = "cuda:0"
    x = torch.zeros((2, 0, 2, 8), device=d)
    out = sw.swimba_mixer_fwd_selected(x, torch.zeros((2, 0, 2), device=d), -torch.ones(2, device=d), None,
                                       torch.zeros((2, 0, 2, 1, 4), device=d), torch.zeros((2, 0, 2, 1, 4), device=d),
                                       torch.zeros((2, 0, 2), device=d), 16)
    torch.cuda.synchronize()
    assert out.y.shape == (2, 0, 2, 8) and float(out.h_final.abs().max()) == 0.0
    out = sw.swimba_mixer_fwd_proj(torch.zeros((2, 0, 16), device=d), torch.zeros((3, 1, 4, 16), device=d),
                                   torch.zeros((3, 1, 4, 16), device=d), x, torch.zeros((2, 0, 2), device=d),
                                   -torch.ones(2, device=d), None, torch.zeros((2, 0, 3), device=d), 2, 16)
    torch.cuda.synchronize()
    assert out.y.shape == (2, 0, 2, 8)
    x = torch.zeros((1, 8, 2, 8), device=d)
    with pytest.raises(RuntimeError):
        sw.swimba_mixer_fwd_proj(torch.zeros((1, 8, 16), device=d), torch.zeros((3, 1, 4, 16), device=d),
                                 torch.zeros((3, 1, 4, 16), device=d), x, torch.zeros((1, 8, 2), device=d),
                                 -torch.ones(2, device=d), None, torch.zeros((1, 8, 3), device=d), 2, 16,
                                 workspace=torch.empty(256, dtype=torch.uint8, device=d))
