"""GPU parity of the mixed forward with one input stream per expert (the rank-k form of
the mixed state update) against the oracle's sequential evaluation."""
import numpy as np
import pytest
import torch

from oracle import swimba_oracle as orc
from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import (IO, TOL, abs_inputs, comp_tol, componentwise_excess, host, rel_errors, run_mixer,
                      to_device)

pytestmark = pytest.mark.gpu


def make_problem(cfg, seed):
    B, L, H, P, N, G, E, k, Q, io = cfg
    w = synth.Workload("xe", B, L, H, P, N, G, E, k, Q, io, 7)
    p = synth.make_inputs(w, seed=seed)
    rng = np.random.default_rng(seed + 17)
    xe = rng.standard_normal((B, L, E, H, P)).astype(np.float32)
    p["x_experts"] = synth.round_to_bf16(xe) if io == "bf16" else xe
    p["D"] = rng.standard_normal(H).astype(np.float32)
    return w, p


def run_xe(p, top_k, chunk, io, h0=None, d_none=False):
    d = to_device(p, io)
    xe = torch.from_numpy(p["x_experts"]).to(IO[io]).to("cuda:0")
    h0d = None if h0 is None else torch.from_numpy(np.asarray(h0, dtype=np.float32)).to("cuda:0")
    out = sw.swimba_mixer_fwd_xe(xe, d["dt"], d["A"], None if d_none else d["D"], d["B_experts"], d["C_experts"],
                                 d["router_logits"], top_k, chunk, h0d, want_topk=True)
    torch.cuda.synchronize()
    return out


SHAPES = [
    # B, L, H, P, N, G, E, k, Q, io
    (2, 96, 4, 16, 16, 2, 4, 2, 32, "f32"),
    (1, 77, 6, 8, 24, 3, 5, 5, 16, "f32"),       # ragged, dense routing
    (2, 130, 2, 32, 64, 1, 3, 1, 64, "f32"),     # top-1
    (1, 40, 3, 5, 7, 1, 4, 3, 8, "f32"),         # H*P not a multiple of 8: scalar gather
    (2, 96, 4, 16, 16, 2, 4, 2, 32, "bf16"),     # bf16 io on the fp32 kernels
    (2, 300, 4, 64, 128, 2, 8, 2, 128, "bf16"),  # MFMA kernels, ragged tail, groups
    (1, 257, 2, 64, 128, 1, 4, 3, 64, "bf16"),
    (1, 520, 4, 64, 128, 2, 16, 1, 256, "bf16"),
    (2, 700, 8, 64, 128, 2, 8, 2, 256, "bf16"),  # several full chunks of 256 and a tail, two slots
    (1, 333, 4, 24, 120, 2, 6, 4, 128, "bf16"),  # padded P and N, the most slots the slot kernels take
    (1, 200, 2, 64, 128, 1, 6, 5, 64, "bf16"),   # more slots than that: one MFMA pass per slot
]


def selected_rows(p, topk_idx, topk_w):
    """rows of the k selected experts per token, as a projection restricted to the active set leaves them"""
    idx = np.asarray(topk_idx).astype(np.int64)
    take = lambda a: np.take_along_axis(a, idx.reshape(idx.shape + (1,) * (a.ndim - 3)), axis=2)
    return take(p["x_experts"]), take(p["B_experts"]), take(p["C_experts"]), np.asarray(topk_w, dtype=np.float32)


def run_xe_selected(p, topk_idx, topk_w, chunk, io, h0=None, d_none=False):
    xs, bs, cs, w = selected_rows(p, topk_idx, topk_w)
    dev = "cuda:0"
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(IO[io]).to(dev)
    d = to_device(p, io)
    h0d = None if h0 is None else torch.from_numpy(np.asarray(h0, dtype=np.float32)).to(dev)
    out = sw.swimba_mixer_fwd_xe_selected(t(xs), d["dt"], d["A"], None if d_none else d["D"], t(bs), t(cs),
                                          torch.from_numpy(w).to(dev), chunk, h0d)
    torch.cuda.synchronize()
    return out


@pytest.mark.parametrize("cfg", SHAPES, ids=lambda c: "B%dL%dH%dP%dN%dG%dE%dk%dQ%d%s" % c)
def test_xe_matches_oracle(cfg):
    B, L, H, P, N, G, E, k, Q, io = cfg
    w, p = make_problem(cfg, seed=hash(cfg[:9]) % 100000 + 3)
    h0 = np.random.default_rng(9).standard_normal((B, H, P, N)).astype(np.float32) * 0.1
    for d_none, h0v in ((True, None), (False, h0)):
        ref = orc.mixer_fwd_xe(p["x_experts"], p["dt"], p["A"], None if d_none else p["D"], p["B_experts"],
                               p["C_experts"], p["router_logits"], k, h0=h0v)
        out = run_xe(p, k, Q, io, h0=h0v, d_none=d_none)
        np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
        np.testing.assert_allclose(host(out.topk_w), ref["topk_w"], rtol=1e-5, atol=1e-30)
        l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
        print(cfg, "D=0" if d_none else "D,h0", "y rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
        assert l2 <= TOL[io] and linf <= TOL[io], ("y", d_none, l2, linf)
        l2, linf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
        assert l2 <= TOL[io] and linf <= TOL[io], ("h_final", d_none, l2, linf)
        # every element within the forward-error bound of its own sum of term magnitudes
        q = abs_inputs(p)
        aref = orc.mixer_fwd_xe(q["x_experts"], p["dt"], p["A"], None if d_none else q["D"], q["B_experts"],
                                q["C_experts"], p["router_logits"], k, h0=None if h0v is None else np.abs(h0v))
        ex_y = componentwise_excess(host(out.y), ref["y"], aref["y"])
        ex_h = componentwise_excess(host(out.h_final), ref["h_final"], aref["h_final"])
        print("   componentwise y %.3e h_final %.3e" % (ex_y, ex_h), flush=True)
        assert ex_y <= comp_tol(io) and ex_h <= comp_tol(io), (ex_y, ex_h)
        # the same forward on the rows of the selected experts only
        # (selection and weights as the routed call returned them, so both calls mix with the same bits)
        sel = run_xe_selected(p, out.topk_idx.cpu().numpy(), out.topk_w.cpu().numpy(), Q, io, h0=h0v, d_none=d_none)
        l2, linf = rel_errors(host(sel.y), ref["y"], (0, 2))
        assert l2 <= TOL[io] and linf <= TOL[io], ("selected y", d_none, l2, linf)
        l2, linf = rel_errors(host(sel.h_final), ref["h_final"], (0, 1))
        assert l2 <= TOL[io] and linf <= TOL[io], ("selected h_final", d_none, l2, linf)
        if io == "bf16" and P % 8 == 0 and N % 8 == 0 and Q in (64, 128, 256) and k <= 4:
            # slot kernels: both entries run the same launches on the same rows
            assert torch.equal(sel.y, out.y) and torch.equal(sel.h_final, out.h_final)


def test_xe_with_one_shared_stream_is_the_shared_x_forward():
    """Equal x^(e) for all experts: the rank-k injection collapses to Bmix x^T."""
    cfg = (2, 200, 4, 16, 32, 2, 4, 2, 32, "f32")
    w, p = make_problem(cfg, seed=5)
    p["x_experts"] = np.repeat(p["x"][:, :, None], 4, axis=2).copy()
    xe = run_xe(p, w.top_k, w.chunk, "f32", d_none=True)
    mixed = run_mixer(p, w.top_k, w.chunk, "f32", d_none=True)
    l2, linf = rel_errors(host(xe.y), host(mixed.y), (0, 2))
    assert l2 <= 1e-4 and linf <= 1e-4, (l2, linf)
    l2, linf = rel_errors(host(xe.h_final), host(mixed.h_final), (0, 1))
    assert l2 <= 1e-4 and linf <= 1e-4, (l2, linf)


def test_xe_empty_sequence_and_workspace_errors():
    dev = "cuda:0"
    h0 = torch.randn((2, 2, 8, 4), device=dev)
    out = sw.swimba_mixer_fwd_xe(torch.zeros((2, 0, 3, 2, 8), device=dev), torch.zeros((2, 0, 2), device=dev),
                                 -torch.ones(2, device=dev), None, torch.zeros((2, 0, 3, 1, 4), device=dev),
                                 torch.zeros((2, 0, 3, 1, 4), device=dev), torch.zeros((2, 0, 3), device=dev), 2, 16, h0)
    torch.cuda.synchronize()
    assert out.y.shape == (2, 0, 2, 8)
    assert torch.equal(out.h_final, h0)
    with pytest.raises(RuntimeError):
        sw.swimba_mixer_fwd_xe(torch.zeros((1, 8, 3, 2, 8), device=dev), torch.zeros((1, 8, 2), device=dev),
                               -torch.ones(2, device=dev), None, torch.zeros((1, 8, 3, 1, 4), device=dev),
                               torch.zeros((1, 8, 3, 1, 4), device=dev), torch.zeros((1, 8, 3), device=dev), 2, 16,
                               workspace=torch.empty(256, dtype=torch.uint8, device=dev))
