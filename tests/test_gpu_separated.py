"""GPU parity of the separated-SSM contrast (one state trajectory per expert) against
the oracle's sequential evaluation of the same definition."""
import numpy as np
import pytest
import torch

from oracle import swimba_oracle as orc
from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import TOL, host, rel_errors, run_mixer, to_device

pytestmark = pytest.mark.gpu


def run_separated(p, top_k, chunk, io, d_none=False):
    d = to_device(p, io)
    out = sw.swimba_separated_fwd(d["x"], d["dt"], d["A"], None if d_none else d["D"], d["B_experts"],
                                  d["C_experts"], d["router_logits"], top_k, chunk, want_topk=True)
    torch.cuda.synchronize()
    return out


SHAPES = [
    # B, L, H, P, N, G, E, k, Q, io
    (2, 96, 4, 16, 16, 2, 4, 2, 32, "f32"),
    (1, 77, 6, 8, 24, 3, 5, 5, 16, "f32"),       # ragged, dense routing
    (2, 130, 2, 32, 64, 1, 3, 1, 64, "f32"),     # top-1
    (2, 96, 4, 16, 16, 2, 4, 2, 32, "bf16"),     # bf16 io on the fp32 kernels
    (2, 300, 4, 64, 128, 2, 8, 2, 128, "bf16"),  # MFMA kernels, ragged tail, groups
    (1, 257, 2, 64, 128, 1, 4, 3, 64, "bf16"),
    (1, 520, 4, 64, 128, 2, 16, 1, 256, "bf16"),
]


@pytest.mark.parametrize("cfg", SHAPES, ids=lambda c: "B%dL%dH%dP%dN%dG%dE%dk%dQ%d%s" % c)
def test_separated_matches_oracle(cfg):
    B, L, H, P, N, G, E, k, Q, io = cfg
    w = synth.Workload("sep", B, L, H, P, N, G, E, k, Q, io, 7)
    p = synth.make_inputs(w, seed=hash(cfg[:9]) % 100000 + 1)
    p["D"] = np.random.default_rng(5).standard_normal(H).astype(np.float32)
    for d_none in (True, False):
        ref = orc.separated_fwd(p["x"], p["dt"], p["A"], None if d_none else p["D"], p["B_experts"],
                                p["C_experts"], p["router_logits"], k)
        out = run_separated(p, k, Q, io, d_none=d_none)
        np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
        np.testing.assert_allclose(host(out.topk_w), ref["topk_w"], rtol=1e-5, atol=1e-30)
        l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
        print(cfg, "D=0" if d_none else "D", "rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
        assert l2 <= TOL[io] and linf <= TOL[io], (d_none, l2, linf)


def test_separated_equals_mixed_when_experts_share_b():
    """Shared input projection, dense routing (paper: the mixed/separated equivalence
    theorem): with B^(e) = B for all e and k = E the two paths give the same output.
    Both run on the GPU here; each is also tied to its own oracle above."""
    w = synth.Workload("thm", 2, 200, 4, 16, 32, 2, 4, 4, 32, "f32", 11)
    p = synth.make_inputs(w, seed=77)
    p["B_experts"] = np.repeat(p["B_experts"][:, :, :1], w.nexperts, axis=2).copy()
    mixed = run_mixer(p, w.top_k, w.chunk, "f32")
    sep = run_separated(p, w.top_k, w.chunk, "f32")
    l2, linf = rel_errors(host(sep.y), host(mixed.y), (0, 2))
    assert l2 <= 1e-4 and linf <= 1e-4, (l2, linf)
    ref = orc.separated_fwd(p["x"], p["dt"], p["A"], p["D"], p["B_experts"], p["C_experts"],
                            p["router_logits"], w.top_k)
    l2, linf = rel_errors(host(sep.y), ref["y"], (0, 2))
    assert l2 <= 1e-4 and linf <= 1e-4, (l2, linf)


def test_separated_empty_and_workspace_errors():
    dev = "cuda:0"
    x = torch.zeros((2, 0, 2, 8), device=dev)
    out = sw.swimba_separated_fwd(x, torch.zeros((2, 0, 2), device=dev), -torch.ones(2, device=dev), None,
                                  torch.zeros((2, 0, 3, 1, 4), device=dev), torch.zeros((2, 0, 3, 1, 4), device=dev),
                                  torch.zeros((2, 0, 3), device=dev), 2, 16)
    assert out.y.shape == (2, 0, 2, 8)
    x = torch.zeros((1, 8, 2, 8), device=dev)
    with pytest.raises(RuntimeError):
        sw.swimba_separated_fwd(x, torch.zeros((1, 8, 2), device=dev), -torch.ones(2, device=dev), None,
                                torch.zeros((1, 8, 3, 1, 4), device=dev), torch.zeros((1, 8, 3, 1, 4), device=dev),
                                torch.zeros((1, 8, 3), device=dev), 2, 16,
                                workspace=torch.empty(256, dtype=torch.uint8, device=dev))
