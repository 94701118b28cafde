"""GPU parity of the routed expert in-projection (the step upstream of the mixer) against
the oracle, and of projection + mixer end to end."""
import numpy as np
import pytest
import torch

from oracle import swimba_oracle as orc
from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import IO, TOL, host, rel_errors

pytestmark = pytest.mark.gpu
SENTINEL = 7.0


def make_problem(B, L, Dm, E, G, N, io, seed):
    rng = np.random.default_rng(seed)
    rd = synth.round_to_bf16 if io == "bf16" else (lambda a: a)
    u = rd(rng.standard_normal((B, L, Dm)).astype(np.float32))
    # weights ~ N(0, 1/Dm): projected rows have unit-order entries
    WB = rd((rng.standard_normal((E, G, N, Dm)) / np.sqrt(Dm)).astype(np.float32))
    WC = rd((rng.standard_normal((E, G, N, Dm)) / np.sqrt(Dm)).astype(np.float32))
    g = rd(rng.standard_normal((B, L, E)).astype(np.float32))
    return u, WB, WC, g


def dev(a, io):
    return torch.from_numpy(np.ascontiguousarray(a)).to(IO[io]).to("cuda:0")


SHAPES = [
    # B, L, Dm, E, G, N, k, io
    (2, 37, 24, 4, 2, 8, 2, "f32"),
    (1, 50, 33, 5, 1, 20, 5, "f32"),        # dense routing, odd sizes
    (2, 40, 48, 4, 1, 24, 2, "bf16"),       # bf16 on the plain-arithmetic kernel (G*N % 64 != 0)
    (2, 300, 256, 8, 1, 128, 2, "bf16"),    # MFMA: ragged token tiles
    (1, 130, 80, 8, 2, 64, 1, "bf16"),      # MFMA: d_model = 64 + 16 (tail k-step), top-1
    (1, 70, 64, 16, 8, 128, 3, "bf16"),     # MFMA: 2048 output columns (8 column blocks), k = 3
    (1, 5, 32, 16, 1, 64, 2, "bf16"),       # MFMA: most experts receive no token
    (1, 256, 768, 8, 1, 128, 2, "bf16"),    # MFMA: a 130M-sized model width
]


@pytest.mark.parametrize("cfg", SHAPES, ids=lambda c: "B%dL%dD%dE%dG%dN%dk%d%s" % c)
def test_expert_proj_matches_oracle(cfg):
    B, L, Dm, E, G, N, k, io = cfg
    u, WB, WC, g = make_problem(B, L, Dm, E, G, N, io, seed=hash(cfg[:7]) % 100000)
    ref = orc.expert_proj(u, WB, WC, g, k, fill=SENTINEL)
    Bo = torch.full((B, L, E, G, N), SENTINEL, dtype=IO[io], device="cuda:0")
    Co = torch.full((B, L, E, G, N), SENTINEL, dtype=IO[io], device="cuda:0")
    out = sw.swimba_expert_proj(dev(u, io), dev(WB, io), dev(WC, io), dev(g, io), k, B_experts=Bo, C_experts=Co,
                                want_topk=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
    np.testing.assert_allclose(host(out.topk_w), ref["topk_w"], rtol=1e-5, atol=1e-30)
    keep = np.zeros((B, L, E), dtype=bool)
    np.put_along_axis(keep, ref["topk_idx"].astype(np.int64), True, axis=-1)
    for name, got, want in (("B", host(out.B_experts), ref["B_experts"]), ("C", host(out.C_experts), ref["C_experts"])):
        # rows of inactive experts are untouched
        assert (got[~keep] == SENTINEL).all(), name
        l2 = np.linalg.norm(got[keep] - want[keep]) / np.linalg.norm(want[keep])
        linf = np.abs(got[keep] - want[keep]).max() / np.abs(want[keep]).max()
        print(cfg, name, "rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
        assert l2 <= TOL[io] and linf <= TOL[io], (name, l2, linf)


ROUTER_LINEAR_SHAPES = [
    # B, L, Dm, E, io
    (2, 37, 24, 4, "f32"), (1, 50, 33, 5, "f32"), (1, 3, 700, 256, "f32"),
    (2, 40, 48, 4, "bf16"), (1, 130, 77, 8, "bf16"),          # 77 features: element-wise path
    (2, 300, 768, 8, "bf16"), (1, 9, 1024, 16, "bf16"), (1, 1, 8, 1, "bf16"),
]


@pytest.mark.parametrize("cfg", ROUTER_LINEAR_SHAPES, ids=lambda c: "B%dL%dD%dE%d%s" % c)
def test_router_linear_matches_oracle(cfg):
    B, L, Dm, E, io = cfg
    rng = np.random.default_rng(hash(cfg[:4]) % 100000)
    rd = synth.round_to_bf16 if io == "bf16" else (lambda a: a)
    u = rd(rng.standard_normal((B, L, Dm)).astype(np.float32))
    Wg = rd((rng.standard_normal((E, Dm)) / np.sqrt(Dm)).astype(np.float32))
    ref = orc.router_linear(u, Wg)
    got = sw.swimba_router_linear(dev(u, io), dev(Wg, io))
    torch.cuda.synchronize()
    assert got.shape == (B, L, E) and got.dtype == IO[io]
    g = host(got)
    l2 = np.linalg.norm(g - ref) / np.linalg.norm(ref)
    linf = np.abs(g - ref).max() / np.abs(ref).max()
    print(cfg, "logits rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
    assert l2 <= TOL[io] and linf <= TOL[io], (l2, linf)


def test_projection_then_mixer_end_to_end():
    """Token features -> routed projection -> mixer, all on the GPU, against the oracle chain
    (oracle projections are not rounded to bf16 in between)."""
    B, L, Dm, E, G, N, k, H, P, Q = 2, 300, 128, 8, 1, 128, 2, 4, 64, 128
    u, WB, WC, g = make_problem(B, L, Dm, E, G, N, "bf16", seed=99)
    w = synth.Workload("e2e", B, L, H, P, N, G, E, k, Q, "bf16", 7)
    p = synth.make_inputs(w, seed=98)
    proj = sw.swimba_expert_proj(dev(u, "bf16"), dev(WB, "bf16"), dev(WC, "bf16"), dev(g, "bf16"), k)
    out = sw.swimba_mixer_fwd(dev(p["x"], "bf16"), dev(p["dt"], "bf16"), torch.from_numpy(p["A"]).to("cuda:0"), None,
                              proj.B_experts, proj.C_experts, dev(g, "bf16"), k, Q)
    torch.cuda.synchronize()
    rp = orc.expert_proj(u, WB, WC, g, k, fill=0.0)
    ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], None, rp["B_experts"].astype(np.float32),
                        rp["C_experts"].astype(np.float32), g, k)
    l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
    print("projection + mixer: y rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)


def test_expert_proj_empty_and_errors():
    d = "cuda:0"
    out = sw.swimba_expert_proj(torch.zeros((2, 0, 16), device=d), torch.zeros((3, 1, 4, 16), device=d),
                                torch.zeros((3, 1, 4, 16), device=d), torch.zeros((2, 0, 3), device=d), 2)
    assert out.B_experts.shape == (2, 0, 3, 1, 4)
    with pytest.raises(RuntimeError):
        sw.swimba_expert_proj(torch.zeros((1, 4, 16), device=d), torch.zeros((3, 1, 4, 16), device=d),
                              torch.zeros((3, 1, 4, 16), device=d), torch.zeros((1, 4, 3), device=d), 2,
                              workspace=torch.empty(256, dtype=torch.uint8, device=d))
