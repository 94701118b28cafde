"""GPU parity of the routed in-projection with the experts' input streams as a third block of
output columns, and of token features -> y through the expert-X forward, against the oracle."""
import numpy as np
import pytest
import torch

from oracle import swimba_oracle as orc
from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import IO, TOL, U_BF16, host, rel_errors

pytestmark = pytest.mark.gpu


def make_problem(B, L, Dm, E, G, N, H, P, io, seed):
    rng = np.random.default_rng(seed)
    rd = synth.round_to_bf16 if io == "bf16" else (lambda a: a)
    u = rd(rng.standard_normal((B, L, Dm)).astype(np.float32))
    # weights ~ N(0, 1/Dm): projected rows have unit-order entries
    WB = rd((rng.standard_normal((E, G, N, Dm)) / np.sqrt(Dm)).astype(np.float32))
    WC = rd((rng.standard_normal((E, G, N, Dm)) / np.sqrt(Dm)).astype(np.float32))
    WX = rd((rng.standard_normal((E, H, P, Dm)) / np.sqrt(Dm)).astype(np.float32))
    g = rd(rng.standard_normal((B, L, E)).astype(np.float32))
    return u, WB, WC, WX, g


def dev(a, io):
    return torch.from_numpy(np.ascontiguousarray(a)).to(IO[io]).to("cuda:0")


SHAPES = [
    # B, L, Dm, E, G, N, H, P, k, io
    (2, 37, 24, 4, 2, 8, 4, 6, 2, "f32"),
    (1, 50, 33, 5, 1, 20, 3, 5, 5, "f32"),         # dense routing, odd sizes
    (2, 40, 48, 4, 1, 24, 2, 16, 2, "bf16"),       # bf16 on the plain-arithmetic kernel
    (2, 300, 256, 8, 1, 128, 4, 64, 2, "bf16"),    # MFMA: 256 + 256 columns, ragged token tiles
    (1, 130, 80, 8, 2, 64, 6, 32, 1, "bf16"),      # MFMA: X block of 192 columns ends inside a workgroup's 256
    (1, 70, 64, 16, 8, 128, 8, 64, 3, "bf16"),     # MFMA: 2048 + 512 columns, k = 3
    (1, 5, 32, 16, 1, 64, 1, 64, 2, "bf16"),       # MFMA: most experts receive no token
    (1, 256, 768, 8, 1, 128, 24, 64, 2, "bf16"),   # MFMA: a 130M-sized model width, 1536 X columns
    (1, 64, 64, 4, 1, 64, 3, 16, 2, "bf16"),       # H*P = 48: the X block keeps the whole product off the GEMM
]


@pytest.mark.parametrize("cfg", SHAPES, ids=lambda c: "B%dL%dD%dE%dG%dN%dH%dP%dk%d%s" % c)
def test_expert_proj_x_matches_oracle(cfg):
    B, L, Dm, E, G, N, H, P, k, io = cfg
    u, WB, WC, WX, g = make_problem(B, L, Dm, E, G, N, H, P, io, seed=hash(cfg[:9]) % 100000)
    rbc = orc.expert_proj(u, WB, WC, g, k, fill=0.0)
    rx = orc.expert_proj_x(u, WX, g, k)
    Bs, Cs, xs, idx, w = sw.swimba_expert_proj_x_selected(dev(u, io), dev(WB, io), dev(WC, io), dev(WX, io),
                                                          dev(g, io), k)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), rx["topk_idx"])
    np.testing.assert_allclose(host(w), rx["topk_w"], rtol=1e-5, atol=1e-30)
    take = lambda a: np.take_along_axis(a, rx["topk_idx"].astype(np.int64)[..., None, None], axis=2)
    # one rounding of an fp32-accumulated sum; entries are of order one
    tol = 2 * U_BF16 if io == "bf16" else 1e-5
    for name, got, want in (("B", host(Bs), take(rbc["B_experts"])), ("C", host(Cs), take(rbc["C_experts"])),
                            ("x", host(xs), rx["x_sel"])):
        assert got.shape == want.shape, name
        err = np.abs(got - want).max() / max(np.abs(want).max(), 1e-300)
        l2, _ = rel_errors(got, want, (0,))
        print(cfg, name, "linf %.3e l2 %.3e" % (err, l2), flush=True)
        assert err <= tol and l2 <= tol, (name, err, l2)
    # the B and C blocks are the same numbers the two-block projection writes
    two = sw.swimba_expert_proj_selected(dev(u, io), dev(WB, io), dev(WC, io), dev(g, io), k)
    torch.cuda.synchronize()
    assert torch.equal(two.B_experts, Bs) and torch.equal(two.C_experts, Cs)


@pytest.mark.parametrize("cfg", [(2, 300, 128, 8, 2, 128, 4, 64, 2, 128, "bf16"), (1, 77, 40, 5, 1, 16, 3, 8, 3, 16, "f32"),
                                 (1, 520, 256, 8, 1, 128, 8, 64, 2, 256, "bf16")],
                         ids=lambda c: "B%dL%dD%dE%dG%dN%dH%dP%dk%dQ%d%s" % c)
def test_features_to_y_with_projected_input_streams(cfg):
    """Token features -> [B | C | X] of the selected experts -> expert-X forward, one call, against the
    oracle chain (whose projections are not rounded to the io dtype in between)."""
    B, L, Dm, E, G, N, H, P, k, Q, io = cfg
    u, WB, WC, WX, g = make_problem(B, L, Dm, E, G, N, H, P, io, seed=11 + L)
    rng = np.random.default_rng(5 + L)
    w = synth.Workload("xp", B, L, H, P, N, G, E, k, Q, io, 3)
    p = synth.make_inputs(w, seed=7)
    D = rng.standard_normal(H).astype(np.float32)
    h0 = (rng.standard_normal((B, H, P, N)) * 0.1).astype(np.float32)
    rbc = orc.expert_proj(u, WB, WC, g, k, fill=0.0)
    rx = orc.expert_proj_x(u, WX, g, k)
    xe = np.zeros((B, L, E, H, P))
    np.put_along_axis(xe, rx["topk_idx"].astype(np.int64)[..., None, None], rx["x_sel"], axis=2)
    ref = orc.mixer_fwd_xe(xe.astype(np.float32), p["dt"], p["A"], D, rbc["B_experts"].astype(np.float32),
                           rbc["C_experts"].astype(np.float32), g, k, h0=h0)
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    out = sw.swimba_mixer_fwd_xe_proj(dev(u, io), dev(WB, io), dev(WC, io), dev(WX, io), dev(p["dt"], io), d(p["A"]),
                                      d(D), dev(g, io), k, Q, d(h0), want_topk=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
    l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
    print(cfg, "features -> y: rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
    # the oracle's float32 copies of its own projections differ from the exact ones by 6e-8: far below the bar
    assert l2 <= TOL[io] and linf <= TOL[io], (l2, linf)
    l2, linf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
    assert l2 <= TOL[io] and linf <= TOL[io], (l2, linf)
    # the same result from the two calls it is made of
    Bs, Cs, xs, idx, wts = sw.swimba_expert_proj_x_selected(dev(u, io), dev(WB, io), dev(WC, io), dev(WX, io),
                                                            dev(g, io), k)
    two = sw.swimba_mixer_fwd_xe_selected(xs, dev(p["dt"], io), d(p["A"]), d(D), Bs, Cs, wts, Q, d(h0))
    torch.cuda.synchronize()
    assert torch.equal(two.y, out.y) and torch.equal(two.h_final, out.h_final)


def test_expert_proj_x_empty_and_errors():
    dv = "cuda:0"
    Bs, Cs, xs, idx, w = sw.swimba_expert_proj_x_selected(
        torch.zeros((2, 0, 16), device=dv), torch.zeros((3, 1, 4, 16), device=dv), torch.zeros((3, 1, 4, 16), device=dv),
        torch.zeros((3, 2, 8, 16), device=dv), torch.zeros((2, 0, 3), device=dv), 2)
    torch.cuda.synchronize()
    assert xs.shape == (2, 0, 2, 2, 8)
    with pytest.raises(RuntimeError):   # workspace too small
        sw.swimba_expert_proj_x_selected(
            torch.zeros((1, 4, 16), device=dv), torch.zeros((3, 1, 4, 16), device=dv),
            torch.zeros((3, 1, 4, 16), device=dv), torch.zeros((3, 2, 8, 16), device=dv),
            torch.zeros((1, 4, 3), device=dv), 2, workspace=torch.empty(256, dtype=torch.uint8, device=dv))
