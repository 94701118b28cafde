"""Seeded random shapes through the bf16 MFMA path (P = 64, N = 128) and the projection in front
of it: ragged lengths, every chunk size, group / head / expert / top-k combinations, with and
without an initial state and a skip term.  Each case is checked element by element against the
oracle like the fixed cases elsewhere; the point is coverage of combinations nobody wrote down."""
import numpy as np
import pytest
import torch

from oracle import swimba_oracle as orc
from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import TOL, host, rel_errors, to_device

pytestmark = pytest.mark.gpu


def random_cases(n, seed, min_len=1):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        G = int(rng.choice([1, 1, 2, 4]))
        H = G * int(rng.choice([1, 2, 3]))
        Q = int(rng.choice([64, 128, 256]))
        L = int(rng.integers(min_len, 3 * Q + 40))
        B = int(rng.choice([1, 2, 3]))
        E = int(rng.choice([1, 2, 3, 4, 8, 16, 33]))
        k = int(rng.integers(1, min(E, 6) + 1))
        cases.append((B, L, H, G, E, k, Q, bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), 1000 + i))
    return cases


def head_dim_of(seed):
    """P = 64 is the kernels' own size; smaller multiples of 8 run on them with zero channels."""
    return [64, 32, 64, 16, 8, 40, 64, 48, 24, 64, 56][seed % 11]


def state_size_of(seed):
    """N = 128 is the kernels' own size; smaller multiples of 8 run on them zero-padded."""
    return [128, 128, 64, 16, 96, 8, 32, 120][seed % 8]


@pytest.mark.parametrize("case", random_cases(24, 20260311), ids=lambda c: "B%dL%dH%dG%dE%dk%dQ%d_h0%d_D%d_s%d" % c)
def test_random_mfma_shapes_match_oracle(case):
    B, L, H, G, E, k, Q, with_h0, with_D, seed = case
    P, N = head_dim_of(seed), state_size_of(seed)
    w = synth.Workload("rnd", B, L, H, P, N, G, E, k, Q, "bf16", 7)
    p = synth.make_inputs(w, seed=seed)
    rng = np.random.default_rng(seed)
    p["D"] = rng.standard_normal(H).astype(np.float32)
    h0 = (0.1 * rng.standard_normal((B, H, P, N))).astype(np.float32) if with_h0 else None
    D = p["D"] if with_D else None
    ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], D, p["B_experts"], p["C_experts"], p["router_logits"], k, h0=h0)
    d = to_device(p, "bf16")
    out = sw.swimba_mixer_fwd(d["x"], d["dt"], d["A"], d["D"] if with_D else None, d["B_experts"], d["C_experts"],
                              d["router_logits"], k, Q, None if h0 is None else torch.from_numpy(h0).to("cuda:0"),
                              want_topk=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
    np.testing.assert_allclose(host(out.topk_w), ref["topk_w"], rtol=1e-5, atol=1e-30)
    l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
    hl2, hlinf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
    print(case, "P", P, "N", N, "y l2 %.2e linf %.2e  h_final l2 %.2e" % (l2, linf, hl2), flush=True)
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)
    assert hl2 <= TOL["bf16"] and hlinf <= TOL["bf16"], (hl2, hlinf)


# at least 16 tokens: the projected streams are rounded to bf16 on the way (two more roundings per
# product than with given streams), and the worst (batch, head) slice of a 2-token output is a
# noisy statistic right at the bar
@pytest.mark.parametrize("case", random_cases(10, 77, min_len=16), ids=lambda c: "B%dL%dH%dG%dE%dk%dQ%d_h0%d_D%d_s%d" % c)
def test_random_features_to_y_match_oracle_chain(case):
    B, L, H, G, E, k, Q, with_h0, with_D, seed = case
    P, N = head_dim_of(seed + 3), state_size_of(seed + 1)
    rng = np.random.default_rng(seed + 5)
    Dm = int(rng.choice([16, 48, 64, 80, 256]))
    rd = synth.round_to_bf16
    u = rd(rng.standard_normal((B, L, Dm)).astype(np.float32))
    WB = rd((rng.standard_normal((E, G, N, Dm)) / np.sqrt(Dm)).astype(np.float32))
    WC = rd((rng.standard_normal((E, G, N, Dm)) / np.sqrt(Dm)).astype(np.float32))
    w = synth.Workload("rnd", B, L, H, P, N, G, E, k, Q, "bf16", 7)
    p = synth.make_inputs(w, seed=seed)
    g = p["router_logits"]
    D = rng.standard_normal(H).astype(np.float32) if with_D else None
    h0 = (0.1 * rng.standard_normal((B, H, P, N))).astype(np.float32) if with_h0 else None
    rp = orc.expert_proj(u, WB, WC, g, k, fill=0.0)
    ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], D, rp["B_experts"].astype(np.float32),
                        rp["C_experts"].astype(np.float32), g, k, h0=h0)
    bf = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).to("cuda:0")
    out = sw.swimba_mixer_fwd_proj(bf(u), bf(WB), bf(WC), bf(p["x"]), bf(p["dt"]), torch.from_numpy(p["A"]).to("cuda:0"),
                                   None if D is None else torch.from_numpy(D).to("cuda:0"), bf(g), k, Q,
                                   None if h0 is None else torch.from_numpy(h0).to("cuda:0"), want_topk=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
    l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
    hl2, hlinf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
    print(case, "P", P, "N", N, "Dm", Dm, "y l2 %.2e linf %.2e  h_final l2 %.2e" % (l2, linf, hl2), flush=True)
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)
    assert hl2 <= TOL["bf16"] and hlinf <= TOL["bf16"], (hl2, hlinf)


def random_generic_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for i in range(n):
        G = int(rng.choice([1, 2, 3]))
        H = G * int(rng.choice([1, 2]))
        P = int(rng.choice([1, 3, 8, 16, 24, 40]))
        N = int(rng.choice([1, 5, 16, 33, 64, 70]))
        Q = int(rng.choice([1, 7, 16, 32, 48, 100]))
        L = int(rng.integers(1, 3 * Q + 9))
        E = int(rng.choice([1, 2, 5, 8, 19]))
        k = int(rng.integers(1, min(E, 4) + 1))
        io = str(rng.choice(["f32", "bf16"]))
        cases.append((int(rng.choice([1, 2])), L, H, P, N, G, E, k, Q, io, 2000 + i))
    return cases


@pytest.mark.parametrize("case", random_generic_cases(16, 5), ids=lambda c: "B%dL%dH%dP%dN%dG%dE%dk%dQ%d%s_s%d" % c)
def test_random_shapes_on_the_fp32_kernels_match_oracle(case):
    B, L, H, P, N, G, E, k, Q, io, seed = case
    w = synth.Workload("rnd", B, L, H, P, N, G, E, k, Q, io, 7)
    p = synth.make_inputs(w, seed=seed)
    rng = np.random.default_rng(seed)
    p["D"] = rng.standard_normal(H).astype(np.float32)
    h0 = (0.1 * rng.standard_normal((B, H, P, N))).astype(np.float32)
    ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], p["D"], p["B_experts"], p["C_experts"], p["router_logits"], k, h0=h0)
    d = to_device(p, io)
    out = sw.swimba_mixer_fwd(d["x"], d["dt"], d["A"], d["D"], d["B_experts"], d["C_experts"], d["router_logits"],
                              k, Q, torch.from_numpy(h0).to("cuda:0"), want_topk=True)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
    l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
    hl2, hlinf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
    print(case, "y l2 %.2e linf %.2e  h_final l2 %.2e" % (l2, linf, hl2), flush=True)
    assert l2 <= TOL[io] and linf <= TOL[io], (l2, linf)
    assert hl2 <= 1e-4 and hlinf <= 1e-4, (hl2, hlinf)      # the state is fp32 arithmetic on both io types
