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
from gpu_util import TOL, abs_inputs, comp_tol, componentwise_excess, host, rel_errors, to_device

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


# Slices of fewer tokens than this are held to the componentwise bound only.  The norm of such a
# slice of y is made of a handful of scalars Cmix_t . Bmix_s, each a sum of N products of either
# sign whose value can come out far below the size of its terms, while the rounding error
# follows the terms: error / norm is then a ratio with a heavy tail (for one scalar,
# P(ratio > 10 x typical) is about 8 %), whatever the kernel does.  Seen on the case
# B3 L2 H8 G4 E4 k3 Q128 (P 24, N 120, projected from 48 features): worst slice 1.84e-2 against a
# typical 4e-3, while every element sits at 8e-4 of its own sum of absolute products.
MIN_TOKENS_NORMWISE = 16


def assert_normwise(L, l2, linf, hl2, hlinf):
    if L >= MIN_TOKENS_NORMWISE:
        assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)
    assert hl2 <= TOL["bf16"] and hlinf <= TOL["bf16"], (hl2, hlinf)


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
    q = abs_inputs(p)
    aref = orc.mixer_fwd(q["x"], q["dt"], q["A"], None if D is None else np.abs(D), q["B_experts"], q["C_experts"],
                         q["router_logits"], k, h0=None if h0 is None else np.abs(h0))
    ey = componentwise_excess(host(out.y), ref["y"], aref["y"])
    eh = componentwise_excess(host(out.h_final), ref["h_final"], aref["h_final"])
    print(case, "P", P, "N", N, "y l2 %.2e linf %.2e  h_final l2 %.2e  componentwise %.2e %.2e" % (l2, linf, hl2, ey, eh),
          flush=True)
    assert ey <= comp_tol("bf16") and eh <= comp_tol("bf16"), (ey, eh)
    assert_normwise(L, l2, linf, hl2, hlinf)


@pytest.mark.parametrize("case", random_cases(10, 77), ids=lambda c: "B%dL%dH%dG%dE%dk%dQ%d_h0%d_D%d_s%d" % c)
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
    aB, aC = np.abs(rp["B_experts"]).astype(np.float32), np.abs(rp["C_experts"]).astype(np.float32)
    aref = orc.mixer_fwd(np.abs(p["x"]), p["dt"], p["A"], None if D is None else np.abs(D), aB, aC, g, k,
                         h0=None if h0 is None else np.abs(h0))
    # the projected streams are stored in bf16 before they are mixed: one more rounding on each
    # side of every product than with given streams
    ctol = comp_tol("bf16", roundings=7)
    ey = componentwise_excess(host(out.y), ref["y"], aref["y"])
    eh = componentwise_excess(host(out.h_final), ref["h_final"], aref["h_final"])
    print(case, "P", P, "N", N, "Dm", Dm, "y l2 %.2e linf %.2e  h_final l2 %.2e  componentwise %.2e %.2e"
          % (l2, linf, hl2, ey, eh), flush=True)
    assert ey <= ctol and eh <= ctol, (ey, eh)
    assert_normwise(L, l2, linf, hl2, hlinf)


@pytest.mark.parametrize("L", [1, 2, 3, 5, 8, 15])
def test_short_sequences_hold_the_componentwise_bound(L):
    """Sequences shorter than MIN_TOKENS_NORMWISE through both the forward on given streams and the
    features-to-y call: every element of y and h_final within the forward error bound of its own sum
    of products (5 roundings with given streams, 7 with projected ones), active sets exact."""
    for seed in range(4):
        B, H, G, E, k, Q = 3, 8, 4, 4, 3, (64, 128, 256)[seed % 3]
        P, N = head_dim_of(seed + 3), state_size_of(seed + 1)
        rng = np.random.default_rng(900 + 10 * L + seed)
        Dm = int(rng.choice([16, 48, 64]))
        rd = synth.round_to_bf16
        u = rd(rng.standard_normal((B, L, Dm)).astype(np.float32))
        WB = rd((rng.standard_normal((E, G, N, Dm)) / np.sqrt(Dm)).astype(np.float32))
        WC = rd((rng.standard_normal((E, G, N, Dm)) / np.sqrt(Dm)).astype(np.float32))
        w = synth.Workload("short", B, L, H, P, N, G, E, k, Q, "bf16", 7)
        p = synth.make_inputs(w, seed=700 + seed)
        g = p["router_logits"]
        D = rng.standard_normal(H).astype(np.float32)
        h0 = (0.1 * rng.standard_normal((B, H, P, N))).astype(np.float32) if seed % 2 else None
        ah0 = None if h0 is None else np.abs(h0)
        h0d = None if h0 is None else torch.from_numpy(h0).to("cuda:0")
        bf = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(torch.bfloat16).to("cuda:0")
        # given streams
        d = to_device(p, "bf16")
        out = sw.swimba_mixer_fwd(d["x"], d["dt"], d["A"], torch.from_numpy(D).to("cuda:0"), d["B_experts"],
                                  d["C_experts"], d["router_logits"], k, Q, h0d, want_topk=True)
        torch.cuda.synchronize()
        ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], D, p["B_experts"], p["C_experts"], g, k, h0=h0)
        q = abs_inputs(p)
        aref = orc.mixer_fwd(q["x"], q["dt"], q["A"], np.abs(D), q["B_experts"], q["C_experts"], g, k, h0=ah0)
        np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
        ey = componentwise_excess(host(out.y), ref["y"], aref["y"])
        eh = componentwise_excess(host(out.h_final), ref["h_final"], aref["h_final"])
        assert ey <= comp_tol("bf16") and eh <= comp_tol("bf16"), ("given", L, seed, ey, eh)
        # projected streams
        rp = orc.expert_proj(u, WB, WC, g, k, fill=0.0)
        rB, rC = rp["B_experts"].astype(np.float32), rp["C_experts"].astype(np.float32)
        ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], D, rB, rC, g, k, h0=h0)
        aref = orc.mixer_fwd(q["x"], q["dt"], q["A"], np.abs(D), np.abs(rB), np.abs(rC), g, k, h0=ah0)
        out = sw.swimba_mixer_fwd_proj(bf(u), bf(WB), bf(WC), d["x"], d["dt"], d["A"], torch.from_numpy(D).to("cuda:0"),
                                       d["router_logits"], k, Q, h0d, want_topk=True)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
        ey2 = componentwise_excess(host(out.y), ref["y"], aref["y"])
        eh2 = componentwise_excess(host(out.h_final), ref["h_final"], aref["h_final"])
        print("L", L, "seed", seed, "given %.2e %.2e  projected %.2e %.2e" % (ey, eh, ey2, eh2), flush=True)
        assert ey2 <= comp_tol("bf16", 7) and eh2 <= comp_tol("bf16", 7), ("projected", L, seed, ey2, eh2)


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
