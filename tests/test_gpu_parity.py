"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element
by element on the same seeded stored values."""
import numpy as np
import pytest
import torch

from oracle import swimba_oracle as orc
from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import TOL, abs_inputs, comp_tol, componentwise_excess, host, rel_errors, run_mixer, to_device

pytestmark = pytest.mark.gpu


def oracle_fwd(p, top_k, h0=None, d_none=False, **kw):
    return orc.mixer_fwd(p["x"], p["dt"], p["A"], None if d_none else p["D"], p["B_experts"],
                         p["C_experts"], p["router_logits"], top_k, h0=h0, **kw)


def check_componentwise(out, ref, p, w, h0=None, d_none=False, tag=""):
    """every element of y and h_final within the forward error bound of its own sum of products"""
    aref = oracle_fwd(abs_inputs(p), w.top_k, h0=None if h0 is None else np.abs(h0), d_none=d_none)
    ctol = comp_tol(w.io_dtype)
    ey = componentwise_excess(host(out.y), ref["y"], aref["y"])
    eh = componentwise_excess(host(out.h_final), ref["h_final"], aref["h_final"])
    assert ey <= ctol and eh <= ctol, (tag, "componentwise", d_none, ey, eh, ctol)


def check_fwd(p, w, h0=None, tag=""):
    """y with D as given, y with D = NULL (so the SSM term is not hidden behind the
    skip term), final state, and bit-exact active sets."""
    tol = TOL[w.io_dtype]
    for d_none in (False, True):
        ref = oracle_fwd(p, w.top_k, h0=h0, d_none=d_none)
        out = run_mixer(p, w.top_k, w.chunk, w.io_dtype, h0=h0, d_none=d_none)
        check_componentwise(out, ref, p, w, h0=h0, d_none=d_none, tag=tag)
        np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"], err_msg=tag)
        np.testing.assert_allclose(host(out.topk_w), ref["topk_w"], rtol=1e-5, atol=1e-30, err_msg=tag)
        l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
        assert l2 <= tol and linf <= tol, (tag, "y", d_none, l2, linf)
        l2, linf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
        # the state is fp32 on both io types; its operands are bf16-rounded on the MFMA path
        assert l2 <= tol and linf <= tol, (tag, "h_final", l2, linf)
    return out, ref


# ---- router ---------------------------------------------------------------------------

@pytest.mark.parametrize("E,k,io", [(4, 2, "f32"), (8, 2, "bf16"), (16, 2, "bf16"), (16, 16, "bf16"),
                                    (5, 1, "f32"), (64, 8, "bf16"), (1, 1, "bf16")])
def test_router_bit_exact(E, k, io):
    rng = np.random.default_rng(E * 100 + k)
    g = synth.to_storage(rng.standard_normal((3, 4099, E)).astype(np.float32), io)
    g[0, :7, : min(E, 3)] = 0.5          # planted ties
    g[0, 7, 0] = -0.0
    if E > 1:
        g[0, 7, 1] = 0.0
        g[1, :5, E - 1] = -np.inf
    ridx, rw = orc.router(g, k)
    t = torch.from_numpy(g).to({"f32": torch.float32, "bf16": torch.bfloat16}[io]).cuda()
    idx, wgt = sw.swimba_router_topk(t, k)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(idx.cpu().numpy(), ridx)
    np.testing.assert_allclose(host(wgt), rw, rtol=1e-5, atol=1e-30)


# ---- stages -------------------------------------------------------------------------------

@pytest.mark.parametrize("wi,L", [(0, 256), (0, 200), (1, 700)])
def test_stage_cumsum_and_carried_states(wi, L):
    w = synth.workload(wi).with_(seqlen=L, batch=2)
    if wi == 1:
        w = w.with_(nheads=6)
    p = synth.make_inputs(w)
    d = to_device(p, w.io_dtype)
    dims = sw.dims_of(d["x"], d["B_experts"], w.top_k, w.chunk)
    ws = sw.alloc_workspace(dims, "cuda:0")
    ws.zero_()
    sw.swimba_stage_router(dims, d["router_logits"], ws)
    sw.swimba_stage_cumsum(dims, d["dt"], d["A"], ws)
    sw.swimba_stage_mix(dims, d["B_experts"], d["C_experts"], d["router_logits"], ws)
    sw.swimba_stage_chunk_state(dims, d["x"], d["dt"], d["A"], d["B_experts"], ws)
    hf = torch.empty((w.batch, w.nheads, w.headdim, w.dstate), device="cuda:0")
    sw.swimba_stage_state_scan(dims, None, hf, ws)
    y = torch.empty_like(d["x"])
    sw.swimba_stage_output(dims, d["x"], d["dt"], d["D"], d["B_experts"], d["C_experts"], y, ws)
    torch.cuda.synchronize()
    v = sw.workspace_views(dims, ws)
    # cumsum against its plain definition in double
    Q, nc = w.chunk, (L + w.chunk - 1) // w.chunk
    a = np.zeros((w.batch, nc * Q, w.nheads))
    a[:, :L] = p["dt"].astype(np.float64) * p["A"].astype(np.float64)
    cs_ref = a.reshape(w.batch, nc, Q, w.nheads).cumsum(axis=2).transpose(0, 1, 3, 2)
    np.testing.assert_allclose(host(v["cs"]), cs_ref, rtol=2e-6, atol=1e-6)
    # carried states against the oracle's snapshots
    ref = oracle_fwd(p, w.top_k, snap_every=Q)
    tol = TOL[w.io_dtype]
    l2, linf = rel_errors(host(v["states"])[:, 1:], ref["snaps"][:, 1:], (0, 1, 2))
    assert l2 <= tol and linf <= tol, (l2, linf)
    assert not host(v["states"])[:, 0].any()
    l2, linf = rel_errors(host(hf), ref["h_final"], (0, 1))
    assert l2 <= tol and linf <= tol
    l2, linf = rel_errors(host(y), ref["y"], (0, 2))
    assert l2 <= tol and linf <= tol


# ---- whole forward, small shapes ---------------------------------------------------------

def test_workload0_fp32():
    w = synth.workload(0)
    check_fwd(synth.make_inputs(w), w, tag="workload0")


SMALL = [
    # B, L, H, P, N, G, E, k, Q, io
    (2, 96, 4, 16, 16, 2, 4, 2, 32, "f32"),
    (1, 77, 6, 8, 24, 3, 5, 5, 16, "f32"),      # ragged L, dense routing (k = E)
    (2, 130, 2, 32, 64, 1, 3, 1, 64, "f32"),    # top-1, ragged
    (1, 50, 2, 12, 20, 2, 4, 2, 256, "f32"),    # one chunk longer than L
    (3, 33, 3, 5, 7, 1, 2, 2, 1, "f32"),        # chunk of one token: pure recurrence
    (2, 300, 4, 64, 128, 2, 8, 2, 128, "f32"),  # fp32 at the MFMA shape
    (2, 96, 4, 16, 16, 2, 4, 2, 32, "bf16"),
    (1, 200, 4, 32, 64, 1, 8, 2, 64, "bf16"),
    # bf16 MFMA shape (P=64, N=128), every supported chunk length, ragged tails, groups, k=1, k=E
    (2, 300, 4, 64, 128, 2, 8, 2, 128, "bf16"),
    (1, 700, 6, 64, 128, 1, 8, 2, 256, "bf16"),
    (2, 256, 3, 64, 128, 3, 4, 4, 64, "bf16"),
    (1, 520, 8, 64, 128, 2, 16, 1, 256, "bf16"),
    (1, 31, 2, 64, 128, 1, 4, 2, 256, "bf16"),
    (2, 257, 2, 64, 128, 1, 8, 3, 64, "bf16"),
    # the limits of the routing tables: 256 experts, 16 active
    (1, 70, 2, 64, 128, 1, 256, 16, 64, "bf16"),
    (1, 40, 2, 8, 16, 2, 256, 16, 16, "f32"),
]


@pytest.mark.parametrize("cfg", SMALL, ids=lambda c: "B%dL%dH%dP%dN%dG%dE%dk%dQ%d%s" % c)
def test_small_shapes(cfg):
    B, L, H, P, N, G, E, k, Q, io = cfg
    w = synth.Workload("small", B, L, H, P, N, G, E, k, Q, io, 7)
    p = synth.make_inputs(w, seed=hash(cfg[:9]) % 100000)
    rng = np.random.default_rng(3)
    p["D"] = rng.standard_normal(H).astype(np.float32)
    h0 = rng.standard_normal((B, H, P, N)).astype(np.float32) * 0.1
    check_fwd(p, w, tag="zero-h0")
    check_fwd(p, w, h0=h0, tag="h0")


def test_chunk_size_invariance_and_extreme_decay():
    w = synth.workload(0).with_(seqlen=192)
    p = synth.make_inputs(w)
    p["dt"][:, 100:140] = 1.0
    p["A"][:] = np.array([-16, -16, -1, -8], np.float32)    # cumsum reaches about -1000 per chunk
    ref = oracle_fwd(p, w.top_k)
    for Q in (16, 64, 192, 256):
        out = run_mixer(p, w.top_k, Q, w.io_dtype)
        assert torch.isfinite(out.y).all()
        l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
        assert l2 <= 1e-4 and linf <= 1e-4, (Q, l2, linf)


@pytest.mark.parametrize("Q", [64, 128, 256])
def test_extreme_decay_on_the_mfma_kernels(Q):
    """bf16 io at the MFMA shape with A = -16 and dt = 1 over stretches of tokens, one inside a
    chunk and one across a chunk boundary for every Q: the per-chunk cumsum reaches about -640,
    far below the fp32 exponent range of exp(cs_i) * exp(-cs_j).  The decay has to be formed
    from differences only; the output must be finite and within the bf16 bar."""
    w = synth.Workload("decay", 2, 600, 4, 64, 128, 2, 8, 2, Q, "bf16", 7)
    p = synth.make_inputs(w, seed=1212)
    p["dt"][:, 100:140] = 1.0
    p["dt"][:, 250:262] = 1.0
    p["dt"][:, 500:530, 1] = 4.0            # dt * A = -64 per token on one head
    p["A"][:] = np.array([-16, -16, -1, -8], np.float32)
    rng = np.random.default_rng(5)
    h0 = rng.standard_normal((2, 4, 64, 128)).astype(np.float32) * 0.1
    for d_none in (True, False):
        ref = oracle_fwd(p, w.top_k, h0=h0, d_none=d_none)
        out = run_mixer(p, w.top_k, Q, "bf16", h0=h0, d_none=d_none)
        assert torch.isfinite(out.y).all() and torch.isfinite(out.h_final).all()
        check_componentwise(out, ref, p, w, h0=h0, d_none=d_none, tag="Q%d" % Q)
        l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
        assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (Q, d_none, l2, linf)
        l2, linf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
        assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (Q, "h_final", l2, linf)


@pytest.mark.parametrize("Q,io,P,N", [(256, "bf16", 64, 128), (64, "bf16", 64, 128), (128, "bf16", 32, 64),
                                      (64, "f32", 16, 16)])
def test_causality_is_bitwise(Q, io, P, N):
    """Changing every input at tokens >= s leaves y at tokens < s bitwise unchanged (paper: the
    recurrence is causal; in the chunked form nothing a token's output reads may depend on later
    tokens of its chunk or tile).  s inside a 32-token tile, at a tile edge, at a chunk edge."""
    w = synth.Workload("causal", 2, 2 * Q + 50, 4, P, N, 2, 8, 2, Q, io, 7)
    p = synth.make_inputs(w, seed=99)
    q = synth.make_inputs(w, seed=100)
    base = run_mixer(p, w.top_k, Q, io).y.clone()
    for s in (1, 37, 64, Q - 1, Q, Q + 32 + 5, 2 * Q + 49):
        mod = {}
        for name, v in p.items():
            if name in ("x", "dt", "B_experts", "C_experts", "router_logits"):
                mod[name] = np.concatenate([v[:, :s], q[name][:, s:]], axis=1)
            else:
                mod[name] = v
        got = run_mixer(mod, w.top_k, Q, io).y
        assert torch.equal(got[:, :s], base[:, :s]), s
        assert not torch.equal(got[:, s:], base[:, s:]), s


@pytest.mark.parametrize("io,P,N,Q", [("bf16", 64, 128, 256), ("f32", 16, 16, 64)])
def test_linearity_in_x(io, P, N, Q):
    """y(a x1 + b x2) = a y(x1) + b y(x2) with everything else fixed (paper: for given router
    weights and streams the layer is a linear map of x), to the path's tolerance; D = NULL and
    D given.  a and b are powers of two, so the combined input is rounded once."""
    w = synth.Workload("lin", 2, Q + 70, 4, P, N, 1, 4, 2, Q, io, 7)
    p = synth.make_inputs(w, seed=31)
    x2 = synth.make_inputs(w, seed=32)["x"]
    a, b = 0.5, -2.0
    comb = dict(p)
    comb["x"] = synth.to_storage(a * p["x"] + b * x2, io)
    for d_none in (True, False):
        ref = oracle_fwd(comb, w.top_k, d_none=d_none)["y"]
        y1 = host(run_mixer(p, w.top_k, Q, io, d_none=d_none).y)
        y2 = host(run_mixer(dict(p, x=x2), w.top_k, Q, io, d_none=d_none).y)
        yc = host(run_mixer(comb, w.top_k, Q, io, d_none=d_none).y)
        l2, linf = rel_errors(yc, ref, (0, 2))
        assert l2 <= TOL[io] and linf <= TOL[io], (d_none, l2, linf)
        # the linear combination of two GPU outputs carries both outputs' rounding errors
        l2, linf = rel_errors(a * y1 + b * y2, ref, (0, 2))
        assert l2 <= 2 * TOL[io] and linf <= 2 * TOL[io], (d_none, l2, linf)


def test_split_sequence_resume_and_determinism():
    w = synth.workload(0)
    p = synth.make_inputs(w)
    full = run_mixer(p, w.top_k, w.chunk, w.io_dtype)
    again = run_mixer(p, w.top_k, w.chunk, w.io_dtype)
    assert torch.equal(full.y, again.y) and torch.equal(full.h_final, again.h_final)
    half = {k: (v[:, :100] if v.ndim > 1 else v) for k, v in p.items()}
    rest = {k: (v[:, 100:] if v.ndim > 1 else v) for k, v in p.items()}
    r1 = run_mixer(half, w.top_k, w.chunk, w.io_dtype)
    r2 = run_mixer(rest, w.top_k, w.chunk, w.io_dtype, h0=r1.h_final.cpu().numpy())
    ref = oracle_fwd(p, w.top_k)
    got = np.concatenate([host(r1.y), host(r2.y)], 1)
    l2, linf = rel_errors(got, ref["y"], (0, 2))
    assert l2 <= 1e-4 and linf <= 1e-4
    l2, linf = rel_errors(host(r2.h_final), ref["h_final"], (0, 1))
    assert l2 <= 1e-4 and linf <= 1e-4


def test_empty_inputs():
    dev = "cuda:0"
    for B, L in ((0, 16), (2, 0)):
        x = torch.zeros((B, L, 2, 4), device=dev)
        Be = torch.zeros((B, L, 3, 1, 8), device=dev)
        h0 = torch.randn((B, 2, 4, 8), device=dev)
        out = sw.swimba_mixer_fwd(x, torch.ones((B, L, 2), device=dev), -torch.ones(2, device=dev), None,
                                  Be, Be, torch.zeros((B, L, 3), device=dev), 2, 8, h0)
        torch.cuda.synchronize()
        assert out.y.shape == x.shape
        assert torch.equal(out.h_final, h0)


# ---- decode step ---------------------------------------------------------------------------

@pytest.mark.parametrize("cfg", [(3, 4, 16, 16, 1, 4, 2, "f32"), (2, 6, 24, 40, 3, 5, 5, "f32"),
                                 (2, 4, 64, 128, 2, 8, 2, "bf16"), (2, 2, 48, 128, 1, 8, 1, "f32"),
                                 (1, 2, 64, 128, 1, 8, 2, "f32"),
                                 (3, 8, 64, 128, 1, 4, 1, "bf16"),      # 4 experts, top-1 (the paper's large model)
                                 (2, 16, 64, 128, 8, 8, 2, "bf16")],    # 8 B/C groups
                         ids=lambda c: "B%dH%dP%dN%dG%dE%dk%d%s" % c)
def test_step_matches_oracle_over_a_few_tokens(cfg):
    B, H, P, N, G, E, k, io = cfg
    steps = 5
    w = synth.Workload("dec", B, steps, H, P, N, G, E, k, 0, io, 9)
    p = synth.make_decode_inputs(w)
    p["D"] = np.linspace(-1, 1, H).astype(np.float32)
    d = to_device(p, io)
    st_gpu = d["state"].clone()
    st_ref = p["state"].astype(np.float64)
    tol = TOL[io]
    for t in range(steps):
        out = sw.swimba_step(st_gpu, d["x"][:, t].contiguous(), d["dt"][:, t].contiguous(), d["A"], d["D"],
                             d["B_experts"][:, t].contiguous(), d["C_experts"][:, t].contiguous(),
                             d["router_logits"][:, t].contiguous(), k, want_topk=True)
        torch.cuda.synchronize()
        y_ref, st_ref, idx_ref = orc.step(st_ref, p["x"][:, t], p["dt"][:, t], p["A"], p["D"],
                                          p["B_experts"][:, t], p["C_experts"][:, t],
                                          p["router_logits"][:, t], k)
        np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), idx_ref)
        l2, linf = rel_errors(host(out.y), y_ref, (0, 1))
        assert l2 <= tol and linf <= tol, (t, l2, linf)
        l2, linf = rel_errors(host(st_gpu), st_ref, (0, 1))
        assert l2 <= 1e-5 and linf <= 1e-5, (t, l2, linf)   # state arithmetic is fp32 on both types


def test_step_out_of_place_leaves_input_untouched():
    w = synth.Workload("dec", 2, 1, 2, 64, 128, 1, 4, 2, 0, "bf16", 9)
    p = synth.make_decode_inputs(w)
    d = to_device(p, "bf16")
    before = d["state"].clone()
    dst = torch.empty_like(before)
    args = (d["x"][:, 0].contiguous(), d["dt"][:, 0].contiguous(), d["A"], d["D"],
            d["B_experts"][:, 0].contiguous(), d["C_experts"][:, 0].contiguous(),
            d["router_logits"][:, 0].contiguous(), 2)
    o1 = sw.swimba_step(d["state"], *args, state_out=dst)
    torch.cuda.synchronize()
    assert torch.equal(d["state"], before)
    o2 = sw.swimba_step(d["state"], *args)
    torch.cuda.synchronize()
    assert torch.equal(d["state"], dst) and torch.equal(o1.y, o2.y)


def test_prefill_hands_its_state_to_decode():
    """Prefill of the first L tokens, then one swimba_step per further token from h_final,
    equals the oracle's forward over all tokens (state handed over in fp32)."""
    w = synth.Workload("handoff", 2, 140, 4, 64, 128, 2, 8, 2, 64, "bf16", 7)
    p = synth.make_inputs(w, seed=4242)
    L0 = 128
    ref = oracle_fwd(p, w.top_k)
    d = to_device(p, "bf16")
    pre = sw.swimba_mixer_fwd(d["x"][:, :L0].contiguous(), d["dt"][:, :L0].contiguous(), d["A"], d["D"],
                              d["B_experts"][:, :L0].contiguous(), d["C_experts"][:, :L0].contiguous(),
                              d["router_logits"][:, :L0].contiguous(), w.top_k, w.chunk)
    state = pre.h_final
    ys = []
    for t in range(L0, w.seqlen):
        out = sw.swimba_step(state, d["x"][:, t].contiguous(), d["dt"][:, t].contiguous(), d["A"], d["D"],
                             d["B_experts"][:, t].contiguous(), d["C_experts"][:, t].contiguous(),
                             d["router_logits"][:, t].contiguous(), w.top_k)
        ys.append(out.y)
    torch.cuda.synchronize()
    y = torch.cat([pre.y, torch.stack(ys, dim=1)], dim=1)
    l2, linf = rel_errors(host(y), ref["y"], (0, 2))
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)
    l2, linf = rel_errors(host(state), ref["h_final"], (0, 1))
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"], (l2, linf)


@pytest.mark.parametrize("cfg", [(3, 5, 4, 16, 16, 1, 4, 2, "f32"), (2, 7, 6, 24, 40, 3, 5, 5, "f32"),
                                 (2, 4, 4, 64, 128, 2, 8, 2, "bf16"), (2, 8, 2, 48, 128, 1, 8, 1, "f32"),
                                 (1, 1, 2, 64, 128, 1, 8, 2, "bf16")],
                         ids=lambda c: "B%dL%dH%dP%dN%dG%dE%dk%d%s" % c)
def test_step_multi_matches_oracle(cfg):
    """L decode tokens in one call == the oracle's forward over those L tokens from the same state."""
    B, L, H, P, N, G, E, k, io = cfg
    w = synth.Workload("multi", B, L, H, P, N, G, E, k, 0, io, 7)
    p = synth.make_decode_inputs(w, seed=hash(cfg[:8]) % 100000)
    d = to_device(p, io)
    state0 = d["state"].clone()
    out = sw.swimba_step_multi(d["state"], d["x"], d["dt"], d["A"], d["D"], d["B_experts"], d["C_experts"],
                               d["router_logits"], k, state_out=torch.empty_like(state0), want_topk=True)
    torch.cuda.synchronize()
    assert torch.equal(d["state"], state0)          # out of place: the input state is untouched
    ref = oracle_fwd(p, k, h0=p["state"].astype(np.float64))
    np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
    l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
    assert l2 <= TOL[io] and linf <= TOL[io], ("y", l2, linf)
    l2, linf = rel_errors(host(out.state), ref["h_final"], (0, 1))
    assert l2 <= 1e-5 and linf <= 1e-5, ("state", l2, linf)


def test_step_multi_chain_equals_single_steps():
    """64 tokens as 8 calls of 8 tokens, in place, against 64 single-token steps: same fp32
    recurrence, so the states agree to rounding."""
    w = synth.Workload("chain", 2, 64, 4, 64, 128, 1, 8, 2, 0, "bf16", 7)
    p = synth.make_decode_inputs(w, seed=77)
    d = to_device(p, "bf16")
    s_multi, s_single = d["state"].clone(), d["state"].clone()
    ys_m, ys_s = [], []
    for c in range(0, 64, 8):
        sl = slice(c, c + 8)
        ys_m.append(sw.swimba_step_multi(s_multi, d["x"][:, sl].contiguous(), d["dt"][:, sl].contiguous(), d["A"], d["D"],
                                         d["B_experts"][:, sl].contiguous(), d["C_experts"][:, sl].contiguous(),
                                         d["router_logits"][:, sl].contiguous(), w.top_k).y)
    for t in range(64):
        ys_s.append(sw.swimba_step(s_single, d["x"][:, t].contiguous(), d["dt"][:, t].contiguous(), d["A"], d["D"],
                                   d["B_experts"][:, t].contiguous(), d["C_experts"][:, t].contiguous(),
                                   d["router_logits"][:, t].contiguous(), w.top_k).y)
    torch.cuda.synchronize()
    l2, linf = rel_errors(host(s_multi), host(s_single), (0, 1))
    assert l2 <= 1e-6 and linf <= 1e-6, (l2, linf)
    # y is rounded to bf16 on both sides: at most an occasional one-ulp difference
    l2, linf = rel_errors(host(torch.cat(ys_m, dim=1)), host(torch.stack(ys_s, dim=1)), (0, 2))
    assert l2 <= 1e-3 and linf <= 4e-3, (l2, linf)
