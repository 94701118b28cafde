"""GPU parity at the full benchmark sizes, in the launch configuration bench.py
times.  The oracle is fast enough (a few seconds per workload on the host
cores) to check every output element, not a sample."""
import numpy as np
import pytest
import torch

from oracle import swimba_oracle as orc
from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import TOL, abs_inputs, comp_tol, componentwise_excess, host, rel_errors, run_mixer, to_device

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("wi", [1, 2, 3])
def test_prefill_workload_full_size(wi):
    w = synth.workload(wi)
    print("workload", w, flush=True)
    p = synth.make_inputs(w)
    tol = TOL[w.io_dtype]
    # the sums of absolute values behind every output element (the componentwise bound's scale)
    q = abs_inputs(p)
    aref = orc.mixer_fwd(q["x"], q["dt"], q["A"], None, q["B_experts"], q["C_experts"], q["router_logits"], w.top_k)
    for d_none in (True, False):
        out = run_mixer(p, w.top_k, w.chunk, w.io_dtype, d_none=d_none)
        ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], None if d_none else p["D"], p["B_experts"],
                            p["C_experts"], p["router_logits"], w.top_k)
        np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
        np.testing.assert_allclose(host(out.topk_w), ref["topk_w"], rtol=1e-5, atol=1e-30)
        l2, linf = rel_errors(host(out.y), ref["y"], (0, 2))
        print("D=%s  y rel l2 %.3e linf %.3e" % ("0" if d_none else "1", l2, linf), flush=True)
        assert l2 <= tol and linf <= tol, (d_none, l2, linf)
        l2, linf = rel_errors(host(out.h_final), ref["h_final"], (0, 1))
        print("      h_final rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
        assert l2 <= tol and linf <= tol, (l2, linf)
        ay = aref["y"] if d_none else aref["y"] + np.abs(p["D"])[None, None, :, None] * q["x"]
        ey = componentwise_excess(host(out.y), ref["y"], ay)
        eh = componentwise_excess(host(out.h_final), ref["h_final"], aref["h_final"])
        print("      componentwise: y %.3e h_final %.3e (bound %.3e)" % (ey, eh, comp_tol(w.io_dtype)), flush=True)
        assert ey <= comp_tol(w.io_dtype) and eh <= comp_tol(w.io_dtype), (d_none, ey, eh)
        del out, ref, ay


@pytest.mark.parametrize("G", [1, 8])
def test_decode_1024_steps(G):
    w = synth.workload(4).with_(ngroups=G)
    steps = w.seqlen
    p = synth.make_decode_inputs(w)
    d = to_device(p, w.io_dtype)
    # per-step tensors, step-major on the device
    xs = d["x"].transpose(0, 1).contiguous()
    dts = d["dt"].transpose(0, 1).contiguous()
    Bs = d["B_experts"].transpose(0, 1).contiguous()
    Cs = d["C_experts"].transpose(0, 1).contiguous()
    gs = d["router_logits"].transpose(0, 1).contiguous()
    state = d["state"].clone()
    ys = torch.empty_like(xs)
    idx = torch.empty((steps, w.batch, w.top_k), dtype=torch.int32, device="cuda:0")
    ws = torch.empty(sw.swimba_step_workspace_bytes(
        sw.make_dims(w.batch, 1, w.nheads, w.headdim, w.dstate, w.ngroups, w.nexperts, w.top_k, 0, torch.bfloat16)),
        dtype=torch.uint8, device="cuda:0")
    for t in range(steps):
        sw.swimba_step(state, xs[t], dts[t], d["A"], d["D"], Bs[t], Cs[t], gs[t], w.top_k,
                       y=ys[t], topk_idx=idx[t], workspace=ws)
    torch.cuda.synchronize()
    # 1024 steps of the recurrence == the sequential forward from the same initial state
    ref = orc.mixer_fwd(p["x"], p["dt"], p["A"], p["D"], p["B_experts"], p["C_experts"],
                        p["router_logits"], w.top_k, h0=p["state"].astype(np.float64))
    np.testing.assert_array_equal(idx.cpu().numpy().transpose(1, 0, 2), ref["topk_idx"])
    l2, linf = rel_errors(host(state), ref["h_final"], (0, 1))
    print("final state rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
    assert l2 <= 1e-4 and linf <= 1e-4
    assert torch.isfinite(state).all()
    l2, linf = rel_errors(host(ys).transpose(1, 0, 2, 3), ref["y"], (0, 2))
    print("y rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
    assert l2 <= TOL["bf16"] and linf <= TOL["bf16"]


def test_expert_proj_workload1_size():
    """Routed in-projection at the token count of workload 1 from 768 features (the width of
    the 130M model): every written row against the oracle."""
    w = synth.workload(1)
    B, L, E, G, N, k, Dm = w.batch, w.seqlen, w.nexperts, w.ngroups, w.dstate, w.top_k, 768
    rng = np.random.default_rng(69380 + 201)
    u = synth.round_to_bf16(rng.standard_normal((B, L, Dm)).astype(np.float32))
    WB = synth.round_to_bf16((rng.standard_normal((E, G, N, Dm)) / np.sqrt(Dm)).astype(np.float32))
    WC = synth.round_to_bf16((rng.standard_normal((E, G, N, Dm)) / np.sqrt(Dm)).astype(np.float32))
    g = synth.make_inputs(w)["router_logits"]
    bf = lambda a: torch.from_numpy(a).to(torch.bfloat16).to("cuda:0")
    out = sw.swimba_expert_proj(bf(u), bf(WB), bf(WC), bf(g), k, want_topk=True)
    torch.cuda.synchronize()
    ref = orc.expert_proj(u, WB, WC, g, k, fill=0.0)
    np.testing.assert_array_equal(out.topk_idx.cpu().numpy(), ref["topk_idx"])
    for name, got, want in (("B", host(out.B_experts), ref["B_experts"]), ("C", host(out.C_experts), ref["C_experts"])):
        l2 = np.linalg.norm(got - want) / np.linalg.norm(want)
        linf = np.abs(got - want).max() / np.abs(want).max()
        print(name, "rel l2 %.3e linf %.3e" % (l2, linf), flush=True)
        assert l2 <= TOL["bf16"] and linf <= TOL["bf16"]
