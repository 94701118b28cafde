"""The entry points only enqueue kernels (and device-to-device copies) on the caller's
stream, allocate nothing and never synchronise, so a serving loop can capture them in a HIP
graph.  Replays are checked against the eager results, with eager work between replays."""
import numpy as np
import pytest
import torch

from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def test_forward_and_decode_steps_replay_from_a_graph():
    w = synth.Workload("graph", 2, 300, 4, 64, 128, 2, 8, 2, 128, "bf16", 7)
    p = synth.make_inputs(w, seed=31)
    d = to_device(p, "bf16")
    dims = sw.dims_of(d["x"], d["B_experts"], w.top_k, w.chunk)
    ws = torch.empty(sw.swimba_mixer_workspace_bytes(dims), dtype=torch.uint8, device="cuda:0")
    y = torch.empty_like(d["x"])
    hf = torch.empty((w.batch, w.nheads, w.headdim, w.dstate), dtype=torch.float32, device="cuda:0")
    state = torch.empty_like(hf)
    nsteps = 4
    ys = torch.empty((nsteps,) + tuple(d["x"][:, 0].shape), dtype=d["x"].dtype, device="cuda:0")
    xs = [d["x"][:, t].contiguous() for t in range(nsteps)]
    dts = [d["dt"][:, t].contiguous() for t in range(nsteps)]
    Bs = [d["B_experts"][:, t].contiguous() for t in range(nsteps)]
    Cs = [d["C_experts"][:, t].contiguous() for t in range(nsteps)]
    gs = [d["router_logits"][:, t].contiguous() for t in range(nsteps)]
    sdims = sw.make_dims(w.batch, 1, w.nheads, w.headdim, w.dstate, w.ngroups, w.nexperts, w.top_k, 0, torch.bfloat16)
    sws = torch.empty(sw.swimba_step_workspace_bytes(sdims), dtype=torch.uint8, device="cuda:0")

    def work():
        # prefill, then a few decode steps from its final state (copied, so a replay starts afresh)
        sw.swimba_mixer_fwd(d["x"], d["dt"], d["A"], d["D"], d["B_experts"], d["C_experts"], d["router_logits"],
                            w.top_k, w.chunk, None, y=y, h_final=hf, workspace=ws)
        state.copy_(hf)
        for t in range(nsteps):
            sw.swimba_step(state, xs[t], dts[t], d["A"], d["D"], Bs[t], Cs[t], gs[t], w.top_k, y=ys[t], workspace=sws)

    work()                                   # eager reference (also the warm-up before capture)
    torch.cuda.synchronize()
    y_ref, ys_ref, state_ref = y.clone(), ys.clone(), state.clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            work()
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(3):
        y.zero_(); ys.zero_(); state.zero_()
        # unrelated eager work between replays
        junk = torch.randn(1 << 16, device="cuda:0").sum().item()
        assert np.isfinite(junk)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, y_ref), rep
        assert torch.equal(ys, ys_ref), rep
        assert torch.equal(state, state_ref), rep
