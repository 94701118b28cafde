"""swimba_step_static (the decode step on the library's own scratch array, for callers that cannot
allocate) against swimba_step, through the C ABI: same kernels, so bitwise the same y, state and
active sets; two calls in a row on one GPU, the second with a smaller input, so that what the
first call left in the shared array cannot leak into the second."""
import ctypes

import numpy as np
import pytest
import torch

from paper_2603_06938_amd import binding as sw
from paper_2603_06938_amd import synth
from gpu_util import to_device

pytestmark = pytest.mark.gpu


def one_step(w, seed):
    p = synth.make_decode_inputs(w.with_(seqlen=1), seed=seed)
    p["D"] = np.linspace(-1, 1, w.nheads).astype(np.float32)
    d = to_device(p, w.io_dtype)
    args = (d["x"][:, 0].contiguous(), d["dt"][:, 0].contiguous(), d["A"], d["D"],
            d["B_experts"][:, 0].contiguous(), d["C_experts"][:, 0].contiguous(),
            d["router_logits"][:, 0].contiguous(), w.top_k)
    ref_state = torch.empty_like(d["state"])
    ref = sw.swimba_step(d["state"], *args, state_out=ref_state, want_topk=True)
    y = torch.full_like(ref.y, float("nan"))
    state = torch.full_like(d["state"], float("nan"))
    idx = torch.full_like(ref.topk_idx, -1)
    torch.cuda.synchronize()
    got = sw.swimba_step_static(d["state"], *args, y, state_out=state, topk_idx=idx)
    torch.cuda.synchronize()
    assert torch.equal(got.y, ref.y), "y differs"
    assert torch.equal(state, ref_state), "state differs"
    assert torch.equal(idx, ref.topk_idx), "active sets differ"


@pytest.mark.parametrize("io", ["bf16", "f32"])
def test_static_scratch_step_equals_workspace_step_twice(io):
    # first call: the larger input (8 groups: 64 KB of mixed rows); second: fewer sequences,
    # groups and a smaller state, so it only overwrites the front of what the first one left
    one_step(synth.Workload("dec", 8, 1, 16, 64, 128, 8, 8, 2, 0, io, 9), seed=11)
    one_step(synth.Workload("dec", 3, 1, 6, 24, 40, 3, 5, 5, 0, io, 9), seed=12)
    one_step(synth.Workload("dec", 2, 1, 4, 64, 128, 1, 4, 1, 0, io, 9), seed=13)


def test_static_scratch_limit_is_refused_on_the_host():
    lib = sw._load()
    p = [0x10000 * (i + 1) for i in range(11)]
    # B*G*N*8 bytes = 1 MiB is the largest step that fits
    ok = sw.make_dims(64, 1, 64, 64, 256, 8, 8, 2, 0, torch.bfloat16)
    assert sw.swimba_step_workspace_bytes(ok) == 1 << 20
    big = sw.make_dims(65, 1, 64, 64, 256, 8, 8, 2, 0, torch.bfloat16)
    assert lib.swimba_step_static(ctypes.byref(big), *p, None) == 4
    assert lib.swimba_step_static(ctypes.byref(sw.make_dims(2, 3, 4, 64, 128, 1, 8, 2, 0, torch.bfloat16)), *p, None) == 2
    assert lib.swimba_step_static(ctypes.byref(ok), None, *p[1:], None) == 1
    assert lib.swimba_step_static(ctypes.byref(ok), p[0] + 4, *p[1:], None) == 7
