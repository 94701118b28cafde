"""Helpers of the GPU parity tests: move stored values to the device, run the
HIP path through the binding, and measure the error against the oracle."""
import numpy as np
import torch

from paper_2603_06938_amd import binding as sw

IO = {"f32": torch.float32, "bf16": torch.bfloat16}
# relative-error bars: fp32 path 1e-4; bf16 I/O with fp32 accumulation 2e-2
TOL = {"f32": 1e-4, "bf16": 2e-2}
IO_NAMES = ("x", "dt", "B_experts", "C_experts", "router_logits")


def to_device(p, io_dtype, dev="cuda:0"):
    out = {}
    for k, v in p.items():
        if v is None:
            out[k] = None
            continue
        t = torch.from_numpy(np.ascontiguousarray(v))
        if k in IO_NAMES:
            t = t.to(IO[io_dtype])          # exact: the stored values are representable
        out[k] = t.to(dev)
    return out


def host(t):
    return t.detach().to("cpu").to(torch.float64).numpy()


def rel_errors(got, ref, slice_axes):
    """(max over slices of ||got-ref||_2/||ref||_2, global ||.||_inf ratio).
    slice_axes: the axes that index a slice (e.g. batch and head)."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    red = tuple(a for a in range(ref.ndim) if a not in slice_axes)
    num = np.sqrt(((got - ref) ** 2).sum(axis=red))
    den = np.sqrt((ref ** 2).sum(axis=red))
    l2 = float((num / np.maximum(den, 1e-300)).max()) if num.size else 0.0
    linf = float(np.abs(got - ref).max() / max(np.abs(ref).max(), 1e-300)) if ref.size else 0.0
    return l2, linf


def run_mixer(p, top_k, chunk, io_dtype, h0=None, d_none=False, want_topk=True):
    d = to_device(p, io_dtype)
    h0d = None if h0 is None else torch.from_numpy(np.asarray(h0, dtype=np.float32)).to("cuda:0")
    out = sw.swimba_mixer_fwd(d["x"], d["dt"], d["A"], None if d_none else d["D"], d["B_experts"],
                              d["C_experts"], d["router_logits"], top_k, chunk, h0d, want_topk=want_topk)
    torch.cuda.synchronize()
    return out
