"""Seeded synthetic inputs for the Swimba token-mixer workloads.

This module only draws random tensors and rounds them to the storage type.
It holds none of the method's arithmetic (no router, no mixing, no
recurrence) and imports neither the HIP binding nor the CPU oracle, so both
sides can be fed the same stored values.

Every tensor is returned as a float32 numpy array whose values are exactly
representable in the workload's I/O type (fp32 or bf16), i.e. they are "the
stored values": the GPU side converts them to its storage type without any
further rounding, the oracle upcasts them to double without any rounding.

Value distributions (one recipe for all workloads):
  x            ~ N(0, 1)                              (B, L, H, P)
  dt           = softplus(z + b_h), z ~ N(0, 1),      (B, L, H)
                 b_h = softplus^-1(dt0_h), dt0_h log-uniform in [1e-3, 1e-1]
  A_h          = -exp(U[0, ln 16])  in [-16, -1]      (H)    fp32
  D_h          = 1                                    (H)    fp32
  B_e, C_e     ~ N(0, 1/N) per token, expert, group   (B, L, E, G, N)
  logits       ~ N(0, 1)                              (B, L, E)
  state (decode workload only) ~ N(0, 0.1^2)          (B, H, P, N) fp32
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Dict

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    batch: int
    seqlen: int
    nheads: int
    headdim: int
    dstate: int
    ngroups: int
    nexperts: int
    top_k: int
    chunk: int
    io_dtype: str  # "f32" or "bf16"
    index: int = 0  # position in the workload list; part of the seed

    @property
    def tokens(self) -> int:
        return self.batch * self.seqlen

    def with_(self, **kw) -> "Workload":
        return replace(self, **kw)


# The five workloads the benchmark and the parity tests are quoted on.
WORKLOADS = (
    Workload("tiny_f32", 1, 256, 4, 16, 16, 1, 4, 2, 64, "f32", 0),
    Workload("mamba2_130m_layer", 8, 2048, 24, 64, 128, 1, 8, 2, 256, "bf16", 1),
    Workload("mamba2_370m_layer", 8, 4096, 32, 64, 128, 1, 8, 2, 256, "bf16", 2),
    Workload("long_seq_g8_e16", 2, 16384, 64, 64, 128, 8, 16, 2, 256, "bf16", 3),
    # decode: seqlen is the number of consecutive single-token steps
    Workload("decode_step", 64, 1024, 64, 64, 128, 1, 8, 2, 0, "bf16", 4),
)

SEED_BASE = 69380


def workload(i_or_name) -> Workload:
    for w in WORKLOADS:
        if w.index == i_or_name or w.name == i_or_name:
            return w
    raise KeyError(i_or_name)


def round_to_bf16(a: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16 (ties to even), return as float32."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    bits = a.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    out = rounded.view(np.float32)
    # keep non-finite values as they are (the carry trick is for finite numbers)
    return np.where(np.isfinite(a), out, a).astype(np.float32)


def to_storage(a: np.ndarray, io_dtype: str) -> np.ndarray:
    if io_dtype == "bf16":
        return round_to_bf16(a)
    if io_dtype == "f32":
        return np.ascontiguousarray(a, dtype=np.float32)
    raise ValueError(io_dtype)


def _softplus(v: np.ndarray) -> np.ndarray:
    return np.logaddexp(v, 0.0)


def make_inputs(w: Workload, seed: int | None = None, d_skip: float = 1.0) -> Dict[str, np.ndarray]:
    """Draw the tensors of a prefill workload in a fixed order.

    Returns x, dt, A, D, B_experts, C_experts, router_logits (float32 arrays
    holding storage-exact values).
    """
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + w.index if seed is None else seed))
    B, L, H, P, N, G, E = w.batch, w.seqlen, w.nheads, w.headdim, w.dstate, w.ngroups, w.nexperts
    f32 = np.float32
    x = rng.standard_normal((B, L, H, P), dtype=f32)
    dt0 = np.exp(rng.uniform(np.log(1e-3), np.log(1e-1), size=H))
    bias = np.log(np.expm1(dt0))
    z = rng.standard_normal((B, L, H), dtype=f32)
    dt = _softplus(z.astype(np.float64) + bias[None, None, :]).astype(f32)
    A = (-np.exp(rng.uniform(0.0, np.log(16.0), size=H))).astype(f32)
    D = np.full(H, d_skip, dtype=f32)
    scale = f32(1.0 / np.sqrt(N))
    Be = rng.standard_normal((B, L, E, G, N), dtype=f32)
    Be *= scale
    Ce = rng.standard_normal((B, L, E, G, N), dtype=f32)
    Ce *= scale
    logits = rng.standard_normal((B, L, E), dtype=f32)
    io = w.io_dtype
    dt_s = to_storage(dt, io)
    # a stored dt must stay strictly positive (bf16 rounding never produces 0 here)
    assert (dt_s > 0).all()
    return {
        "x": to_storage(x, io),
        "dt": dt_s,
        "A": A,
        "D": D,
        "B_experts": to_storage(Be, io),
        "C_experts": to_storage(Ce, io),
        "router_logits": to_storage(logits, io),
    }


def make_decode_inputs(w: Workload, steps: int | None = None, seed: int | None = None,
                       d_skip: float = 1.0) -> Dict[str, np.ndarray]:
    """Decode workload: an initial fp32 state and `steps` consecutive tokens.

    Per-step tensors carry the step as their second axis, so they are drawn
    exactly like a prefill workload of seqlen == steps:
      x (B, S, H, P), dt (B, S, H), B/C_experts (B, S, E, G, N), logits (B, S, E).
    """
    steps = w.seqlen if steps is None else steps
    d = make_inputs(w.with_(seqlen=steps), seed=seed, d_skip=d_skip)
    rng = np.random.Generator(np.random.PCG64((SEED_BASE + w.index if seed is None else seed) + 1_000_003))
    d["state"] = (0.1 * rng.standard_normal((w.batch, w.nheads, w.headdim, w.dstate), dtype=np.float32))
    return d
