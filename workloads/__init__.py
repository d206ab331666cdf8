"""Seeded synthetic attention inputs shared by the CPU oracle's tests and the GPU path.

This module holds input recipes only: shapes, lengths, value distributions and
rounding of the drawn values to the storage type.  None of the attention
arithmetic lives here.  The five named workloads stand in for per-layer Q/K/V
activations of a 12-head, head_dim-64 ModernBERT-style classifier at 512 to
32K tokens (paper Sec. 2.4 / Sec. 4.1.3: alternating 128-token local layers
and global layers; Table "SDPA vs FA" sequence lengths); the model weights and
the paper's payloads are not available, so values are i.i.d. normal.

Every array is returned as float32 holding values that are exactly
representable in the storage type (fp16 or bf16), so the oracle (which widens
to fp64) and the GPU path (which narrows to the storage type) see identical
numbers.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

__all__ = ["Workload", "CONFIGS", "NEXT_CONFIGS", "ALL_CONFIGS", "round_to_storage", "draw", "make_inputs"]


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """Round float32 values to the nearest fp16 / bf16 value (ties to even) and
    return them as float32."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "fp16":
        return x.astype(np.float16).astype(np.float32)
    if dtype == "bf16":
        u = x.view(np.uint32)
        bias = np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
        r = (u + bias) & np.uint32(0xFFFF0000)
        return r.view(np.float32)
    raise ValueError(f"unknown storage dtype {dtype!r}")


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    dtype: str                 # "fp16" | "bf16"
    batch: int
    heads: int
    max_len: int
    head_dim: int
    scale: float
    window: int                # < 0 global, W >= 1 local band of W keys
    seq_lens: tuple | None     # fixed lengths, or None
    random_lens: tuple | None = None   # (lo, hi) inclusive, drawn before Q
    qk_gain: float = 1.0       # Q and K are gain * N(0,1)
    note: str = ""
    extra: dict = field(default_factory=dict)


CONFIGS = {
    # single call, 512 tokens, no padding
    "c1_512": Workload("c1_512", 0, "fp16", 1, 12, 512, 64, 0.125, -1, None),
    # post-compression short-sequence batch, lengths uniform on [256, 512]
    "c2_batch32": Workload("c2_batch32", 1, "fp16", 32, 12, 512, 64, 0.125, -1, None,
                           random_lens=(256, 512)),
    # 8K global layer, valid length 7900, peaked softmax
    "c3_8k": Workload("c3_8k", 2, "fp16", 1, 12, 8192, 64, 0.125, -1, (7900,), qk_gain=1.5),
    # three concurrent classifiers at 16K
    "c4_16k_x3": Workload("c4_16k_x3", 3, "bf16", 3, 12, 16384, 64, 0.125, -1,
                          (16384, 12000, 9000)),
    # 32K global / 32K local band of 128 keys (63 left, 64 right)
    "c5a_32k_global": Workload("c5a_32k_global", 4, "bf16", 1, 12, 32768, 64, 0.125, -1, None),
    "c5b_32k_local": Workload("c5b_32k_local", 4, "bf16", 1, 12, 32768, 64, 0.125, 128, None),
}


def draw(seed, batch, heads, max_len, head_dim, dtype, qk_gain=1.0, random_lens=None):
    """Draw (seq_lens or None, q, k, v) in that fixed order from PCG64(seed).

    Padded positions are filled with the same random values as valid ones, so a
    masking mistake shows up in the output.
    """
    rng = np.random.Generator(np.random.PCG64(seed))
    lens = None
    if random_lens is not None:
        lo, hi = random_lens
        lens = rng.integers(lo, hi + 1, size=batch).astype(np.int32)
    shape = (batch, heads, max_len, head_dim)
    q = rng.standard_normal(shape, dtype=np.float32)
    k = rng.standard_normal(shape, dtype=np.float32)
    v = rng.standard_normal(shape, dtype=np.float32)
    if qk_gain != 1.0:
        q *= np.float32(qk_gain)
        k *= np.float32(qk_gain)
    return lens, round_to_storage(q, dtype), round_to_storage(k, dtype), round_to_storage(v, dtype)

# Workloads for the operator's other head sizes (paper Sec. 4.1.3: run-time dispatch on
# head_dim 32 / 64 / 128).  Not among the five above: 8 heads of 128 (hidden size 1024),
# scale 1/sqrt(128), and 24 heads of 32, otherwise the recipe of the 8K and 32K workloads.
NEXT_CONFIGS = {
    "d128_8k": Workload("d128_8k", 5, "fp16", 1, 8, 8192, 128, 128 ** -0.5, -1, (7900,), qk_gain=1.5),
    "d128_32k": Workload("d128_32k", 6, "bf16", 1, 8, 32768, 128, 128 ** -0.5, -1, None),
    "d128_32k_local": Workload("d128_32k_local", 6, "bf16", 1, 8, 32768, 128, 128 ** -0.5, 128, None),
    # 24 heads of 32 (hidden size 768, as the five main workloads), scale 1/sqrt(32)
    "d32_8k": Workload("d32_8k", 7, "fp16", 1, 24, 8192, 32, 32 ** -0.5, -1, (7900,), qk_gain=1.5),
    "d32_32k": Workload("d32_32k", 8, "bf16", 1, 24, 32768, 32, 32 ** -0.5, -1, None),
    "d32_32k_local": Workload("d32_32k_local", 8, "bf16", 1, 24, 32768, 32, 32 ** -0.5, 128, None),
}
ALL_CONFIGS = {**CONFIGS, **NEXT_CONFIGS}


def make_inputs(w: Workload):
    """Returns (seq_lens int32[B], q, k, v) for a named workload."""
    lens, q, k, v = draw(w.seed, w.batch, w.heads, w.max_len, w.head_dim, w.dtype,
                         w.qk_gain, w.random_lens)
    if lens is None:
        if w.seq_lens is not None:
            lens = np.asarray(w.seq_lens, dtype=np.int32)
        else:
            lens = np.full((w.batch,), w.max_len, dtype=np.int32)
    return lens, q, k, v
