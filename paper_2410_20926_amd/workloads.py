"""Seeded synthetic workloads for tensorized attention.

Holds the shapes of the benchmark configurations and the random-input recipe,
and nothing of the method's arithmetic: it is the one module that both the
GPU path's callers and the CPU oracle's callers may use.  It imports neither.

Recipe: NumPy `default_rng(seed)` (PCG64), `standard_normal` in float32, drawn
in the order Q, K, V, dO, each as a dense C-ordered [B, N, H, D] array, then
scaled, then (for bf16 workloads) rounded to the nearest bf16 value, ties to
even, and kept as float32 holding exactly representable numbers, so that the
GPU path and the oracle consume identical inputs.

The shapes stand in for the paper's language-model workloads: Llama-3-8B
attention geometry (32 query / 8 key-value heads, head width 128), training
context 32,768 as {32,32,32} (Sec. 4.1) and inference at 128k (Table 3).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np

BASE_SEED = 241020926


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                  # 1-based configuration number
    dtype: str                  # "f32" or "bf16"
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    dims: Tuple[int, ...]
    causal: bool
    qk_prescale: float          # Q and K are N(0,1) times this
    backward: bool = False
    rope_base: Optional[float] = None   # the per-axis rotary encoding inside the hops (Sec. 3.2), or None

    @property
    def seq_len(self) -> int:
        return int(np.prod(self.dims))

    @property
    def seed(self) -> int:
        return BASE_SEED + self.index


WORKLOADS = {
    "c1": Workload("c1", 1, "f32", 1, 1, 1, 64, (16, 16), False, 1.0),
    "c2": Workload("c2", 2, "bf16", 1, 32, 32, 128, (32, 16, 16), True, 1.0 / math.sqrt(128)),
    "c3": Workload("c3", 3, "bf16", 1, 32, 8, 128, (32, 32, 32), True, 1.0 / math.sqrt(128)),
    "c4": Workload("c4", 4, "bf16", 1, 32, 8, 128, (64, 64, 32), True, 1.0 / math.sqrt(128)),
    "c5": Workload("c5", 5, "bf16", 2, 32, 8, 128, (32, 32, 32), True, 1.0 / math.sqrt(128),
                   backward=True),
    # not one of the five benchmark configurations: the paper's own route to 128k tokens, the
    # first axis of a {32,32,32} model lengthened to 128 (Sec. 4.3)
    "c6": Workload("c6", 6, "bf16", 1, 32, 8, 128, (128, 32, 32), True, 1.0 / math.sqrt(128)),
    # config 3 with the tensorized positional encoding applied inside every hop (Sec. 3.2)
    "c3_rope": Workload("c3_rope", 3, "bf16", 1, 32, 8, 128, (32, 32, 32), True, 1.0 / math.sqrt(128), rope_base=10000.0),
    # config 4's shape as a training step (forward + backward): axes of 64 positions in the backward
    "c4_train": Workload("c4_train", 4, "bf16", 1, 32, 8, 128, (64, 64, 32), True, 1.0 / math.sqrt(128), backward=True),
    # the attention geometry of the smallest of the paper's three backbones (Sec. 4.1): 32 heads of width 100, no grouping,
    # as a training step on config 3's shape; rows of 200 bytes, neither 16-byte aligned nor whole cache lines
    "c3_w100_train": Workload("c3_w100_train", 3, "bf16", 1, 32, 32, 100, (32, 32, 32), True, 0.1, backward=True),
}


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bfloat16 (ties to even); the result
    is float32 whose low 16 mantissa bits are zero."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    bits = x.view(np.uint32)
    lsb = (bits >> np.uint32(16)) & np.uint32(1)
    rounded = (bits + np.uint32(0x7FFF) + lsb) & np.uint32(0xFFFF0000)
    return rounded.view(np.float32)


def bf16_bits(x: np.ndarray) -> np.ndarray:
    """Upper 16 bits (as int16) of float32 values that are already exactly
    representable in bf16; the raw storage a bf16 device buffer holds."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    return (x.view(np.uint32) >> np.uint32(16)).astype(np.uint16).view(np.int16)


def bf16_bits_to_f32(bits: np.ndarray) -> np.ndarray:
    """Inverse of `bf16_bits`."""
    u = np.ascontiguousarray(bits).view(np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32)


def draw(shape, rng: np.random.Generator, scale: float, dtype: str) -> np.ndarray:
    x = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        x *= np.float32(scale)
    if dtype == "bf16":
        x = round_to_bf16(x)
    return x


def make_inputs(batch: int, seq_len: int, n_q_heads: int, n_kv_heads: int, head_dim: int,
                seed: int, dtype: str = "f32", qk_scale: float = 1.0,
                with_grad: bool = False):
    """Q [B,N,Hq,D], K, V [B,N,Hkv,D] (and dO [B,N,Hq,D] when `with_grad`),
    float32 arrays (bf16-representable when dtype == "bf16")."""
    rng = np.random.default_rng(seed)
    q = draw((batch, seq_len, n_q_heads, head_dim), rng, qk_scale, dtype)
    k = draw((batch, seq_len, n_kv_heads, head_dim), rng, qk_scale, dtype)
    v = draw((batch, seq_len, n_kv_heads, head_dim), rng, 1.0, dtype)
    if with_grad:
        d_o = draw((batch, seq_len, n_q_heads, head_dim), rng, 1.0, dtype)
        return q, k, v, d_o
    return q, k, v


def make_workload_inputs(w: Workload, with_grad: Optional[bool] = None):
    if with_grad is None:
        with_grad = w.backward
    return make_inputs(w.batch, w.seq_len, w.n_q_heads, w.n_kv_heads, w.head_dim,
                       w.seed, w.dtype, w.qk_prescale, with_grad)
