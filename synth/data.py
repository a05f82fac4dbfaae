"""Seeded prompts, uniforms and layer-microbenchmark inputs (input data only)."""
from __future__ import annotations

from typing import List, Tuple

import numpy as np

from .shapes import ModelShape
from .weights import fill_normal


def make_prompts(batch: int, len_range: Tuple[int, int], vocab: int, seed: int = 0) -> List[np.ndarray]:
    """``batch`` prompts of uniform-random token ids; lengths uniform in the inclusive range.

    Fixed 512-token prompts stand in for the mean prompt length of the paper's
    summarisation workload and U[256,1024] spans the mean-to-maximum range of its four
    datasets (Table 2); the datasets themselves are not used.
    """
    rng = np.random.default_rng([seed, 0x5EED])
    lo, hi = len_range
    lens = rng.integers(lo, hi + 1, size=batch) if hi > lo else np.full(batch, lo)
    return [rng.integers(0, vocab, size=int(n), dtype=np.int64).astype(np.int32) for n in lens]


def make_uniforms(shape, seed: int = 0) -> np.ndarray:
    """float32 uniforms in [0,1) on the 2^-24 grid: (uint32 >> 8) * 2^-24."""
    rng = np.random.default_rng([seed, 0xA11CE])
    bits = rng.integers(0, 1 << 32, size=shape, dtype=np.uint64).astype(np.uint32)
    return ((bits >> 8).astype(np.float32) * np.float32(2.0 ** -24)).astype(np.float32)


def make_layer_inputs(shape: ModelShape, batch: int, n_new: int, ctx: int, seed: int = 0):
    """Inputs of the one-layer verify microbenchmark.

    Returns (x, k_ctx, v_ctx): activations ``x`` [batch*n_new, d] ~ N(0,1) and an existing
    KV context ``k_ctx``/``v_ctx`` [batch, Hkv, ctx, dh] ~ N(0,1) (keys taken as already
    rotated), all in the model's storage type (uint16 bf16 bit patterns or float32).
    """
    dt = np.uint16 if shape.dtype == "bf16" else np.float32
    x = np.empty((batch * n_new, shape.d_model), dtype=dt)
    kc = np.empty((batch, shape.n_kv_heads, ctx, shape.head_dim), dtype=dt)
    vc = np.empty_like(kc)
    fill_normal(x.reshape(-1), seed, 900001, std=1.0)
    fill_normal(kc.reshape(-1), seed, 900002, std=1.0)
    fill_normal(vc.reshape(-1), seed, 900003, std=1.0)
    return x, kc, vc
