"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module only draws random numbers and names workload shapes.  It contains
none of the method's arithmetic (no packing, no dequantisation, no products)
and imports neither the oracle nor the HIP library, so both sides can be fed
the very same arrays.

The arrays stand in for real quantised Llama layers (weights and calibration
data are not available offline): bit-planes are i.i.d. fair bits stored to
p_max planes; every precision p has its own independently drawn scale set with
alpha_1 = |N(0, 0.02)| and alpha_{i+1} = alpha_i * U(0.4, 0.6) per (row, group);
activations are N(0, 1).  Scales and activations are rounded to float16 once,
here, so every consumer sees identical bits.  Layer shapes follow the
GEMV-latency table of the paper (Llama-3-8B, Phi-4-14B, Llama-3-70B).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

BASE_SEED = 251010467
P_MAX = 4
GROUP = 128

# (name, m = output rows, n = input columns)
LLAMA3_8B_LAYERS = [
    ("q_proj", 4096, 4096),
    ("k_proj", 1024, 4096),
    ("v_proj", 1024, 4096),
    ("o_proj", 4096, 4096),
    ("gate_proj", 14336, 4096),
    ("up_proj", 14336, 4096),
    ("down_proj", 4096, 14336),
]
PHI4_14B_SHAPES = [("attn", 5120, 5120), ("up", 17920, 5120), ("down", 5120, 17920)]
LLAMA3_70B_SHAPES = [("attn", 8192, 8192), ("up", 28672, 8192), ("down", 8192, 28672)]


@dataclass
class BcqLayer:
    """One synthetic quantised linear layer."""
    m: int
    n: int
    group: int
    planes: np.ndarray            # uint32 [p_max][m][n/32]
    scales: dict                  # p -> float16 [p][m][n/group]


def _rng(*key: int) -> np.random.Generator:
    return np.random.default_rng([BASE_SEED, *[int(k) for k in key]])


def make_planes(m: int, n: int, p_max: int = P_MAX, seed=(0, 0)) -> np.ndarray:
    """uint32 [p_max][m][n/32] of i.i.d. fair bits."""
    assert n % 32 == 0
    rng = _rng(1, *seed)
    return rng.integers(0, 2 ** 32, size=(p_max, m, n // 32), dtype=np.uint32)


def make_scales(p: int, m: int, n: int, group: int = GROUP, seed=(0, 0), signed: bool = False) -> np.ndarray:
    """float16 [p][m][n/group]; an independent draw for every p."""
    assert n % group == 0
    rng = _rng(2, p, *seed)
    g = n // group
    out = np.empty((p, m, g), dtype=np.float32)
    a = np.abs(rng.normal(0.0, 0.02, size=(m, g))).astype(np.float32)
    out[0] = a
    for i in range(1, p):
        a = a * rng.uniform(0.4, 0.6, size=(m, g)).astype(np.float32)
        out[i] = a
    if signed:
        out *= rng.choice(np.array([-1.0, 1.0], dtype=np.float32), size=out.shape)
    return out.astype(np.float16)


def make_offsets(p: int, m: int, n: int, group: int = GROUP, seed=(0, 0)) -> np.ndarray:
    """float16 [m][n/group]: offsets of the asymmetric scheme for precision p, N(0, 0.01^2) per
    (row, group), an independent draw for every p (half the spread of the first scale)."""
    assert n % group == 0
    rng = _rng(6, p, *seed)
    return rng.normal(0.0, 0.01, size=(m, n // group)).astype(np.float16)


def make_weights(m: int, n: int, seed=(0, 0), heavy_tail: bool = True) -> np.ndarray:
    """float16 [m][n]: full-precision weights for the quantiser, standing in for trained layers.

    Per output row a spread sigma_r = 0.02 * exp(N(0, 0.25^2)); entries sigma_r * N(0, 1); with
    ``heavy_tail`` one entry in 256 is multiplied by 6 (trained layers have a few large weights per
    group).  Rounded to float16 once, here.
    """
    rng = _rng(7, *seed)
    sigma = 0.02 * np.exp(rng.normal(0.0, 0.25, size=(m, 1)))
    w = rng.standard_normal(size=(m, n)) * sigma
    if heavy_tail:
        w = np.where(rng.random(size=(m, n)) < 1.0 / 256.0, 6.0 * w, w)
    return w.astype(np.float16)


def make_x(batch: int, n: int, seed=(0, 0), scale: float = 1.0) -> np.ndarray:
    """float16 [batch][n] ~ N(0, scale^2)."""
    rng = _rng(3, *seed)
    return (rng.normal(0.0, 1.0, size=(batch, n)) * scale).astype(np.float16)


def make_layer(m: int, n: int, p_max: int = P_MAX, group: int = GROUP, seed=(0, 0),
               precisions=None, signed: bool = False) -> BcqLayer:
    """Planes to p_max plus one scale set for each requested precision."""
    precisions = range(1, p_max + 1) if precisions is None else precisions
    planes = make_planes(m, n, p_max, seed)
    scales = {p: make_scales(p, m, n, group, seed, signed) for p in precisions}
    return BcqLayer(m=m, n=n, group=group, planes=planes, scales=scales)


def make_p_req(batch: int, lo: int = 2, hi: int = 4, seed=(0, 0)) -> np.ndarray:
    """int32 [batch], each request's precision drawn uniformly from lo..hi."""
    rng = _rng(4, *seed)
    return rng.integers(lo, hi + 1, size=batch, dtype=np.int32)


def make_codes(p_max: int, m: int, n: int, seed=(0, 0)) -> np.ndarray:
    """int8 [p_max][m][n] in {-1,+1}: unpacked codes for the packing tests."""
    rng = _rng(5, *seed)
    return (rng.integers(0, 2, size=(p_max, m, n), dtype=np.int8) * 2 - 1).astype(np.int8)


def algorithmic_bytes(m: int, n: int, p: int, batch: int = 1, group: int = GROUP) -> int:
    """Bytes the method itself must move for one uniform-precision call:
    the first p planes, scale set p, the activations in and the outputs out."""
    return m * n * p // 8 + m * (n // group) * p * 2 + batch * n * 2 + batch * m * 2
