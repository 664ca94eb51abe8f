"""CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.

The uniform quantizer of Section V-B (networks compressed without retraining): for one weight
matrix, take the range [w_min, w_max] of its elements, place K = 2^b equidistant points on it
(they become the codebook), and replace every element by the nearest point.  Plain numpy, one
statement per step.

Precision.  The paper fixes none.  Which point is "nearest" is an integer decision taken by
floating-point arithmetic, so it is defined here in the arithmetic the GPU path uses -- IEEE
binary32, one rounding per operation, in this order:

    step    = (w_max - w_min) / (K - 1)
    point_j = w_min + j * step          (j < K - 1),   point_{K-1} = w_max
    code(w) = clamp(round_half_even((w - w_min) / step), 0, K - 1)

Readings of what the paper leaves open:
  * the two ends of the range are themselves points (K points, K - 1 intervals);
  * an element halfway between two points goes to the even code (round-half-even of the scaled
    coordinate);
  * a constant matrix (w_min = w_max) has the single point w_min;
  * -0.0 counts as +0.0; NaN or infinite weights are an error.

Pinned in tests/test_quantizer_pins.py against an exact integer grid (hand-written codes), a brute
force nearest-point search in binary64, idempotence and monotonicity.
"""
from __future__ import annotations

import numpy as np

f32 = np.float32


def uniform_codebook(w_min: float, w_max: float, bits: int) -> np.ndarray:
    """The K = 2^bits points on [w_min, w_max] (one point if the range is empty)."""
    if not 1 <= bits <= 16:
        raise ValueError("bits must be in 1..16")
    w_min, w_max = f32(w_min) + f32(0), f32(w_max) + f32(0)  # -0.0 -> +0.0
    if not (np.isfinite(w_min) and np.isfinite(w_max)) or w_max < w_min:
        raise ValueError("range must be finite and ordered")
    if w_min == w_max:
        return np.array([w_min], dtype=f32)
    K = 1 << bits
    step = f32(f32(w_max - w_min) / f32(K - 1))
    j = np.arange(K, dtype=f32)
    points = (j * step).astype(f32) + w_min  # float32 product, then float32 sum
    points = points.astype(f32)
    points[K - 1] = w_max
    if not np.all(np.diff(points) > 0):
        raise ValueError("range too narrow for 2^bits distinct binary32 points")
    return points


def uniform_quantize(W: np.ndarray, bits: int):
    """Returns (codes, codebook): int64 codes of W's shape, float32 codebook; W_q = codebook[codes]."""
    W = np.asarray(W, dtype=f32)
    if W.size == 0:
        return np.zeros(W.shape, dtype=np.int64), np.zeros(0, dtype=f32)
    if not np.all(np.isfinite(W)):
        raise ValueError("weights must be finite")
    w_min, w_max = f32(W.min()) + f32(0), f32(W.max()) + f32(0)
    codebook = uniform_codebook(w_min, w_max, bits)
    if codebook.size == 1:
        return np.zeros(W.shape, dtype=np.int64), codebook
    K = codebook.size
    step = f32(f32(w_max - w_min) / f32(K - 1))
    t = ((W - w_min).astype(f32) / step).astype(f32)
    codes = np.clip(np.rint(t), 0, K - 1).astype(np.int64)
    return codes, codebook
