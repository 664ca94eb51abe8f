"""Pins of the oracle's uniform quantizer (Section V-B) -- CPU only, no HIP library.

The oracle takes the nearest-point decision in binary32 arithmetic; these tests tie it to things it
does not compute itself: hand-written codes on a grid where every step is exact, a brute-force
nearest-point search in binary64, and properties any nearest-point quantizer has.
"""
import numpy as np
import pytest

import oracle
from oracle import quantizer as q
from paper_1805_10692_amd import workloads as wl


def test_integer_grid_by_hand():
    """Range [0, 7] with 3 bits: step = 1 exactly, points 0..7, code = round-half-even(w)."""
    w = np.array([[0.0, 7.0, 0.49, 0.5, 0.51, 1.5, 2.5, 3.5],
                  [2.49, 6.5, 6.51, 5.5, 4.5, 3.0, 1.0, 6.99]], np.float32)
    expect = [[0, 7, 0, 0, 1, 2, 2, 4],
              [2, 6, 7, 6, 4, 3, 1, 7]]
    codes, cb = q.uniform_quantize(w, 3)
    assert cb.tolist() == [0, 1, 2, 3, 4, 5, 6, 7]
    assert codes.tolist() == expect


def test_shifted_scaled_grid_by_hand():
    """Range [-2, 1] with 2 bits: step = 1, points -2,-1,0,1.  One bit: the two ends only."""
    w = np.array([-2.0, 1.0, -1.4, -0.6, 0.4, 0.75, -0.5, -1.5, 0.5], np.float32)
    codes, cb = q.uniform_quantize(w, 2)
    assert cb.tolist() == [-2, -1, 0, 1]
    assert codes.tolist() == [0, 3, 1, 1, 2, 3, 2, 0, 2]     # -0.5 -> t=1.5 -> 2; -1.5 -> t=0.5 -> 0; 0.5 -> t=2.5 -> 2
    codes, cb = q.uniform_quantize(w, 1)
    assert cb.tolist() == [-2, 1]
    assert codes.tolist() == [0, 1, 0, 0, 1, 1, 0, 0, 1]     # midpoint is -0.5 -> t=0.5 -> even code 0


@pytest.mark.parametrize("bits", [1, 2, 4, 7, 8])
def test_nearest_point_brute_force(bits):
    """Every element goes to a point that a binary64 exhaustive search finds nearest; a different
    point is tolerated only for an element that sits on a midpoint to within binary32 rounding."""
    W = wl.dense_weights(64, 300, seed=11)
    codes, cb = q.uniform_quantize(W, bits)
    assert cb.dtype == np.float32 and len(cb) == 2 ** bits
    d = np.abs(W.astype(np.float64)[..., None] - cb.astype(np.float64)[None, None, :])   # all distances
    best = d.argmin(axis=-1)
    chosen = np.take_along_axis(d, codes[..., None], axis=-1)[..., 0]
    step = (float(cb[-1]) - float(cb[0])) / (len(cb) - 1)
    slack = 4 * np.finfo(np.float32).eps * max(abs(float(cb[0])), abs(float(cb[-1])))
    assert np.all(chosen <= d.min(axis=-1) + slack)
    assert np.all(chosen <= step / 2 + slack)
    differs = codes != best
    assert differs.mean() < 1e-3
    # and where it differs the two candidates are neighbours
    assert np.all(np.abs(codes[differs] - best[differs]) == 1)


def test_codebook_shape():
    W = wl.dense_weights(50, 200, seed=3)
    for bits in (1, 3, 7, 8, 10):
        codes, cb = q.uniform_quantize(W, bits)
        assert cb[0] == W.min() and cb[-1] == W.max()
        assert np.all(np.diff(cb) > 0)
        gaps = np.diff(cb.astype(np.float64))
        assert np.allclose(gaps, gaps.mean(), rtol=0, atol=2e-7 * max(abs(float(cb[0])), abs(float(cb[-1]))))
        assert codes[np.unravel_index(W.argmin(), W.shape)] == 0
        assert codes[np.unravel_index(W.argmax(), W.shape)] == len(cb) - 1
        # monotone: a larger weight never gets a smaller code
        order = np.argsort(W, axis=None, kind="stable")
        assert np.all(np.diff(codes.reshape(-1)[order]) >= 0)


def test_idempotent_and_lossless_chain():
    """Quantizing an already quantized matrix changes nothing, and the quantized matrix survives the
    CER / CSER round trip bit for bit (the conversion after quantization is lossless, Section V-B)."""
    W = wl.dense_weights(40, 333, seed=8)
    codes, cb = q.uniform_quantize(W, 7)
    Wq = cb[codes]
    codes2, cb2 = q.uniform_quantize(Wq, 7)
    assert np.array_equal(cb, cb2) and np.array_equal(codes, codes2)
    for fmt in ("cer", "cser"):
        A = oracle.encode(Wq, cb, fmt)
        assert np.array_equal(oracle.decode(A).view(np.uint32), Wq.view(np.uint32))
        # the encoder keeps only the points that occur, most frequent first
        used, cnt = np.unique(codes, return_counts=True)
        assert A.K == len(used)
        assert A.count.tolist() == sorted(cnt.tolist(), reverse=True)


def test_degenerate_inputs():
    codes, cb = q.uniform_quantize(np.full((3, 4), 0.25, np.float32), 7)
    assert cb.tolist() == [0.25] and not codes.any()
    codes, cb = q.uniform_quantize(np.zeros((0, 5), np.float32), 4)
    assert codes.shape == (0, 5) and cb.size == 0
    codes, cb = q.uniform_quantize(np.array([[-0.0, 1.0]], np.float32), 1)
    assert not np.signbit(cb[0])
    with pytest.raises(ValueError):
        q.uniform_quantize(np.array([[0.0, np.nan]], np.float32), 4)
    with pytest.raises(ValueError):
        q.uniform_quantize(np.array([[0.0, np.inf]], np.float32), 4)
    with pytest.raises(ValueError):      # 256 distinct binary32 numbers do not fit between 1 and 1 + 8 ulp
        q.uniform_quantize(np.array([[1.0, 1.0 + 8 * 2.0 ** -23]], np.float32), 8)


def test_statistics_in_the_papers_range():
    """Seven-bit quantization of the synthetic layer lands between the paper's ResNet152 and
    DenseNet rows of Table IV (p0 0.12 .. 0.36, H 3.7 .. 4.1 bits, within a margin)."""
    W = wl.dense_weights(512, 4608)
    codes, cb = q.uniform_quantize(W, 7)
    p = np.bincount(codes.ravel(), minlength=128) / codes.size
    p = p[p > 0]
    H = float(-(p * np.log2(p)).sum())
    assert 0.10 < p.max() < 0.40 and 3.0 < H < 4.5
