"""Seeded synthetic inputs: quantized low-entropy weight matrices W, their codebooks, and inputs X.

This module holds no arithmetic of the CER/CSER method: it only draws symbols from a stated
probability mass function and looks them up in a codebook.  The same arrays are handed to the CPU
oracle, to the HIP library and to the dense baseline, so no random-number difference can leak into
a parity check.

The matrices stand in for the paper's trained and quantized networks (Section V), which are not
available: shapes follow AlexNet fc6, VGG-16 fc6 and a 3x3x512 convolution written as a matrix
(Appendix A-A2); the element statistics (sparsity p0, entropy H) lie in the range of Table IV.
"""
from __future__ import annotations

import dataclasses
import math

import numpy as np


@dataclasses.dataclass
class Workload:
    name: str
    W: np.ndarray          # (m, n) float32, every element is a codebook value
    codebook: np.ndarray   # (K,) float32, distinct
    X: np.ndarray          # (n, L) float32, row-major
    pmf: np.ndarray        # (K,) float64, the distribution the symbols were drawn from
    seed: int

    @property
    def m(self) -> int:
        return self.W.shape[0]

    @property
    def n(self) -> int:
        return self.W.shape[1]

    @property
    def L(self) -> int:
        return self.X.shape[1]


def _order_by_abs(codebook: np.ndarray, skip: int) -> list[int]:
    """Indices of all codebook entries except `skip`, ascending |v|, the negative one first on ties."""
    idx = [j for j in range(len(codebook)) if j != skip]
    idx.sort(key=lambda j: (abs(float(codebook[j])), float(codebook[j])))
    return idx


def pmf_geometric(codebook: np.ndarray, dominant: int, p_dom: float, ratio: float) -> np.ndarray:
    """P(dominant)=p_dom; the rest decays geometrically over the other values sorted by |v|."""
    K = len(codebook)
    pmf = np.zeros(K, dtype=np.float64)
    order = _order_by_abs(codebook, dominant)
    w = np.array([ratio ** i for i in range(len(order))], dtype=np.float64)
    w *= (1.0 - p_dom) / w.sum()
    pmf[order] = w
    pmf[dominant] = p_dom
    return pmf


def pmf_laplace(codebook: np.ndarray, dominant: int, p_dom: float, scale: float) -> np.ndarray:
    """P(dominant)=p_dom; the rest proportional to exp(-|v|/scale)."""
    K = len(codebook)
    w = np.exp(-np.abs(codebook.astype(np.float64)) / scale)
    w[dominant] = 0.0
    w *= (1.0 - p_dom) / w.sum()
    w[dominant] = p_dom
    assert len(w) == K
    return w


def pmf_spike_slab(K: int, dominant: int, p_dom: float) -> np.ndarray:
    """P(dominant)=p_dom; the rest uniform over the other K-1 values."""
    pmf = np.full(K, (1.0 - p_dom) / (K - 1) if K > 1 else 0.0, dtype=np.float64)
    pmf[dominant] = p_dom
    return pmf


def sample_matrix(rng: np.random.Generator, m: int, n: int, codebook: np.ndarray,
                  pmf: np.ndarray, chunk_rows: int = 256) -> np.ndarray:
    """i.i.d. symbols by inverse-CDF sampling, looked up in the codebook; float32 (m, n)."""
    cdf = np.cumsum(pmf)
    cdf[-1] = 1.0
    W = np.empty((m, n), dtype=np.float32)
    cb = codebook.astype(np.float32)
    for r0 in range(0, m, chunk_rows):
        r1 = min(m, r0 + chunk_rows)
        u = rng.random((r1 - r0, n))
        sym = np.searchsorted(cdf, u, side="right")
        np.minimum(sym, len(cb) - 1, out=sym)
        W[r0:r1] = cb[sym]
    return W


def sample_X(rng: np.random.Generator, n: int, L: int, relu: bool = False) -> np.ndarray:
    X = rng.standard_normal((n, L)).astype(np.float32)
    if relu:
        np.maximum(X, 0.0, out=X)
    return np.ascontiguousarray(X)


def entropy_bits(pmf: np.ndarray) -> float:
    p = pmf[pmf > 0]
    return float(-(p * np.log2(p)).sum())


# ---------------------------------------------------------------------------------------------
# The named configurations.  `scale` shrinks m and n (keeping the distribution) for parity tests
# that must finish in seconds on the CPU; scale=1 is the full size.
# ---------------------------------------------------------------------------------------------

def _shrink(v: int, scale: int, ragged: int) -> int:
    return v if scale == 1 else max(1, v // scale + ragged)


def config1(seed: int = 0) -> Workload:
    """256x512, 16-value grid on [-1, 1) containing 0, P(0)=0.9, geometric (0.7) tail, L=1."""
    cb = np.array([(j - 8) / 8.0 for j in range(16)], dtype=np.float32)
    pmf = pmf_geometric(cb, dominant=8, p_dom=0.9, ratio=0.7)
    rng = np.random.Generator(np.random.PCG64(seed))
    W = sample_matrix(rng, 256, 512, cb, pmf)
    X = sample_X(rng, 512, 1)
    return Workload("c1_256x512_K16_p0.90", W, cb, X, pmf, seed)


def alexnet_fc6(L: int = 32, scale: int = 1, seed: int = 1) -> Workload:
    """4096x9216, 5-bit uniform levels on [-0.05, 0.05), P(0)=0.85, Laplace-shaped tail."""
    cb = np.array([(j - 16) * 0.1 / 32.0 for j in range(32)], dtype=np.float64).astype(np.float32)
    pmf = pmf_laplace(cb, dominant=16, p_dom=0.85, scale=0.01)
    m, n = _shrink(4096, scale, 3), _shrink(9216, scale, 5)
    rng = np.random.Generator(np.random.PCG64(seed))
    W = sample_matrix(rng, m, n, cb, pmf)
    X = sample_X(rng, n, L)
    return Workload(f"alexnet_fc6_{m}x{n}_K32_p0.85_L{L}", W, cb, X, pmf, seed)


def vgg_fc6(L: int = 1, scale: int = 1, seed: int = 2) -> Workload:
    """4096x25088, 16 levels spaced 0.01, P(0)=0.95, geometric (0.6) tail over |v|-sorted values."""
    cb = np.array([(j - 8) * 0.01 for j in range(16)], dtype=np.float64).astype(np.float32)
    pmf = pmf_geometric(cb, dominant=8, p_dom=0.95, ratio=0.6)
    m, n = _shrink(4096, scale, 3), _shrink(25088, scale, 5)
    rng = np.random.Generator(np.random.PCG64(seed))
    W = sample_matrix(rng, m, n, cb, pmf)
    X = sample_X(rng, n, L)
    return Workload(f"vgg_fc6_{m}x{n}_K16_p0.95_L{L}", W, cb, X, pmf, seed)


def vgg_fc6_unequal_rows(L: int = 64, sigma: float = 1.0, scale: int = 1, seed: int = 7) -> Workload:
    """The vgg_fc6 shape, values and number of indexed elements (5 % on average), but with log-normal row lengths
    (standard deviation `sigma` of the logarithm, capped at a full row): a stand-in for pruned layers, whose rows
    are not equally long.  Not one of the benchmark's configurations."""
    cb = np.array([(j - 8) * 0.01 for j in range(16)], dtype=np.float64).astype(np.float32)
    pmf = pmf_geometric(cb, dominant=8, p_dom=0.95, ratio=0.6)
    m, n = _shrink(4096, scale, 3), _shrink(25088, scale, 5)
    rng = np.random.Generator(np.random.PCG64(seed))
    density = np.minimum(0.05 * np.exp(sigma * rng.standard_normal(m) - sigma * sigma / 2), 1.0)
    others = np.array([j for j in range(16) if j != 8])
    tail = pmf[others] / pmf[others].sum()
    W = np.zeros((m, n), dtype=np.float32)
    for r in range(m):
        count = int(rng.binomial(n, density[r]))
        cols = rng.choice(n, size=count, replace=False)
        W[r, cols] = cb[others[rng.choice(len(others), size=count, p=tail)]]
    X = sample_X(rng, n, L)
    return Workload(f"vgg_fc6_unequal_rows_{m}x{n}_sigma{sigma}_L{L}", W, cb, X, pmf, seed)


SWEEP_K = (2, 4, 16, 64, 256)
SWEEP_P0 = (0.5, 0.7, 0.9, 0.99)


def sweep_cell(K: int, p0: float, L: int = 16, scale: int = 1, seed: int | None = None) -> Workload:
    """2048x2048 spike-and-slab cell: K levels on [-1, 1), P(0)=p0, the rest uniform."""
    cell = SWEEP_K.index(K) * len(SWEEP_P0) + SWEEP_P0.index(p0) if (
        K in SWEEP_K and p0 in SWEEP_P0) else 0
    if seed is None:
        seed = 3 + cell
    cb = np.array([(j - K // 2) / (K / 2.0) for j in range(K)], dtype=np.float64).astype(np.float32)
    pmf = pmf_spike_slab(K, dominant=K // 2, p_dom=p0)
    m, n = _shrink(2048, scale, 3), _shrink(2048, scale, 5)
    rng = np.random.Generator(np.random.PCG64(seed))
    W = sample_matrix(rng, m, n, cb, pmf)
    X = sample_X(rng, n, L)
    return Workload(f"sweep_{m}x{n}_K{K}_p0{p0:.2f}_L{L}", W, cb, X, pmf, seed)


def conv3x3(L: int = 3136, nonzero_dominant: bool = False, scale: int = 1, seed: int = 4) -> Workload:
    """512x4608 (3x3x512 filters as a matrix), 8 levels spaced 0.25, one value with P=0.6 (0, or
    0.25 in the variant whose most frequent value is not 0), the rest uniform; X = ReLU(N(0,1))."""
    cb = np.array([(j - 4) / 4.0 for j in range(8)], dtype=np.float32)
    dom = 5 if nonzero_dominant else 4
    pmf = pmf_spike_slab(8, dominant=dom, p_dom=0.6)
    m, n = _shrink(512, scale, 3), _shrink(4608, scale, 5)
    rng = np.random.Generator(np.random.PCG64(seed))
    W = sample_matrix(rng, m, n, cb, pmf)
    X = sample_X(rng, n, L, relu=True)
    tag = "dom0.25" if nonzero_dominant else "dom0"
    return Workload(f"conv3x3_{m}x{n}_K8_{tag}_L{L}", W, cb, X, pmf, seed)


def random_lowentropy(m: int, n: int, K: int, p_dom: float, L: int, seed: int,
                      ratio: float = 0.7, dominant: int | None = None) -> Workload:
    """Free-form small case for tests: K levels spaced 1/8 (exact in fp32), geometric tail."""
    cb = np.array([(j - K // 2) / 8.0 for j in range(K)], dtype=np.float32)
    dom = K // 2 if dominant is None else dominant
    pmf = pmf_geometric(cb, dominant=dom, p_dom=p_dom, ratio=ratio) if K > 1 else np.ones(1)
    rng = np.random.Generator(np.random.PCG64(seed))
    W = sample_matrix(rng, m, n, cb, pmf)
    X = sample_X(rng, n, L)
    return Workload(f"rand_{m}x{n}_K{K}_p{p_dom:.2f}_L{L}_s{seed}", W, cb, X, pmf, seed)


def dense_weights(m: int, n: int, seed: int = 5, outliers: float = 1e-4, sigma: float = 0.01,
                  tail: float = 5.0) -> np.ndarray:
    """Unquantized fp32 weights for the quantizer front-end (Section V-B): a Laplace body of scale
    `sigma` with a fraction `outliers` of elements drawn `tail` times wider, the heavy tail that makes
    the range of a trained layer several times its bulk.  Stands in for a trained layer's weights."""
    rng = np.random.Generator(np.random.PCG64(seed))
    W = rng.laplace(0.0, sigma, size=(m, n)).astype(np.float32)
    if outliers > 0 and W.size:
        k = max(1, int(round(outliers * W.size)))
        pos = rng.integers(0, W.size, size=k)
        W.reshape(-1)[pos] = rng.laplace(0.0, tail * sigma, size=k).astype(np.float32)
    return W


def describe(pmf: np.ndarray) -> dict:
    return {"H_bits": entropy_bits(pmf), "p_max": float(pmf.max()), "K": int(len(pmf)),
            "min_entropy_bits": -math.log2(float(pmf.max()))}
