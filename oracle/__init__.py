"""CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.

Thin ctypes wrapper around ``cer_oracle.c`` (the plain C implementation written from the paper)
plus the storage-cost and statistics formulas of Sections IIII and V.  Only ``tests/``, the smoke
check and the benchmark's ``cpu_baseline`` leg may import this package; the HIP library and its
Python binding never do, and this package never imports them.
"""
from __future__ import annotations

import ctypes
import dataclasses
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cer_oracle.c")
_LIB = os.path.join(_HERE, "libcer_oracle.so")


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (no GPU involved)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall",
                               "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None
_i64p = ctypes.POINTER(ctypes.c_int64)
_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)


def _L():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        lib.orc_min_bits.restype = ctypes.c_int
        lib.orc_min_bits.argtypes = [ctypes.c_int64]
        lib.orc_encode.restype = ctypes.c_int
        lib.orc_encode.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int64, _f32p, ctypes.c_int64,
                                   ctypes.c_int, ctypes.POINTER(ctypes.c_void_p)]
        lib.orc_free.argtypes = [ctypes.c_void_p]
        lib.orc_get_dims.argtypes = [ctypes.c_void_p] + [_i64p] * 5
        lib.orc_get_arrays.argtypes = [ctypes.c_void_p, _f32p, _i64p, _i64p, _i64p, _i64p, _i64p]
        lib.orc_decode.restype = ctypes.c_int
        lib.orc_decode.argtypes = [ctypes.c_int64, ctypes.c_int64, _f32p, ctypes.c_int64, _i64p, _i64p,
                                   _i64p, _i64p, _f32p]
        lib.orc_dot_cer.argtypes = [ctypes.c_int64, ctypes.c_int64, _f32p, _i64p, _i64p, _i64p, _f32p,
                                    ctypes.c_int64, _f64p, ctypes.c_int]
        lib.orc_dot_cser.argtypes = [ctypes.c_int64, ctypes.c_int64, _f32p, _i64p, _i64p, _i64p, _i64p,
                                     _f32p, ctypes.c_int64, _f64p, ctypes.c_int]
        lib.orc_dot_dense.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int64, _f32p, ctypes.c_int64, _f64p,
                                      ctypes.c_int]
        lib.orc_abs_dot_dense.argtypes = lib.orc_dot_dense.argtypes
        lib.orc_csr_encode.restype = ctypes.c_int64
        lib.orc_csr_encode.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int64, _f32p, _i64p, _i64p]
        lib.orc_dot_csr.argtypes = [ctypes.c_int64, _f32p, _i64p, _i64p, _f32p, ctypes.c_int64, _f64p]
        _lib = lib
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(_f32p)


def _i64(a):
    a = np.ascontiguousarray(a, dtype=np.int64)
    return a, a.ctypes.data_as(_i64p)


class OracleError(RuntimeError):
    def __init__(self, code: int):
        super().__init__({-1: "matrix element not in codebook", -2: "bad codebook",
                          -3: "out of memory", -4: "inconsistent arrays"}.get(code, f"error {code}"))
        self.code = code


@dataclasses.dataclass
class Encoded:
    """The arrays of Section III-A.  ``omegaI`` is None for CER."""
    fmt: str                 # "cer" | "cser"
    m: int
    n: int
    omega: np.ndarray        # float32 (K,), frequency-major; omega[0] is never indexed by a group
    count: np.ndarray        # int64 (K,), occurrences of omega[k] in the matrix
    colI: np.ndarray         # int64 (nnz,)
    omegaPtr: np.ndarray     # int64 (G+1,)
    rowPtr: np.ndarray       # int64 (m+1,)
    omegaI: np.ndarray | None  # int64 (G,)

    @property
    def K(self) -> int:
        return len(self.omega)

    @property
    def nnz(self) -> int:
        return len(self.colI)

    @property
    def G(self) -> int:
        return len(self.omegaPtr) - 1


def min_bits(max_value: int) -> int:
    """Section V: smallest of 8 / 16 / 32 bits that holds an unsigned index."""
    return int(_L().orc_min_bits(int(max_value)))


def encode(W: np.ndarray, codebook: np.ndarray, fmt: str) -> Encoded:
    """Dense matrix + codebook -> CER or CSER arrays (Section III-A)."""
    assert fmt in ("cer", "cser")
    W, Wp = _f32(W)
    cb, cbp = _f32(codebook)
    m, n = W.shape
    h = ctypes.c_void_p()
    rc = _L().orc_encode(Wp, m, n, cbp, len(cb), int(fmt == "cser"), ctypes.byref(h))
    if rc != 0:
        raise OracleError(rc)
    try:
        d = [ctypes.c_int64() for _ in range(5)]
        _L().orc_get_dims(h, *[ctypes.byref(x) for x in d])
        _, _, K, nnz, G = [int(x.value) for x in d]
        omega = np.empty(K, np.float32)
        count = np.empty(K, np.int64)
        colI = np.empty(nnz, np.int64)
        omegaPtr = np.empty(G + 1, np.int64)
        rowPtr = np.empty(m + 1, np.int64)
        omegaI = np.empty(G, np.int64) if fmt == "cser" else None
        _L().orc_get_arrays(h, omega.ctypes.data_as(_f32p), count.ctypes.data_as(_i64p),
                            colI.ctypes.data_as(_i64p), omegaPtr.ctypes.data_as(_i64p),
                            rowPtr.ctypes.data_as(_i64p),
                            omegaI.ctypes.data_as(_i64p) if omegaI is not None else None)
    finally:
        _L().orc_free(h)
    return Encoded(fmt, m, n, omega, count, colI, omegaPtr, rowPtr, omegaI)


def decode(A: Encoded) -> np.ndarray:
    """CER / CSER arrays -> dense float32 matrix."""
    W = np.empty((A.m, A.n), np.float32)
    om, omp = _f32(A.omega)
    ci, cip = _i64(A.colI)
    op, opp = _i64(A.omegaPtr)
    rp, rpp = _i64(A.rowPtr)
    if A.omegaI is not None:
        oi, oip = _i64(A.omegaI)
    else:
        oi, oip = None, None
    rc = _L().orc_decode(A.m, A.n, omp, len(om), cip, opp, rpp, oip, W.ctypes.data_as(_f32p))
    if rc != 0:
        raise OracleError(rc)
    return W


def dot(A: Encoded, X: np.ndarray, threads: int = 1) -> np.ndarray:
    """Group-sum product of Algorithm 3 (CER) or 4 (CSER); returns float64 (m, L)."""
    X, Xp = _f32(X)
    assert X.ndim == 2 and X.shape[0] == A.n
    L = X.shape[1]
    Y = np.empty((A.m, L), np.float64)
    om, omp = _f32(A.omega)
    ci, cip = _i64(A.colI)
    op, opp = _i64(A.omegaPtr)
    rp, rpp = _i64(A.rowPtr)
    Yp = Y.ctypes.data_as(_f64p)
    if A.omegaI is None:
        _L().orc_dot_cer(A.m, A.n, omp, cip, opp, rpp, Xp, L, Yp, threads)
    else:
        oi, oip = _i64(A.omegaI)
        _L().orc_dot_cser(A.m, A.n, omp, cip, oip, opp, rpp, Xp, L, Yp, threads)
    return Y


def dot_dense(W: np.ndarray, X: np.ndarray, threads: int = 1) -> np.ndarray:
    """Algorithm 1, fp64 accumulation; returns float64 (m, L)."""
    W, Wp = _f32(W)
    X, Xp = _f32(X)
    m, n = W.shape
    L = X.shape[1]
    Y = np.empty((m, L), np.float64)
    _L().orc_dot_dense(Wp, m, n, Xp, L, Y.ctypes.data_as(_f64p), threads)
    return Y


def abs_dot_dense(W: np.ndarray, X: np.ndarray, threads: int = 1) -> np.ndarray:
    """sum_c |W[r,c]| |X[c,l]| in fp64 (the scale of the fp32 rounding-error bound)."""
    W, Wp = _f32(W)
    X, Xp = _f32(X)
    m, n = W.shape
    L = X.shape[1]
    S = np.empty((m, L), np.float64)
    _L().orc_abs_dot_dense(Wp, m, n, Xp, L, S.ctypes.data_as(_f64p), threads)
    return S


@dataclasses.dataclass
class CSR:
    m: int
    n: int
    val: np.ndarray
    colI: np.ndarray
    rowPtr: np.ndarray


def csr_encode(W: np.ndarray) -> CSR:
    """CSR of Section III-A (non-zero values, their columns, row pointers)."""
    W, Wp = _f32(W)
    m, n = W.shape
    rowPtr = np.empty(m + 1, np.int64)
    nnz = int(_L().orc_csr_encode(Wp, m, n, None, None, rowPtr.ctypes.data_as(_i64p)))
    val = np.empty(nnz, np.float32)
    colI = np.empty(nnz, np.int64)
    _L().orc_csr_encode(Wp, m, n, val.ctypes.data_as(_f32p), colI.ctypes.data_as(_i64p),
                        rowPtr.ctypes.data_as(_i64p))
    return CSR(m, n, val, colI, rowPtr)


def dot_csr(A: CSR, X: np.ndarray) -> np.ndarray:
    X, Xp = _f32(X)
    L = X.shape[1]
    Y = np.empty((A.m, L), np.float64)
    v, vp = _f32(A.val)
    ci, cip = _i64(A.colI)
    rp, rpp = _i64(A.rowPtr)
    _L().orc_dot_csr(A.m, vp, cip, rpp, Xp, L, Y.ctypes.data_as(_f64p))
    return Y


# ---------------------------------------------------------------------------------------------
# Storage cost (Section IV-C, Theorems 1 and 2 and their proofs) and statistics (Section III, III).
# ---------------------------------------------------------------------------------------------

def entries(A: Encoded) -> int:
    """Number of stored entries, every array counted with its leading-zero sentinel, as in the
    worked example of Section III-A (49 for CER, 59 for CSER of the 5x12 matrix)."""
    e = A.K + A.nnz + len(A.omegaPtr) + len(A.rowPtr)
    if A.omegaI is not None:
        e += len(A.omegaI)
    return int(e)


def array_bits(A: Encoded) -> dict:
    """Width of each array: fp32 values, each index array the smallest of 8/16/32 bits that holds
    its largest possible value (Section V)."""
    bits = {"omega": 32, "colI": min_bits(A.n - 1), "omegaPtr": min_bits(A.nnz),
            "rowPtr": min_bits(A.G)}
    if A.omegaI is not None:
        bits["omegaI"] = min_bits(A.K - 1)
    return bits


def storage_bits(A: Encoded) -> int:
    """Total bits = sum over arrays of length x width (proofs of Theorems 1 and 2, with the
    pointer arrays' leading zeros counted)."""
    b = array_bits(A)
    t = A.K * b["omega"] + A.nnz * b["colI"] + len(A.omegaPtr) * b["omegaPtr"] + len(A.rowPtr) * b["rowPtr"]
    if A.omegaI is not None:
        t += len(A.omegaI) * b["omegaI"]
    return int(t)


def stats(A: Encoded) -> dict:
    """p_k = #(w_k)/N, H = -sum p_k log2 p_k (Section III); k_bar = mean number of distinct
    non-dominant values per row, k_tilde = mean number of padding (empty) groups per row
    (Theorem 1)."""
    N = A.m * A.n
    p = A.count.astype(np.float64) / max(N, 1)
    H = float(-(p[p > 0] * np.log2(p[p > 0])).sum())
    sizes = np.diff(A.omegaPtr)
    nonempty = int((sizes > 0).sum())
    return {"H": H, "p0": float(p[0]) if len(p) else 0.0, "K": A.K, "nnz": A.nnz, "G": A.G,
            "k_bar": nonempty / max(A.m, 1), "k_tilde": (A.G - nonempty) / max(A.m, 1)}
