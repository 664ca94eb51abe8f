"""CPU ORACLE -- TEST INFRASTRUCTURE, NOT PART OF THE PRODUCT.

Elementary-operation counts of one matrix-vector product, obtained by *running* Algorithms 1-4 of
the paper (Appendix A-C) as plain Python loops over the format arrays and counting every read,
multiplication, addition and write as it happens, and the energy those operations cost under
Table I.  Only small matrices: the loops are pure Python.

Two ways of counting, both from the paper:
  "theorem"  what Eq. (2), (4), (10), (12) and the proofs of Theorems 1 and 2 charge: the end of the
             previous row / group is carried over, so a row reads one rowPtr entry and each group one
             OmegaPtr entry; every element that takes part costs one addition.
  "example"  the hand count of Section III-B for a single row: both ends of the row's pointer range
             are read, and a sum of k terms costs k - 1 additions.
"""
from __future__ import annotations

import collections

# Table I (pJ, 45 nm CMOS).  Columns: 8, 16, 32 bits.  The 16-bit entry of the last row is printed
# as 5000.0; the caption says the read/write values were interpolated linearly, which gives 500.0.
TABLE_I = {
    "add": (0.2, 0.4, 0.9),
    "mul": (0.6, 1.1, 3.7),
    "rw_8KB": (1.25, 2.5, 5.0),
    "rw_32KB": (2.5, 5.0, 10.0),
    "rw_1MB": (12.5, 25.0, 50.0),
    "rw_big": (250.0, 500.0, 1000.0),
}


def rw_cost(bits: int, array_bytes: float) -> float:
    col = 0 if bits <= 8 else (1 if bits <= 16 else 2)
    if array_bytes < 8 * 1024:
        return TABLE_I["rw_8KB"][col]
    if array_bytes < 32 * 1024:
        return TABLE_I["rw_32KB"][col]
    if array_bytes < 1024 * 1024:
        return TABLE_I["rw_1MB"][col]
    return TABLE_I["rw_big"][col]


def count_dense(W, how: str) -> dict:
    """Algorithm 1 on one input vector."""
    c = collections.Counter()
    m, n = W.shape
    for _ in range(m):
        terms = 0
        for _ in range(n):
            c["read_weight"] += 1
            c["read_input"] += 1
            c["mul"] += 1
            terms += 1
            if how == "theorem" or terms > 1:
                c["add"] += 1
        c["write"] += 1
    return dict(c)


def count_csr(A, how: str) -> dict:
    """Algorithm 2 (A = oracle.CSR)."""
    c = collections.Counter()
    for r in range(A.m):
        c["read_rowPtr"] += 1 if how == "theorem" else 2
        terms = 0
        for _ in range(int(A.rowPtr[r]), int(A.rowPtr[r + 1])):
            c["read_colI"] += 1
            c["read_weight"] += 1
            c["read_input"] += 1
            c["mul"] += 1
            terms += 1
            if how == "theorem" or terms > 1:
                c["add"] += 1
        c["write"] += 1
    return dict(c)


def count_cer(A, how: str) -> dict:
    """Algorithm 3 (CER) or Algorithm 4 (CSER) (A = oracle.Encoded), multiply after the inner loop
    and only for a non-empty group; Appendix A-A1 when the most frequent value is not 0."""
    c = collections.Counter()
    for r in range(A.m):
        c["read_rowPtr"] += 1 if how == "theorem" else 2
        if how == "example":
            c["read_omegaPtr"] += 1          # the start of the row's first group
        terms = 0
        for g in range(int(A.rowPtr[r]), int(A.rowPtr[r + 1])):
            c["read_omegaPtr"] += 1
            if A.omegaI is not None:
                c["read_omegaI"] += 1
            size = int(A.omegaPtr[g + 1] - A.omegaPtr[g])
            for _ in range(size):
                c["read_colI"] += 1
                c["read_input"] += 1
                terms += 1
                if how == "theorem" or terms > 1:
                    c["add"] += 1            # one addition per gathered input (the first term of a row is free
                                             # in the hand count; Eq. (10) folds the group's add into c_Omega)
            if size > 0:
                c["read_omega"] += 1
                c["mul"] += 1
        c["write"] += 1
    if A.K > 0 and float(A.omega[0]) != 0.0 and A.m > 0:
        c["read_input"] += A.n                # c_out = Omega[0] * sum_i x_i ...
        c["add"] += A.n + A.m                 # ... added to every output
        c["mul"] += 1
        c["read_omega"] += 1
    return dict(c)


def total_ops(c: dict) -> int:
    return int(sum(c.values()))


def energy_pj(c: dict, m: int, n: int, arrays: dict) -> float:
    """arrays: name -> (element bits, array bytes) for weight / omega / colI / omegaPtr / rowPtr / omegaI."""
    e = c.get("mul", 0) * TABLE_I["mul"][2] + c.get("add", 0) * TABLE_I["add"][2]
    e += c.get("read_input", 0) * rw_cost(32, 4 * n) + c.get("write", 0) * rw_cost(32, 4 * m)
    for name, (bits, nbytes) in arrays.items():
        e += c.get("read_" + name, 0) * rw_cost(bits, nbytes)
    return float(e)
