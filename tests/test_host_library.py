"""Host logic of the HIP library, checked on the CPU (no GPU calls): the library's own encoder
against the oracle array by array and bit by bit, decode round trips, storage bits, error codes,
and that the built library exports every symbol the header declares."""
import os
import re

import numpy as np
import pytest

import oracle
from paper_1805_10692_amd import binding as B
from paper_1805_10692_amd import workloads as wl

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "cer.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b((?:cer|cser|csr|dense)_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert hasattr(L, name), name
    assert B.lib().cer_strerror(B.CER_E_FORMAT).decode().startswith("handle")


def _compare(h, A):
    d = B.cer_get_dims(h)
    assert (d["m"], d["n"], d["K"], d["nnz"], d["groups"]) == (A.m, A.n, A.K, A.nnz, A.G)
    assert d["is_cser"] == int(A.fmt == "cser")
    omega = B.cer_get_array(h, B.CER_ARRAY_OMEGA)
    assert omega.dtype == np.float32 and omega.tobytes() == A.omega.tobytes()
    assert np.array_equal(B.cer_get_array(h, B.CER_ARRAY_COUNT), A.count)
    bits = oracle.array_bits(A)
    for which, name in ((B.CER_ARRAY_COLI, "colI"), (B.CER_ARRAY_OMEGAPTR, "omegaPtr"), (B.CER_ARRAY_ROWPTR, "rowPtr")):
        got = B.cer_get_array(h, which)
        assert got.dtype.itemsize * 8 == bits[name], name
        assert np.array_equal(got.astype(np.int64), getattr(A, name)), name
    oi = B.cer_get_array(h, B.CER_ARRAY_OMEGAI)
    if A.fmt == "cser":
        assert oi.dtype.itemsize * 8 == bits["omegaI"]
        assert np.array_equal(oi.astype(np.int64), A.omegaI)
    else:
        assert len(oi) == 0
    assert B.cer_storage_bits(h) == oracle.storage_bits(A)
    st, so = B.cer_get_stats(h), oracle.stats(A)
    for k in ("H", "p0", "k_bar", "k_tilde"):
        assert st[k] == pytest.approx(so[k], rel=1e-12, abs=1e-15)


WORKLOADS = [
    lambda: wl.config1(),
    lambda: wl.alexnet_fc6(L=2, scale=16),
    lambda: wl.vgg_fc6(L=1, scale=16),
    lambda: wl.sweep_cell(256, 0.99, scale=8),
    lambda: wl.sweep_cell(256, 0.5, scale=8),
    lambda: wl.sweep_cell(2, 0.7, scale=8),
    lambda: wl.conv3x3(L=3, scale=4),
    lambda: wl.conv3x3(L=3, nonzero_dominant=True, scale=4),
    lambda: wl.random_lowentropy(m=7, n=200, K=5, p_dom=0.5, L=1, seed=5),      # n <= 256: 8-bit colI
    lambda: wl.random_lowentropy(m=3, n=70000, K=4, p_dom=0.9, L=1, seed=6),    # n > 65536: 32-bit colI
    lambda: wl.random_lowentropy(m=5, n=40, K=1, p_dom=1.0, L=1, seed=7),       # constant matrix
]


@pytest.mark.parametrize("make", WORKLOADS, ids=[str(i) for i in range(len(WORKLOADS))])
def test_encoder_matches_oracle_bit_exact(make):
    w = make()
    for fmt, enc, dec in (("cer", B.cer_encode, B.cer_decode), ("cser", B.cser_encode, B.cser_decode)):
        h = enc(w.W, w.codebook)
        _compare(h, oracle.encode(w.W, w.codebook, fmt))
        assert dec(h).tobytes() == w.W.tobytes()
        B.cer_free(h)


FULL_SIZE = {
    "alexnet_fc6": lambda: wl.alexnet_fc6(L=1),
    "vgg_fc6": lambda: wl.vgg_fc6(L=1),
    "conv3x3": lambda: wl.conv3x3(L=1),
    "conv3x3_nonzero_dominant": lambda: wl.conv3x3(L=1, nonzero_dominant=True),
}
FULL_SIZE.update({f"sweep_K{K}_p{p0}": (lambda K=K, p0=p0: wl.sweep_cell(K, p0, L=1)) for K in wl.SWEEP_K for p0 in wl.SWEEP_P0})


@pytest.mark.parametrize("name", list(FULL_SIZE))
def test_encoder_matches_oracle_bit_exact_at_full_size(name):
    """Every benchmark configuration at the size the benchmark runs it (config 1 is in the list above): all arrays,
    widths, counts, storage bits and statistics of the library's host encoder against the oracle's, both formats,
    and the decode round trip."""
    w = FULL_SIZE[name]()
    for fmt, enc, dec in (("cer", B.cer_encode, B.cer_decode), ("cser", B.cser_encode, B.cser_decode)):
        h = enc(w.W, w.codebook)
        _compare(h, oracle.encode(w.W, w.codebook, fmt))
        assert dec(h).tobytes() == w.W.tobytes()
        B.cer_free(h)


def test_matmul_options_are_validated_before_anything_runs():
    """cer_matmul_ex / cer_matmul_path_ex reject paths, tile widths and flags that the header does not define; on a
    machine without a device a valid call then fails with CER_E_HIP (there is no CPU product)."""
    import ctypes
    h = B.cer_encode(np.array([[0, 1, 2], [2, 2, 0]], np.float32), np.array([0.0, 1.0, 2.0], np.float32))
    L = B.lib()
    for bad in (B.MatmulOpts(path=6), B.MatmulOpts(path=-2), B.MatmulOpts(tile_cols=24), B.MatmulOpts(flags=128),
                B.MatmulOpts(flags=B.CER_OPT_SHORT_CHUNKS | B.CER_OPT_LONG_CHUNKS)):
        assert L.cer_matmul_ex(h.ptr, 16, 16, 1, None, ctypes.byref(bad)) == B.CER_E_INVALID
        assert L.cer_matmul_path_ex(h.ptr, 1, ctypes.byref(bad)) == B.CER_E_INVALID
    assert L.cer_matmul_ex(h.ptr, None, 16, 1, None, None) == B.CER_E_INVALID
    assert L.cer_matmul_path_ex(None, 1, None) == B.CER_E_INVALID
    assert L.cer_matmul_path_ex(h.ptr, 0, None) == B.CER_E_INVALID
    try:
        import torch
        has_gpu = torch.cuda.is_available()
    except ImportError:
        has_gpu = False
    if not has_gpu:
        ok = B.MatmulOpts(path=B.CER_PATH_GEMM, tile_cols=32, flags=B.CER_OPT_ROWS_WHOLE)
        assert L.cer_matmul_ex(h.ptr, 16, 16, 2, None, ctypes.byref(ok)) == B.CER_E_HIP
        assert L.cer_matmul_path_ex(h.ptr, 2, ctypes.byref(ok)) == B.CER_E_HIP
    B.cer_free(h)


def test_worked_example_through_the_library(example):
    M = example["M"].astype(np.float32)
    h = B.cer_encode(M, np.array([0, 2, 3, 4], np.float32))
    assert B.cer_get_array(h, B.CER_ARRAY_OMEGA).tolist() == example["cer_Omega"].tolist()
    assert B.cer_get_array(h, B.CER_ARRAY_COLI).tolist() == example["cer_colI"].tolist()
    assert B.cer_get_array(h, B.CER_ARRAY_OMEGAPTR).tolist() == example["cer_OmegaPtr"].tolist()
    assert B.cer_get_array(h, B.CER_ARRAY_ROWPTR).tolist() == example["cer_rowPtr"].tolist()
    entries = sum(len(B.cer_get_array(h, a)) for a in (B.CER_ARRAY_OMEGA, B.CER_ARRAY_COLI, B.CER_ARRAY_OMEGAPTR,
                                                       B.CER_ARRAY_ROWPTR))
    assert entries == 49
    hs = B.cser_encode(M, np.array([0, 2, 3, 4], np.float32))
    om = B.cer_get_array(hs, B.CER_ARRAY_OMEGA)
    assert om[B.cer_get_array(hs, B.CER_ARRAY_OMEGAI)].tolist() == [4, 3, 2, 4, 4, 3, 2, 4, 3, 4]
    assert entries + len(B.cer_get_array(hs, B.CER_ARRAY_OMEGAI)) == 59


def test_edge_cases_and_errors():
    cb = np.array([0.0, 1.0, 2.0], np.float32)
    # empty matrices
    for shape in ((0, 5), (4, 0), (0, 0)):
        h = B.cer_encode(np.zeros(shape, np.float32), cb)
        d = B.cer_get_dims(h)
        assert d["nnz"] == 0 and d["groups"] == 0
        assert B.cer_get_array(h, B.CER_ARRAY_ROWPTR).tolist() == [0] * (shape[0] + 1)
        assert B.cer_decode(h).shape == shape
    W = np.array([[0, 1, 2], [2, 2, 0]], np.float32)
    with pytest.raises(B.CerError) as e:
        B.cer_encode(W, np.array([0.0, 1.0], np.float32))
    assert e.value.code == B.CER_E_NOT_IN_CODEBOOK
    with pytest.raises(B.CerError) as e:
        B.cer_encode(W, np.array([0.0, 1.0, 2.0, 1.0], np.float32))
    assert e.value.code == B.CER_E_BAD_CODEBOOK
    with pytest.raises(B.CerError) as e:
        B.cser_encode(W, np.array([0.0, 1.0, 2.0, np.inf], np.float32))
    assert e.value.code == B.CER_E_BAD_CODEBOOK
    # -0.0 is +0.0
    h = B.cer_encode(np.array([[-0.0, 1.0, 0.0]], np.float32), np.array([-0.0, 1.0], np.float32))
    assert not np.signbit(B.cer_decode(h)).any()
    # format mismatch and null checks never reach the GPU
    with pytest.raises(B.CerError) as e:
        B.cser_decode(h)
    assert e.value.code == B.CER_E_FORMAT
    assert B.lib().cser_matmul(h.ptr, 16, 16, 1, None) == B.CER_E_FORMAT
    assert B.lib().cer_matmul(h.ptr, None, 16, 1, None) == B.CER_E_INVALID
    assert B.lib().cer_matmul(h.ptr, 16, 16, 0, None) == B.CER_E_INVALID
    assert B.lib().cer_matmul(None, 16, 16, 1, None) == B.CER_E_INVALID
    assert B.lib().dense_matmul(16, 16, None, 2, 2, 1, None) == B.CER_E_INVALID
    assert B.lib().cer_get_array(h.ptr, 99, None, None, None) == B.CER_E_INVALID
    B.cer_free(h)
    B.cer_free(h)  # second free of the wrapper is a no-op


def test_csr_comparator_host_side(example):
    M = example["M"].astype(np.float32)
    h = B.csr_encode(M)
    assert B.csr_get_array(h, 0).tolist() == example["csr_W"].tolist()
    assert B.csr_get_array(h, 1).tolist() == example["csr_colI"].tolist()
    assert B.csr_get_array(h, 2).tolist() == example["csr_rowPtr"].tolist()
    assert sum(len(B.csr_get_array(h, k)) for k in range(3)) == 62
    assert B.csr_decode(h).tobytes() == M.tobytes()
    w = wl.alexnet_fc6(L=1, scale=16)
    h = B.csr_encode(w.W)
    C = oracle.csr_encode(w.W)
    assert B.csr_get_array(h, 0).tobytes() == C.val.tobytes()
    assert np.array_equal(B.csr_get_array(h, 1).astype(np.int64), C.colI)
    assert np.array_equal(B.csr_get_array(h, 2).astype(np.int64), C.rowPtr)
    assert B.csr_decode(h).tobytes() == w.W.tobytes()
    nnz = len(C.val)
    assert B.csr_storage_bits(h) == nnz * 32 + nnz * oracle.min_bits(w.n - 1) + (w.m + 1) * oracle.min_bits(nnz)
    B.csr_free(h)


def test_device_front_end_without_a_device_fails_loudly():
    """No CPU fallback: with no GPU the device encoder reports a HIP error instead of encoding on the host."""
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    out = __import__("ctypes").c_void_p()
    W = np.zeros((2, 2), np.float32)
    cb = np.zeros(1, np.float32)
    rc = B.lib().cer_encode_device(W.ctypes.data, 2, 2, cb.ctypes.data, 1, 0, None, __import__("ctypes").byref(out))
    assert rc == B.CER_E_HIP and not out.value
    rc = B.lib().cer_encode_device(W.ctypes.data, 2, 2, cb.ctypes.data, 1, 7, None, __import__("ctypes").byref(out))
    assert rc == B.CER_E_INVALID
