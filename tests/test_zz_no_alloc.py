"""cer_matmul_noalloc -- the entry point for callers that cannot allocate device memory -- against the existing
entry points through the C ABI, under the bound of every product, |dY| <= 1e-5 * sum_c |W[r,c]| |X[c,l]|: two calls
in a row on one GPU, the second with a smaller input, so that the fixed workspace still holds the first call's
column sums when the second one starts.  Cases with a non-zero most frequent value and batch > 1 are the ones that
use the workspace; the others show that the call is a plain product."""
import numpy as np
import pytest

import oracle
from paper_1805_10692_amd import binding as B
from paper_1805_10692_amd import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5


def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: GPU parity tests need a real MI355X")
    return torch.device("cuda:0")


def _one(w, fmt, dev):
    enc = B.cer_encode if fmt == "cer" else B.cser_encode
    mm = B.cer_matmul if fmt == "cer" else B.cser_matmul
    h = enc(w.W, w.codebook)
    Xd = torch.from_numpy(np.ascontiguousarray(w.X)).to(dev)
    Yn = torch.full((w.m, w.L), float("nan"), dtype=torch.float32, device=dev)
    Ym = torch.full_like(Yn, float("nan"))
    Ys = torch.full_like(Yn, float("nan"))
    print(f"no-alloc case {w.name} {fmt} m={w.m} n={w.n} L={w.L}", flush=True)
    B.cer_matmul_noalloc(h, Xd, Yn, w.L)
    mm(h, Xd, Ym, w.L)                                         # the library's own choice of kernel, own temporaries
    same = B.MatmulOpts(path=B.CER_PATH_GEMM if w.L > 1 else B.CER_PATH_AUTO, flags=B.CER_OPT_ROWS_WHOLE)
    B.cer_matmul_ex(h, Xd, Ys, w.L, None, same)                # the kernel the no-alloc call runs for wide batches
    torch.cuda.synchronize()
    B.cer_free(h)
    yn, ym, ys = (t.cpu().numpy().astype(np.float64) for t in (Yn, Ym, Ys))
    scale = oracle.abs_dot_dense(w.W, w.X, threads=8)
    assert np.isfinite(yn).all(), f"{w.name}/{fmt}: unwritten output"
    assert (np.abs(yn - ym) <= TOL * scale).all(), f"{w.name}/{fmt}: differs from {mm.__name__}"
    assert (np.abs(yn - ys) <= TOL * scale).all(), f"{w.name}/{fmt}: differs from cer_matmul_ex"
    want = oracle.dot(oracle.encode(w.W, w.codebook, fmt), w.X, threads=8)
    assert (np.abs(yn - want) <= TOL * scale).all(), f"{w.name}/{fmt}: differs from the oracle"
    return yn, ys


@pytest.mark.parametrize("fmt", ["cer", "cser"])
def test_two_calls_in_a_row_second_one_smaller(fmt):
    dev = _gpu()
    big = wl.conv3x3(L=200, nonzero_dominant=True, scale=4)      # Omega[0] != 0, batch 200: column sums in the workspace
    small = wl.conv3x3(L=7, nonzero_dominant=True, scale=8)      # fewer rows, fewer columns, narrower batch
    yb, sb = _one(big, fmt, dev)
    ys, ss = _one(small, fmt, dev)
    # wide batches run the same kernel as cer_matmul_ex with every row whole: the same numbers
    assert np.array_equal(yb, sb)
    assert np.array_equal(ys, ss)


def test_other_shapes_and_the_size_limit():
    dev = _gpu()
    for w in (wl.conv3x3(L=1, nonzero_dominant=True, scale=4),                       # batch 1: X summed in LDS
              wl.random_lowentropy(m=9, n=70001, K=8, p_dom=0.9, L=1, seed=33),      # batch 1, X too big for LDS
              wl.alexnet_fc6(L=32, scale=8), wl.vgg_fc6(L=1, scale=8),                # Omega[0] = 0: no workspace
              wl.alexnet_fc6(L=3, scale=2)):                                         # narrow batch: one LDS tile
        for fmt in ("cer", "cser"):
            _one(w, fmt, dev)
    # a batch whose column sums exceed the fixed workspace is refused before anything is launched
    W = np.full((3, 2000), 0.5, np.float32)                      # most frequent value 0.5
    W[:, ::5] = 0.0
    h = B.cer_encode(W, np.array([0.0, 0.5], np.float32))
    assert B.cer_get_array(h, B.CER_ARRAY_OMEGA)[0] == 0.5
    L = 300000
    X = torch.zeros((2000, L), dtype=torch.float32, device=dev)
    Y = torch.zeros((3, L), dtype=torch.float32, device=dev)
    with pytest.raises(B.CerError) as e:
        B.cer_matmul_noalloc(h, X, Y, L)
    assert e.value.code == B.CER_E_TOO_LARGE
    B.cer_free(h)
