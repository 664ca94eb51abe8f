"""Rows much longer than the average row (pruned layers have them; matrices of independent elements do not).

The default batched kernel serves such rows in parts (the row's own work item takes the first part, every
further part is a work item of its own, a second kernel adds the parts' sums to Y); batch 1 keeps them whole.  Checked here against the
oracle element by element, for both formats, aligned and ragged batch widths, few and many groups per row, a
non-zero most frequent value, and against the same product with the rows left whole."""
import numpy as np
import pytest

import oracle
from paper_1805_10692_amd import binding as B

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5
GATHER = B.MatmulOpts(path=B.CER_PATH_GEMM)                                      # the kernel that gathers from L2
GATHER_ROWS_WHOLE = B.MatmulOpts(path=B.CER_PATH_GEMM, flags=B.CER_OPT_ROWS_WHOLE)  # ... rows in place and whole


def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: GPU parity tests need a real MI355X")
    return torch.device("cuda:0")


def skewed_matrix(seed, m, n, K, dominant, long_rows, base=0.02):
    """Sparse rows (`base` of the elements indexed) with a few rows of `long_rows` densities mixed in; one row
    without entries."""
    rng = np.random.default_rng(seed)
    cb = ((np.arange(K) - K // 2) / 8).astype(np.float32)
    dom = np.float32(dominant)
    assert dom in cb
    others = cb[cb != dom]
    W = np.full((m, n), dom, dtype=np.float32)
    dens = np.full(m, base)
    where = rng.choice(m, size=len(long_rows), replace=False)
    dens[where] = long_rows
    dens[(where[0] + 1) % m] = 0.0 if (where[0] + 1) % m not in where else dens[(where[0] + 1) % m]
    for r in range(m):
        cnt = int(round(dens[r] * n))
        cols = rng.choice(n, size=cnt, replace=False)
        W[r, cols] = others[rng.integers(len(others), size=cnt)]
    return W, cb, where


@pytest.mark.parametrize("K,dominant", [(16, 0.0), (200, 0.0), (8, 0.25)])
def test_long_rows_in_parts(K, dominant):
    dev = _gpu()
    m, n = 96, 12000
    W, cb, where = skewed_matrix(11 + K, m, n, K, dominant, [1.0, 0.9, 0.55, 0.36])
    for fmt, enc, mm in (("cer", B.cer_encode, B.cer_matmul), ("cser", B.cser_encode, B.cser_matmul)):
        h = enc(W, cb)
        # average row about 700 indexed elements -> parts of 2048; rows of 12000, 10800, 6600, 4320 elements
        # -> 5 + 5 + 3 + 2 further parts
        assert B.cer_long_row_parts(h) == 15, f"{fmt}: {B.cer_long_row_parts(h)} parts"
        for L in (1, 2, 7, 32, 33, 64, 100):
            rng = np.random.default_rng(100 + L)
            X = rng.standard_normal((n, L)).astype(np.float32)
            want = oracle.dot_dense(W, X, threads=8)
            scale = oracle.abs_dot_dense(W, X, threads=8)     # the stated bound, also with a non-zero most frequent value
            Xd = torch.from_numpy(X).to(dev)
            results = {}
            for split in ("1", "0"):
                print(f"{fmt} K={K} L={L} split={split}", flush=True)
                Yd = torch.full((m, L), float("nan"), dtype=torch.float32, device=dev)
                B.cer_matmul_ex(h, Xd, Yd, L, None, GATHER if split == "1" else GATHER_ROWS_WHOLE)
                torch.cuda.synchronize()
                Y = Yd.cpu().numpy().astype(np.float64)
                assert np.isfinite(Y).all(), f"{fmt} K={K} L={L} split={split}: unwritten output"
                bad = np.abs(Y - want) > TOL * scale
                assert not bad.any(), f"{fmt} K={K} L={L} split={split}: {int(bad.sum())} elements, rows {np.unique(np.nonzero(bad)[0])[:8]}"
                results[split] = Y
            # rows that are not split are computed by the same code either way (batch 1: with so few rows the stream
            # kernel shares every row between waves unless told to keep rows whole, so only the bound applies)
            short = np.setdiff1d(np.arange(m), where)
            if L > 1:
                assert np.array_equal(results["1"][short], results["0"][short]), f"{fmt} K={K} L={L}"
        B.cer_free(h)


@pytest.mark.parametrize("m", [203, 64, 9])
def test_rows_in_order_of_length_without_parts(m):
    """Longest row 2400 indices against 430 - 1130 on average: the batched kernel takes the rows in descending
    order of length (no row is long enough to be split).  Row counts that are not multiples of 4 or of the 8 XCD
    ranges."""
    dev = _gpu()
    n = 4000
    W, cb, _ = skewed_matrix(3 + m, m, n, 16, 0.0, [0.6, 0.6, 0.55, 0.3], base=0.1)
    for fmt, enc, mm in (("cer", B.cer_encode, B.cer_matmul), ("cser", B.cser_encode, B.cser_matmul)):
        h = enc(W, cb)
        assert B.cer_long_row_parts(h) == 0
        for L in (2, 8, 32, 33, 64, 100, 300):
            X = np.random.default_rng(L).standard_normal((n, L)).astype(np.float32)
            want = oracle.dot_dense(W, X, threads=8)
            scale = oracle.abs_dot_dense(W, X, threads=8)
            Xd = torch.from_numpy(X).to(dev)
            results = {}
            for split in ("1", "0"):
                print(f"{fmt} m={m} L={L} split={split}", flush=True)
                Yd = torch.full((m, L), float("nan"), dtype=torch.float32, device=dev)
                B.cer_matmul_ex(h, Xd, Yd, L, None, GATHER if split == "1" else GATHER_ROWS_WHOLE)
                torch.cuda.synchronize()
                Y = Yd.cpu().numpy().astype(np.float64)
                assert np.isfinite(Y).all(), f"{fmt} m={m} L={L} split={split}: unwritten output"
                assert (np.abs(Y - want) <= TOL * scale).all(), f"{fmt} m={m} L={L} split={split}"
                results[split] = Y
            assert np.array_equal(results["1"], results["0"]), f"{fmt} m={m} L={L}: a row's arithmetic does not depend on the order"
        B.cer_free(h)


@pytest.mark.parametrize("fmt", ["cer", "cser"])
def test_device_encoder_builds_the_same_schedule(fmt):
    """A handle made by the device-side encoder serves long rows in the same parts as the host encoder's, and the
    products of the two handles are the same numbers."""
    dev = _gpu()
    m, n = 96, 12000
    W, cb, _ = skewed_matrix(77, m, n, 16, 0.0, [1.0, 0.9, 0.55, 0.36])
    enc = B.cer_encode if fmt == "cer" else B.cser_encode
    hh = enc(W, cb)
    hd = B.cer_encode_device(torch.from_numpy(W).to(dev), m, n, cb, fmt)
    assert B.cer_long_row_parts(hh) == 15
    assert B.cer_long_row_parts(hd) == 15
    for L in (8, 64, 100):
        X = np.random.default_rng(L).standard_normal((n, L)).astype(np.float32)
        Xd = torch.from_numpy(X).to(dev)
        Yh = torch.full((m, L), float("nan"), dtype=torch.float32, device=dev)
        Yd = torch.full((m, L), float("nan"), dtype=torch.float32, device=dev)
        B.cer_matmul_ex(hh, Xd, Yh, L, None, GATHER)
        B.cer_matmul_ex(hd, Xd, Yd, L, None, GATHER)
        torch.cuda.synchronize()
        want = oracle.dot_dense(W, X, threads=8)
        scale = oracle.abs_dot_dense(W, X, threads=8)
        assert (np.abs(Yd.cpu().numpy().astype(np.float64) - want) <= TOL * scale).all(), f"{fmt} L={L}"
        assert torch.equal(Yh, Yd), f"{fmt} L={L}"
    B.cer_free(hh)
    B.cer_free(hd)


def test_layer_shapes_have_no_split_rows():
    """Matrices of independent elements (the benchmark's shapes) keep every row whole, so their products run the
    same kernels as before."""
    from paper_1805_10692_amd import workloads as wl
    for w in (wl.alexnet_fc6(L=1, scale=4), wl.vgg_fc6(L=1, scale=4), wl.sweep_cell(256, 0.5, L=1, scale=2)):
        h = B.cer_encode(w.W, w.codebook)
        assert B.cer_long_row_parts(h) == 0, w.name
        B.cer_free(h)


def test_repeated_and_cloned_products_with_split_rows():
    """The parts' temporary is allocated per call: calls in a row, on a clone and on two streams give the same Y."""
    dev = _gpu()
    W, cb, _ = skewed_matrix(5, 64, 9000, 16, 0.0, [1.0, 0.7])
    X = np.random.default_rng(6).standard_normal((9000, 32)).astype(np.float32)
    Xd = torch.from_numpy(X).to(dev)
    h = B.cer_encode(W, cb)
    assert B.cer_long_row_parts(h) > 0
    c = B.cer_clone_device(h)
    assert B.cer_long_row_parts(c) == B.cer_long_row_parts(h)
    Y0 = torch.empty(64, 32, device=dev)
    B.cer_matmul(h, Xd, Y0, 32)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for i in range(6):
        Y = torch.full((64, 32), float("nan"), device=dev)
        s = s1 if i % 2 else s2
        B.cer_matmul(c if i % 3 == 0 else h, Xd, Y, 32, stream=s)
        outs.append(Y)
    torch.cuda.synchronize()
    for Y in outs:
        assert torch.equal(Y, Y0)
    B.cer_free(h)
    B.cer_free(c)
