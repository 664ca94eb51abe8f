"""Randomised cases (seeded, so every run sees the same ones).

CPU part: the library's host encoder against the oracle on small random matrices with the awkward
ingredients mixed in (ties between counts, codebook values that never occur, -0.0, a non-zero most
frequent value, rows without entries, single rows / columns).
GPU part: products and the device front-end on random shapes and batch widths, against the oracle."""
import numpy as np
import pytest

import oracle
from oracle import quantizer as oq
from paper_1805_10692_amd import binding as B
from test_host_library import _compare

TOL = 1e-5


def random_case(seed):
    rng = np.random.default_rng(seed)
    m = int(rng.integers(1, 14))
    n = int(rng.choice([1, 2, 3, 7, 31, 64, 65, 130, 257, 300]))
    K = int(rng.integers(1, 9))
    cb = rng.choice(np.arange(-12, 13), size=K, replace=False).astype(np.float32) / 4
    if rng.random() < 0.3 and K > 1:
        cb[int(rng.integers(K))] = 0.0 if 0.0 not in cb else cb[0]
    cb = np.unique(cb).astype(np.float32)
    rng.shuffle(cb)
    K = len(cb)
    used = cb[: max(1, int(rng.integers(1, K + 1)))]            # some codebook values never occur
    p = rng.dirichlet(np.full(len(used), 0.4))
    W = used[rng.choice(len(used), size=(m, n), p=p)].astype(np.float32)
    if rng.random() < 0.5:
        W[int(rng.integers(m))] = W.flat[0]                      # a row of one value
    if rng.random() < 0.3:
        W = np.where(W == 0, np.float32(-0.0), W)                # -0.0 counts as +0.0
    return W, cb


@pytest.mark.parametrize("seed", range(60))
def test_host_encoder_random(seed):
    W, cb = random_case(seed)
    for fmt, enc, dec in (("cer", B.cer_encode, B.cer_decode), ("cser", B.cser_encode, B.cser_decode)):
        A = oracle.encode(W, cb, fmt)
        h = enc(W, cb)
        _compare(h, A)
        assert np.array_equal(dec(h).view(np.uint32), (W + np.float32(0)).view(np.uint32))
        B.cer_free(h)


def _gpu():
    torch = pytest.importorskip("torch")
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: GPU parity tests need a real MI355X")
    return torch, torch.device("cuda:0")


@pytest.mark.gpu
@pytest.mark.parametrize("seed", range(40))
def test_products_random(seed):
    torch, dev = _gpu()
    rng = np.random.default_rng(1000 + seed)
    m = int(rng.integers(1, 200))
    n = int(rng.choice([1, 5, 63, 64, 65, 255, 256, 257, 1000, 4099]))
    K = int(rng.choice([1, 2, 3, 8, 17, 64, 65, 200]))
    L = int(rng.choice([1, 1, 2, 3, 4, 7, 8, 16, 31, 32, 33, 64, 100]))
    cb = (rng.permutation(np.arange(-K, K + 1))[:K].astype(np.float32)) / 8
    p = rng.dirichlet(np.full(K, 0.3))
    W = cb[rng.choice(K, size=(m, n), p=p)].astype(np.float32)
    X = rng.standard_normal((n, L)).astype(np.float32)
    want = oracle.dot_dense(W, X, threads=4)
    scale = oracle.abs_dot_dense(W, X, threads=4)
    Xd = torch.from_numpy(X).to(dev)
    print(f"seed {seed}: m={m} n={n} K={K} L={L}", flush=True)
    for fmt, enc, mm in (("cer", B.cer_encode, B.cer_matmul), ("cser", B.cser_encode, B.cser_matmul)):
        h = enc(W, cb)
        # the library's own choice, then each kernel family preferred in turn (taken where it applies)
        # (the batch-1 stream kernel also without the rank table that handles of at most 64 values carry)
        for xt in (None, B.CER_PATH_GEMM, B.CER_PATH_XTILE, B.CER_PATH_DENSE, B.CER_PATH_GEMV, B.CER_PATH_GEMV_EXPAND,
                   "no_rank_table"):
            Yd = torch.full((m, L), float("nan"), dtype=torch.float32, device=dev)
            if xt is None:
                mm(h, Xd, Yd, L)
            elif xt == "no_rank_table":
                B.cer_matmul_ex(h, Xd, Yd, L, None, B.MatmulOpts(path=B.CER_PATH_GEMV, flags=B.CER_OPT_NO_RANK_TABLE))
            else:
                B.cer_matmul_ex(h, Xd, Yd, L, None, B.MatmulOpts(path=xt))
            torch.cuda.synchronize()
            Y = Yd.cpu().numpy().astype(np.float64)
            assert np.isfinite(Y).all(), (fmt, xt)
            assert np.all(np.abs(Y - want) <= TOL * scale), (fmt, xt, float(np.abs(Y - want).max()))
        B.cer_free(h)


@pytest.mark.gpu
@pytest.mark.parametrize("seed", range(30))
def test_front_end_random(seed):
    torch, dev = _gpu()
    rng = np.random.default_rng(2000 + seed)
    m = int(rng.integers(1, 60))
    n = int(rng.choice([1, 2, 3, 4, 63, 64, 65, 255, 256, 257, 300, 1001, 70000 if seed % 10 == 0 else 129]))
    bits = int(rng.integers(1, 9))
    fmt = "cer" if seed % 2 == 0 else "cser"
    W = (rng.laplace(0, 0.02, size=(m, n)) + (0.5 if seed % 3 == 0 else 0.0)).astype(np.float32)
    print(f"seed {seed}: m={m} n={n} bits={bits} {fmt}", flush=True)
    if m * n == 1 or float(W.max()) == float(W.min()):
        W[0, 0] = W[0, 0]                                         # constant: one point
    codes, cb = oq.uniform_quantize(W, bits)
    Wq = cb[codes]
    A = oracle.encode(Wq, cb, fmt)
    Wd = torch.from_numpy(W).to(dev)
    h, got_cb = B.cer_quantize_encode_device(Wd, m, n, bits, fmt)
    assert got_cb.tobytes() == cb.tobytes()
    _compare(h, A)
    B.cer_free(h)
    # the already quantized matrix through the look-up path gives the same handle
    h2 = B.cer_encode_device(torch.from_numpy(Wq).to(dev), m, n, cb, fmt)
    _compare(h2, A)
    B.cer_free(h2)
