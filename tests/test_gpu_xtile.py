"""GPU parity of the batched kernel that keeps the input tile in LDS (reuse of X, Section V-C),
preferred through cer_matmul_ex and checked element by element against the oracle, under the same bound
as every other product:  |Y - Y_oracle| <= 1e-5 * sum_c |W[r,c]| |X[c,l]|."""
import numpy as np
import pytest

import oracle
from paper_1805_10692_amd import binding as B
from paper_1805_10692_amd import workloads as wl

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = 1e-5


XTILE = B.MatmulOpts(path=B.CER_PATH_XTILE)


def _gpu():
    if not torch.cuda.is_available():
        pytest.fail("no GPU visible: GPU parity tests need a real MI355X")
    return torch.device("cuda:0")


def run_and_check(W, codebook, X, what, expect_path=2, fmts=("cer", "cser")):
    dev = _gpu()
    L = X.shape[1]
    print(f"case {what} m={W.shape[0]} n={W.shape[1]} L={L}", flush=True)
    scale = oracle.abs_dot_dense(W, X, threads=8)
    want = oracle.dot_dense(W, X, threads=8)
    Xd = torch.from_numpy(np.ascontiguousarray(X)).to(dev)
    for fmt in fmts:
        h = (B.cer_encode if fmt == "cer" else B.cser_encode)(W, codebook)
        assert B.cer_matmul_path_ex(h, L, XTILE) == expect_path, f"{what}/{fmt}: kernel {B.cer_matmul_path_ex(h, L, XTILE)}"
        Yd = torch.full((W.shape[0], L), float("nan"), dtype=torch.float32, device=dev)
        B.cer_matmul_ex(h, Xd, Yd, L, None, XTILE)
        torch.cuda.synchronize()
        Y = Yd.cpu().numpy().astype(np.float64)
        B.cer_free(h)
        assert np.isfinite(Y).all(), f"{what}/{fmt}: unwritten or non-finite output"
        err = np.abs(Y - want)
        bad = err > TOL * scale
        assert not bad.any(), (f"{what}/{fmt}: {int(bad.sum())} elements beyond tolerance, worst ratio "
                               f"{float((err / np.maximum(scale, 1e-300)).max()):.3e} at {np.argwhere(bad)[:4].tolist()}")


CASES = {
    "alexnet_s8_L32": lambda: wl.alexnet_fc6(L=32, scale=8),          # n = 1152, K = 32: V = 8
    "alexnet_s2_L32": lambda: wl.alexnet_fc6(L=32, scale=2),          # n = 4608: V = 8 just fits
    "vgg_s4_L64": lambda: wl.vgg_fc6(L=64, scale=4),                  # n = 6272: V = 4
    "conv_s4_L200": lambda: wl.conv3x3(L=200, scale=4),
    "conv_s4_dom_L200": lambda: wl.conv3x3(L=200, nonzero_dominant=True, scale=4),   # constant term added at the store
    "conv_s4_dom_L7": lambda: wl.conv3x3(L=7, nonzero_dominant=True, scale=4),
    "sweep_K16_p90": lambda: wl.sweep_cell(16, 0.9, L=16, scale=4),
    "sweep_K64_p50": lambda: wl.sweep_cell(64, 0.5, L=16, scale=4),   # 63 groups in every row: the limit
    "sweep_K2_p70": lambda: wl.sweep_cell(2, 0.7, L=16, scale=4),
    "u8_index_L12": lambda: wl.random_lowentropy(m=70, n=250, K=6, p_dom=0.6, L=12, seed=32),
    "u32_index_L5": lambda: wl.random_lowentropy(m=9, n=70001, K=8, p_dom=0.9, L=5, seed=34),   # too wide for LDS
    "one_row": lambda: wl.random_lowentropy(m=1, n=3000, K=16, p_dom=0.7, L=9, seed=36),
    "one_col": lambda: wl.random_lowentropy(m=300, n=1, K=3, p_dom=0.5, L=4, seed=37),
    "constant": lambda: wl.random_lowentropy(m=10, n=100, K=1, p_dom=1.0, L=3, seed=38),
    "rows_1025": lambda: wl.random_lowentropy(m=1025, n=700, K=12, p_dom=0.85, L=24, seed=44),
    "sparse_rows": lambda: wl.random_lowentropy(m=333, n=900, K=5, p_dom=0.998, L=6, seed=45),   # most rows empty
}
NOT_APPLICABLE = {"u32_index_L5"}


@pytest.mark.parametrize("name", list(CASES))
def test_lds_variant_all_elements(name):
    w = CASES[name]()
    run_and_check(w.W, w.codebook, w.X, w.name, expect_path=1 if name in NOT_APPLICABLE else 2)


@pytest.mark.parametrize("L", [2, 3, 4, 5, 7, 8, 9, 15, 16, 17, 33, 100])
def test_lds_variant_ragged_batch_widths(L):
    w = wl.random_lowentropy(m=67, n=1500, K=16, p_dom=0.8, L=L, seed=200 + L)
    run_and_check(w.W, w.codebook, w.X, w.name)


def test_lds_variant_rows_without_entries_and_padding_groups():
    """Empty rows at the start, in the middle and at the end of a wave's block of rows; a row whose only
    entry has the highest rank (CER pads it with repeated pointers); rows that end exactly on a
    64-position window edge."""
    cb = np.array([0.0, 1.0, -2.0, 0.5, 3.0], np.float32)
    rng = np.random.default_rng(5)
    W = np.zeros((40, 640), np.float32)
    W[3, :64] = 1.0                       # exactly one window
    W[4, :128] = -2.0                     # exactly two windows
    W[5, 7] = 3.0                         # rarest value alone
    W[9] = cb[rng.integers(0, 5, size=640)]
    W[10] = cb[rng.integers(1, 5, size=640)]   # no zero at all
    W[20:24] = cb[rng.integers(0, 5, size=(4, 640))]
    W[39, 639] = 0.5
    X = rng.standard_normal((640, 6)).astype(np.float32)
    run_and_check(W, cb, X, "hand-built rows")


def test_falls_back_when_not_applicable():
    """More than 63 groups in a row or more than 64 values: the L2-gather kernel runs, result unchanged."""
    w = wl.random_lowentropy(m=40, n=2000, K=200, p_dom=0.3, L=8, seed=40, ratio=0.995)
    run_and_check(w.W, w.codebook, w.X, w.name, expect_path=1)


def test_full_size_alexnet_fc6_batch32_all_outputs():
    w = wl.alexnet_fc6(L=32)
    run_and_check(w.W, w.codebook, w.X, w.name)


def test_automatic_choice_for_narrow_batches():
    """Left to itself the library takes this kernel for narrow batches of a large matrix whose input fits in LDS
    (measured 1.1 - 2.2 x faster there) and nowhere else; the products it then computes match the oracle."""
    dev = _gpu()
    w = wl.alexnet_fc6(L=3)
    h = B.cer_encode(w.W, w.codebook)
    assert [B.cer_matmul_path(h, L) for L in (1, 2, 3, 4, 8, 9, 32)] == [0, 2, 2, 2, 2, 1, 1]
    rows = np.sort(np.random.default_rng(5).choice(w.m, 256, replace=False))
    Wr = np.ascontiguousarray(w.W[rows])
    rng = np.random.default_rng(6)
    for L in (2, 3, 4, 7):
        X = rng.standard_normal((w.n, L)).astype(np.float32)
        # at an address that is only 4-byte aligned as well: the tile is then staged element by element
        for shift in (0, 1):
            buf = torch.zeros(w.n * L + 1, dtype=torch.float32, device=dev)
            Xd = buf[shift:shift + w.n * L]
            Xd.copy_(torch.from_numpy(X).reshape(-1))
            Yd = torch.full((w.m, L), float("nan"), dtype=torch.float32, device=dev)
            B.cer_matmul(h, Xd, Yd, L)
            torch.cuda.synchronize()
            Y = Yd.cpu().numpy().astype(np.float64)
            want, scale = oracle.dot_dense(Wr, X, threads=8), oracle.abs_dot_dense(Wr, X, threads=8)
            assert np.isfinite(Y).all()
            assert np.all(np.abs(Y[rows] - want) <= TOL * scale), f"L={L} shift={shift}"
    B.cer_free(h)
    small = wl.sweep_cell(16, 0.9, L=4)             # 0.4 million indices: the launch dominates, L2 gathers stay
    h = B.cer_encode(small.W, small.codebook)
    assert B.cer_matmul_path(h, 4) == 1
    B.cer_free(h)
    big = wl.vgg_fc6(L=4)                           # 25088 input rows do not fit in LDS
    h = B.cer_encode(big.W, big.codebook)
    assert B.cer_matmul_path(h, 4) == 1
    B.cer_free(h)
