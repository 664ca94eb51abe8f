"""GPU parity of the batch-1 stream kernel on matrices of few rows, where a row is shared by 4 or 8 waves of a
workgroup (each takes a contiguous share of the row's windows, the partial sums meet in LDS): every element against
the oracle's group-sum product (Algorithm 3 / 4), in both formats, with the rows shared (the library's choice) and
whole (CER_OPT_ROWS_WHOLE), which must agree with each other to rounding as well."""
import numpy as np
import pytest

import oracle
from paper_1805_10692_amd import binding as B
from paper_1805_10692_amd import workloads as wl
from test_gpu_parity import check, full_check, run_matmul

pytestmark = pytest.mark.gpu

STREAM = B.MatmulOpts(path=B.CER_PATH_GEMV)
WHOLE = B.MatmulOpts(path=B.CER_PATH_GEMV, flags=B.CER_OPT_ROWS_WHOLE)
# the same kernel finding its group boundaries through rowPtr / OmegaPtr instead of the handle's rank table
NO_TABLE = B.MatmulOpts(path=B.CER_PATH_GEMV, flags=B.CER_OPT_NO_RANK_TABLE)
NO_TABLE_WHOLE = B.MatmulOpts(path=B.CER_PATH_GEMV, flags=B.CER_OPT_NO_RANK_TABLE | B.CER_OPT_ROWS_WHOLE)

CASES = {
    # 16-bit indices: windows of 512 positions
    "one_row_8_windows": lambda: wl.random_lowentropy(m=1, n=20000, K=16, p_dom=0.8, L=1, seed=71),
    "seven_rows_dom": lambda: wl.random_lowentropy(m=7, n=5000, K=5, p_dom=0.4, L=1, seed=72, dominant=4),  # Omega[0] != 0
    "two_windows": lambda: wl.random_lowentropy(m=100, n=1500, K=8, p_dom=0.4, L=1, seed=73),
    "share_ends_on_a_window_edge": lambda: wl.random_lowentropy(m=64, n=4096, K=2, p_dom=0.5, L=1, seed=74),
    "more_waves_than_windows": lambda: wl.random_lowentropy(m=20, n=2500, K=6, p_dom=0.55, L=1, seed=75),
    "many_groups_general_list": lambda: wl.random_lowentropy(m=40, n=9000, K=700, p_dom=0.3, L=1, seed=76, ratio=0.995),
    "eight_rows_per_unit": lambda: wl.random_lowentropy(m=2000, n=3000, K=16, p_dom=0.5, L=1, seed=77),
    "four_rows_per_unit": lambda: wl.random_lowentropy(m=1000, n=6000, K=16, p_dom=0.6, L=1, seed=78),
    "unequal_rows": lambda: _unequal(),
    "lds_edge": lambda: wl.random_lowentropy(m=33, n=38000, K=8, p_dom=0.8, L=1, seed=79),
    # 8-bit indices: windows of 1024 positions, so only a row of 256 columns that is nearly all indexed stays whole
    "u8_index": lambda: wl.random_lowentropy(m=50, n=256, K=6, p_dom=0.05, L=1, seed=80),
}


def _unequal():
    """Rows from empty to completely indexed: shares that are empty, shares behind the row's end."""
    rng = np.random.default_rng(81)
    cb = np.array([0.0, 0.5, -1.0, 2.0, 0.25, -0.125], np.float32)
    W = cb[rng.choice(6, size=(60, 6000), p=[0.6, 0.1, 0.1, 0.1, 0.05, 0.05])].astype(np.float32)
    W[3] = 0.0
    W[4, 1:] = 0.0
    W[5] = cb[rng.integers(1, 6, size=6000)]
    W[6, :700] = 0.0
    W[7, 511:] = 0.0
    W[8, 513:] = 0.0
    X = rng.standard_normal((6000, 1)).astype(np.float32)

    class Case:
        pass
    w = Case()
    w.name, w.W, w.codebook, w.X, w.m, w.n, w.L = "unequal rows", W, cb, X, 60, 6000, 1
    return w


@pytest.mark.parametrize("name", list(CASES))
def test_shared_rows_all_elements(name):
    w = CASES[name]()
    full_check(w, opts=STREAM, want_path=0)
    full_check(w, opts=WHOLE, want_path=0)
    full_check(w, opts=NO_TABLE, want_path=0)
    full_check(w, opts=NO_TABLE_WHOLE, want_path=0)
    scale = oracle.abs_dot_dense(w.W, w.X, threads=8)
    for fmt in ("cer", "cser"):
        a = run_matmul(fmt, w.W, w.codebook, w.X, opts=STREAM)
        b = run_matmul(fmt, w.W, w.codebook, w.X, opts=WHOLE)
        check(a, b.astype(np.float64), 2.0 * scale, f"{name}/{fmt}: shared against whole rows")


@pytest.mark.parametrize("dom", [False, True])
def test_conv3x3_batch1_full_size(dom):
    full_check(wl.conv3x3(L=1, nonzero_dominant=dom))
    full_check(wl.conv3x3(L=1, nonzero_dominant=dom), opts=NO_TABLE)
