"""GPU parity of the batched kernels that gather from L2 -- the default one (group values expanded per
position in LDS, then a plain multiply-add stream), the cursor variant that sums each group before its one
multiplication (CER_OPT_SUM_THEN_MULTIPLY), and the default one with ragged batch widths served one column per
lane instead of by 16-byte gathers (CER_OPT_ONE_COLUMN_PER_LANE) -- on every kind of matrix, against the oracle
under the usual bound.  A fourth run forces the 512-position value chunks meant for matrices of short rows
(CER_OPT_SHORT_CHUNKS) onto every matrix, so that long rows walk many chunks; a fifth keeps the default kernel away
from the rank table (CER_OPT_NO_RANK_TABLE).  The variants are selected per call
through cer_matmul_ex."""
import numpy as np
import pytest

from paper_1805_10692_amd import binding as B
from paper_1805_10692_amd import workloads as wl
from test_gpu_parity import full_check as _full_check

pytestmark = pytest.mark.gpu


VARIANTS = {
    "expand": 0,                                                    # the defaults
    "cursor": B.CER_OPT_SUM_THEN_MULTIPLY,
    "expand_one_column_per_lane": B.CER_OPT_ONE_COLUMN_PER_LANE,    # ragged widths without 16-byte gathers
    "expand_short_chunks": B.CER_OPT_SHORT_CHUNKS,                  # 512-position chunks on every matrix
    "expand_no_rank_table": B.CER_OPT_NO_RANK_TABLE,                # rows found through rowPtr -> OmegaPtr (the default kernel
                                                                    # takes handles of 2 - 64 values through their rank table)
}


@pytest.fixture(autouse=True, params=list(VARIANTS), ids=list(VARIANTS))
def variant(request):
    global _opts
    _opts = B.MatmulOpts(path=B.CER_PATH_GEMM, flags=VARIANTS[request.param])
    yield
    _opts = None


_opts = None


def full_check(w, fmts=("cer", "cser")):
    _full_check(w, fmts, opts=_opts, want_path=B.CER_PATH_GEMM)


CASES = {
    "alexnet_s8_L32": lambda: wl.alexnet_fc6(L=32, scale=8),
    "vgg_s8_L64": lambda: wl.vgg_fc6(L=64, scale=8),
    "sweep_K256_p99": lambda: wl.sweep_cell(256, 0.99, L=16, scale=4),       # CER: > 200 empty groups per row
    "sweep_K256_p50": lambda: wl.sweep_cell(256, 0.5, L=16, scale=4),        # the regime the kernel is meant for
    "sweep_K64_p50": lambda: wl.sweep_cell(64, 0.5, L=16, scale=4),
    "sweep_K2_p70": lambda: wl.sweep_cell(2, 0.7, L=16, scale=4),
    "conv_s4_L200": lambda: wl.conv3x3(L=200, scale=4),
    "conv_s4_dom_L200": lambda: wl.conv3x3(L=200, nonzero_dominant=True, scale=4),
    "conv_s4_dom_L7": lambda: wl.conv3x3(L=7, nonzero_dominant=True, scale=4),
    "u8_index_L12": lambda: wl.random_lowentropy(m=70, n=250, K=6, p_dom=0.6, L=12, seed=32),
    "u32_index_L5": lambda: wl.random_lowentropy(m=9, n=70001, K=8, p_dom=0.9, L=5, seed=34),    # several chunks per row
    "dense_rows_L8": lambda: wl.random_lowentropy(m=21, n=9000, K=5, p_dom=0.3, L=8, seed=47),    # 6300 indices per row
    "chunk_edge_L4": lambda: wl.random_lowentropy(m=13, n=4096, K=3, p_dom=0.5, L=4, seed=48),    # about 2048 per row
    "one_col": lambda: wl.random_lowentropy(m=300, n=1, K=3, p_dom=0.5, L=4, seed=37),
    "constant": lambda: wl.random_lowentropy(m=10, n=100, K=1, p_dom=1.0, L=3, seed=38),
    "many_groups_L8": lambda: wl.random_lowentropy(m=40, n=9000, K=700, p_dom=0.3, L=8, seed=40, ratio=0.995),
    "sparse_rows": lambda: wl.random_lowentropy(m=333, n=900, K=5, p_dom=0.998, L=6, seed=45),
}


@pytest.mark.parametrize("name", list(CASES))
def test_batched_variants_all_elements(name):
    full_check(CASES[name]())


@pytest.mark.parametrize("L", [2, 3, 4, 5, 6, 7, 9, 13, 16, 17, 31, 33, 34, 50, 64, 65, 100, 260])
def test_batched_variants_ragged_batch_widths(L):
    full_check(wl.random_lowentropy(m=67, n=1500, K=48, p_dom=0.3, L=L, seed=400 + L, ratio=0.97))


def test_batched_variants_hand_built_rows():
    """Groups of exactly 16 and 17 indices (the switch between one lane and the whole wave writing a group),
    a group that straddles a chunk boundary, rows without entries."""
    cb = np.array([0.0, 1.0, -2.0, 0.5, 3.0], np.float32)
    n = 6000
    W = np.zeros((12, n), np.float32)
    W[1, :16] = 1.0
    W[1, 100:117] = -2.0
    W[2, :2040] = 0.5                 # ends just before the chunk boundary ...
    W[2, 2040:2060] = 3.0             # ... and this group straddles it
    W[2, 3000:5100] = 1.0             # longer than a chunk
    W[5, n - 1] = 3.0
    W[7] = cb[np.random.default_rng(8).integers(0, 5, size=n)]
    W[11, ::3] = -2.0
    X = np.random.default_rng(9).standard_normal((n, 8)).astype(np.float32)

    class Case:
        pass
    w = Case()
    w.name, w.W, w.codebook, w.X, w.m, w.n, w.L = "hand-built", W, cb, X, 12, n, 8
    full_check(w)


@pytest.mark.parametrize("L", [36, 40, 50, 72, 99, 100, 130, 200])
def test_batched_variants_tile_widths_by_cache_lines(L):
    """Enough rows for the launcher to pick 64- and 128-column tiles when the rows of X are not whole
    cache lines (widths 40, 72, 100, 200: aligned; 50, 99, 130: served by 16-byte gathers from 4-byte
    aligned rows; 36: one partial tile)."""
    full_check(wl.random_lowentropy(m=1100, n=700, K=12, p_dom=0.8, L=L, seed=700 + L), fmts=("cer",))
