"""GPU parity of the batch-1 kernel that expands the group values per position (a variant callers can ask for
through cer_matmul_ex), run on every kind of matrix and checked element by element against the oracle under the
bound of every other product; then the automatic choice (always the stream kernel) on full-size cells of the
entropy sweep."""
import numpy as np
import pytest

from paper_1805_10692_amd import binding as B
from paper_1805_10692_amd import workloads as wl
from test_gpu_parity import full_check

pytestmark = pytest.mark.gpu

EXPAND = B.MatmulOpts(path=B.CER_PATH_GEMV_EXPAND)


CASES = {
    "c1": lambda: wl.config1(),
    "vgg_s8_L1": lambda: wl.vgg_fc6(L=1, scale=8),
    "alexnet_s8_L1": lambda: wl.alexnet_fc6(L=1, scale=8),
    "sweep_K256_p50_L1": lambda: wl.sweep_cell(256, 0.5, L=1, scale=4),
    "sweep_K256_p99_L1": lambda: wl.sweep_cell(256, 0.99, L=1, scale=4),      # CER: > 200 empty groups per row
    "sweep_K64_p90_L1": lambda: wl.sweep_cell(64, 0.9, L=1, scale=4),
    "sweep_K2_p70_L1": lambda: wl.sweep_cell(2, 0.7, L=1, scale=4),
    "conv_s4_dom_L1": lambda: wl.conv3x3(L=1, nonzero_dominant=True, scale=4),  # Omega[0] != 0
    "u8_index": lambda: wl.random_lowentropy(m=70, n=250, K=6, p_dom=0.6, L=1, seed=31),
    "u32_index_L1": lambda: wl.random_lowentropy(m=9, n=70001, K=8, p_dom=0.9, L=1, seed=33),   # X too big for LDS: stream kernel
    "chunk_edges": lambda: wl.random_lowentropy(m=33, n=5000, K=5, p_dom=0.38, L=1, seed=51),    # about 3100 indices per row: 4 chunks
    "exactly_one_chunk": lambda: wl.random_lowentropy(m=20, n=2048, K=3, p_dom=0.5, L=1, seed=52),
    "one_row": lambda: wl.random_lowentropy(m=1, n=3000, K=16, p_dom=0.7, L=1, seed=36),
    "one_col": lambda: wl.random_lowentropy(m=300, n=1, K=3, p_dom=0.5, L=1, seed=37),
    "constant": lambda: wl.random_lowentropy(m=10, n=100, K=1, p_dom=1.0, L=1, seed=38),
    "many_groups": lambda: wl.random_lowentropy(m=40, n=9000, K=700, p_dom=0.3, L=1, seed=39, ratio=0.995),
    "sparse_rows": lambda: wl.random_lowentropy(m=333, n=900, K=5, p_dom=0.998, L=1, seed=45),
    "unaligned_n": lambda: wl.random_lowentropy(m=50, n=1001, K=40, p_dom=0.2, L=1, seed=53, ratio=0.98),
}


@pytest.mark.parametrize("name", list(CASES))
def test_gemv_expand_all_elements(name):
    # X too big for LDS: the preference cannot be met and the stream kernel runs
    full_check(CASES[name](), opts=EXPAND, want_path=0 if name == "u32_index_L1" else 4)


def test_gemv_expand_full_size_vgg_fc6():
    full_check(wl.vgg_fc6(L=1), opts=EXPAND, want_path=4)


@pytest.mark.parametrize("K,p0,path", [(256, 0.5, 0), (256, 0.9, 0), (64, 0.5, 0), (16, 0.5, 0)])
def test_automatic_choice_full_sweep_cells(K, p0, path):
    w = wl.sweep_cell(K, p0, L=1)
    h = B.cer_encode(w.W, w.codebook)
    assert B.cer_matmul_path(h, 1) == path
    B.cer_free(h)
    full_check(w)


def test_automatic_choice_keeps_the_layer_shapes_on_the_stream_kernel():
    for w in (wl.vgg_fc6(L=1), wl.alexnet_fc6(L=1)):
        h = B.cer_encode(w.W, w.codebook)
        assert B.cer_matmul_path(h, 1) == 0
        B.cer_free(h)


def test_short_row_variant_with_a_few_long_rows():
    """The variant for matrices of short rows (chosen by the average row) must still walk a long row chunk by
    chunk: most rows hold about 90 indices, three hold 1300 - 2900, one group straddles a chunk boundary."""
    rng = np.random.default_rng(61)
    cb = np.array([0.0, 0.5, -1.0, 2.0, 0.25, -0.125], np.float32)
    W = cb[rng.choice(6, size=(60, 3000), p=[0.97, 0.01, 0.008, 0.006, 0.004, 0.002])].astype(np.float32)
    W[7] = cb[rng.integers(0, 6, size=3000)]            # about 2500 indices in five groups
    W[20, :1300] = 0.5                                   # one group of 1300: crosses two chunk boundaries
    W[41] = cb[rng.choice(6, size=3000, p=[0.04, 0.3, 0.3, 0.2, 0.1, 0.06])]
    X = rng.standard_normal((3000, 1)).astype(np.float32)

    class Case:
        pass
    w = Case()
    w.name, w.W, w.codebook, w.X, w.m, w.n, w.L = "short rows with long ones", W, cb, X, 60, 3000, 1
    full_check(w, opts=EXPAND, want_path=4)
