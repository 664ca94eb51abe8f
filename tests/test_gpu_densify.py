"""GPU parity of the large-batch route of cer_matmul / cser_matmul that decodes the matrix into a dense
temporary and multiplies it on the fp32 matrix cores (cer_matmul_path = 3).  Preferred through cer_matmul_ex
for every kind of matrix and checked element by element against the oracle under the bound of every other
product, |Y - Y_oracle| <= 1e-5 * sum_c |W[r,c]| |X[c,l]|; then the automatic choice is checked on the
full-size workloads: it must take the route where the matrix is not sparse enough for the gathers to win
and leave it alone elsewhere."""
import pytest

from paper_1805_10692_amd import binding as B
from paper_1805_10692_amd import workloads as wl
from test_gpu_parity import full_check

pytestmark = pytest.mark.gpu

DENSE = B.MatmulOpts(path=B.CER_PATH_DENSE)


CASES = {
    "alexnet_s8_L32": lambda: wl.alexnet_fc6(L=32, scale=8),
    "vgg_s8_L64": lambda: wl.vgg_fc6(L=64, scale=8),
    "sweep_K256_p99": lambda: wl.sweep_cell(256, 0.99, L=16, scale=4),
    "sweep_K256_p50_L130": lambda: wl.sweep_cell(256, 0.5, L=130, scale=4),
    "conv_s4_L200": lambda: wl.conv3x3(L=200, scale=4),
    "conv_s4_dom_L200": lambda: wl.conv3x3(L=200, nonzero_dominant=True, scale=4),   # Omega[0] != 0: decoded, no column sums
    "conv_s4_dom_L7": lambda: wl.conv3x3(L=7, nonzero_dominant=True, scale=4),
    "u8_index_L12": lambda: wl.random_lowentropy(m=70, n=250, K=6, p_dom=0.6, L=12, seed=32),
    "u32_index_L5": lambda: wl.random_lowentropy(m=9, n=70001, K=8, p_dom=0.9, L=5, seed=34),
    "one_col": lambda: wl.random_lowentropy(m=300, n=1, K=3, p_dom=0.5, L=4, seed=37),
    "one_row_L2": lambda: wl.random_lowentropy(m=1, n=3000, K=16, p_dom=0.7, L=2, seed=36),
    "constant": lambda: wl.random_lowentropy(m=10, n=100, K=1, p_dom=1.0, L=3, seed=38),
    "many_groups_L8": lambda: wl.random_lowentropy(m=40, n=9000, K=700, p_dom=0.3, L=8, seed=40, ratio=0.995),
    "sparse_rows": lambda: wl.random_lowentropy(m=333, n=900, K=5, p_dom=0.998, L=6, seed=45),
}


@pytest.mark.parametrize("name", list(CASES))
def test_densified_all_elements(name):
    w = CASES[name]()
    h = B.cer_encode(w.W, w.codebook)
    assert B.cer_matmul_path_ex(h, w.L, DENSE) == 3
    assert B.cer_matmul_path_ex(h, 1, DENSE) in (0, 4)     # a single input vector never takes this route
    B.cer_free(h)
    full_check(w, opts=DENSE)


@pytest.mark.parametrize("L", [2, 3, 33, 65, 100, 129, 260])
def test_densified_ragged_batch_widths(L):
    full_check(wl.random_lowentropy(m=67, n=1501, K=48, p_dom=0.3, L=L, seed=500 + L, ratio=0.97), opts=DENSE, want_path=3)


def test_automatic_choice_on_full_size_workloads():
    picks = {}
    for name, w in (("conv3x3_L3136", wl.conv3x3()), ("alexnet_fc6_L32", wl.alexnet_fc6(L=32)),
                    ("vgg_fc6_L64", wl.vgg_fc6(L=64)), ("sweep_K256_p0.5_L16", wl.sweep_cell(256, 0.5))):
        h = B.cer_encode(w.W, w.codebook)
        picks[name] = (B.cer_matmul_path(h, w.L), B.cer_matmul_path(h, 1024), B.cer_matmul_path(h, 1))
        B.cer_free(h)
    # (workload's own batch, batch 1024, batch 1)
    assert picks["conv3x3_L3136"] == (3, 3, 0)          # 40 % of the elements indexed: dense wins at large batches
    assert picks["alexnet_fc6_L32"][0] == 1 and picks["alexnet_fc6_L32"][2] == 0
    assert picks["vgg_fc6_L64"] == (1, 1, 0)            # 5 % indexed: the gathers win at every batch
    assert picks["sweep_K256_p0.5_L16"] == (1, 3, 0)    # half of the elements indexed: small batch stays HBM-bound;
                                                        # batch 1 is always the stream kernel


@pytest.mark.parametrize("variant", [False, True], ids=["zero_dominant", "nonzero_dominant"])
def test_automatic_full_conv_batch3136_all_outputs(variant):
    """The convolution shape at its full size with the library's own choice of kernel (decode + dense)."""
    full_check(wl.conv3x3(nonzero_dominant=variant), want_path=B.CER_PATH_DENSE)


def test_trim_releases_cached_temporaries_and_products_go_on():
    """cer_trim gives the pooled temporaries back; the next products allocate again and stay correct."""
    import torch
    w = wl.conv3x3(L=200, scale=4)
    full_check(w, opts=DENSE)
    before = torch.cuda.mem_get_info()[0]
    B.cer_trim()
    after = torch.cuda.mem_get_info()[0]
    assert after >= before                      # nothing is taken by a trim; what was cached is free again
    full_check(w, opts=DENSE)
    B.cer_trim()
    B.cer_trim()                                # trimming an empty pool is fine
