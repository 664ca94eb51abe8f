"""Op-count / storage / energy analytics (host side): the oracle counts by executing Algorithms 1-4
with counters; it is pinned to the hand counts the paper gives for its example row; the library's
closed-form counts must equal the oracle's, and its energy must equal Eq. (10) / Eq. (12) priced
with Table I."""
import numpy as np
import pytest

import oracle
from oracle import cost_model as cm
from paper_1805_10692_amd import binding as B
from paper_1805_10692_amd import workloads as wl

KEYS = ("read_weight", "read_omega", "read_colI", "read_omegaPtr", "read_rowPtr", "read_omegaI", "read_input",
        "mul", "add", "write")


def test_paper_example_row_counts(example):
    """Section III-B: second row of M: dense 24 loads + 12 mul + 11 add + 1 write = 48; CSR 20 + 6 + 5 + 1 = 32;
    CER 17 loads (2 rowPtr, 2 OmegaPtr, 1 Omega, 6 colI, 6 input) + 1 mul + 5 add + 1 write = 24."""
    row = example["M"][1:2].astype(np.float32)
    d = cm.count_dense(row, "example")
    assert (d["read_weight"] + d["read_input"], d["mul"], d["add"], d["write"]) == (24, 12, 11, 1)
    assert cm.total_ops(d) == int(example["row1_ops_dense"][0]) == 48
    c = cm.count_csr(oracle.csr_encode(row), "example")
    assert (c["read_rowPtr"], c["read_weight"], c["read_colI"], c["read_input"], c["mul"], c["add"], c["write"]) == (2, 6, 6, 6, 6, 5, 1)
    assert cm.total_ops(c) == int(example["row1_ops_csr"][0]) == 32
    e = cm.count_cer(oracle.encode(row, np.array([0, 4], np.float32), "cer"), "example")
    assert (e["read_rowPtr"], e["read_omegaPtr"], e["read_omega"], e["read_colI"], e["read_input"]) == (2, 2, 1, 6, 6)
    assert (e["mul"], e["add"], e["write"]) == (1, 5, 1)
    assert cm.total_ops(e) == int(example["row1_ops_cer"][0]) == 24


def test_table_one_lookup():
    # the paper's own illustration: a 16-bit index in a 30 KB array costs 5.0 pJ to read
    assert cm.rw_cost(16, 30 * 1024) == 5.0
    assert cm.rw_cost(32, 2 * 1024 * 1024) == 1000.0 and cm.rw_cost(8, 100) == 1.25


CASES = [dict(m=23, n=130, K=8, p_dom=0.8, L=1, seed=51), dict(m=12, n=300, K=32, p_dom=0.95, L=1, seed=52),
         dict(m=9, n=64, K=4, p_dom=0.4, L=1, seed=53, dominant=0)]


@pytest.mark.parametrize("case", CASES, ids=lambda c: f"{c['m']}x{c['n']}K{c['K']}")
@pytest.mark.parametrize("how,conv", [("theorem", B.CER_COUNT_THEOREM), ("example", B.CER_COUNT_EXAMPLE)])
def test_library_counts_equal_instrumented_oracle(case, how, conv):
    w = wl.random_lowentropy(**case)
    for fmt, enc in (("cer", B.cer_encode), ("cser", B.cser_encode)):
        A = oracle.encode(w.W, w.codebook, fmt)
        want = cm.count_cer(A, how)
        got = B.cer_cost_model(enc(w.W, w.codebook), conv)
        assert {k: got[k] for k in KEYS} == {k: want.get(k, 0) for k in KEYS}, fmt
        assert got["storage_bits"] == oracle.storage_bits(A)
        bits = oracle.array_bits(A)
        arrays = {"omega": (32, 4 * A.K), "colI": (bits["colI"], A.nnz * bits["colI"] / 8),
                  "omegaPtr": (bits["omegaPtr"], len(A.omegaPtr) * bits["omegaPtr"] / 8),
                  "rowPtr": (bits["rowPtr"], len(A.rowPtr) * bits["rowPtr"] / 8)}
        if A.omegaI is not None:
            arrays["omegaI"] = (bits["omegaI"], len(A.omegaI) * bits["omegaI"] / 8)
        assert got["energy_pj"] == pytest.approx(cm.energy_pj(want, w.m, w.n, arrays), rel=1e-12)
    C = oracle.csr_encode(w.W)
    want = cm.count_csr(C, how)
    got = B.csr_cost_model(B.csr_encode(w.W), conv)
    assert {k: got[k] for k in KEYS} == {k: want.get(k, 0) for k in KEYS}
    want = cm.count_dense(w.W, how)
    got = B.dense_cost_model(w.m, w.n, conv)
    assert {k: got[k] for k in KEYS} == {k: want.get(k, 0) for k in KEYS}
    assert got["energy_pj"] == pytest.approx(cm.energy_pj(want, w.m, w.n, {"weight": (32, 4 * w.m * w.n)}), rel=1e-12)


def test_energy_equals_theorem_formulas():
    """Eq. (10) and Eq. (12) with c_oth = 0, each read priced for the array it touches:
    E/N = (1-p0)(sigma + gamma_a + gamma_colI) + k_bar/n (gamma_OmegaPtr + gamma_Omega + mu [+ gamma_OmegaI])
          + k_tilde/n gamma_OmegaPtr + 1/n (gamma_rowPtr + delta)."""
    w = wl.random_lowentropy(m=40, n=700, K=16, p_dom=0.9, L=1, seed=54)
    N = w.m * w.n
    for fmt, enc in (("cer", B.cer_encode), ("cser", B.cser_encode)):
        A = oracle.encode(w.W, w.codebook, fmt)
        st = oracle.stats(A)
        bits = oracle.array_bits(A)
        g = lambda name, length: cm.rw_cost(bits[name], length * bits[name] / 8)
        sigma, mu = 0.9, 3.7
        per_elem = (1 - st["p0"]) * (sigma + cm.rw_cost(32, 4 * w.n) + g("colI", A.nnz))
        per_group = g("omegaPtr", len(A.omegaPtr)) + cm.rw_cost(32, 4 * A.K) + mu
        if fmt == "cser":
            per_group += g("omegaI", len(A.omegaI))
        per_elem += st["k_bar"] / w.n * per_group + st["k_tilde"] / w.n * g("omegaPtr", len(A.omegaPtr))
        per_elem += (g("rowPtr", len(A.rowPtr)) + cm.rw_cost(32, 4 * w.m)) / w.n
        got = B.cer_cost_model(enc(w.W, w.codebook), B.CER_COUNT_THEOREM)
        assert got["energy_pj"] / N == pytest.approx(per_elem, rel=1e-12)


def test_model_favours_cer_on_low_entropy_and_csr_on_spike_and_slab():
    """Section IV-D / Fig. 4 trend, on the model: geometric tail (low entropy) -> CER cheaper than CSR;
    uniform tail over many values at modest sparsity -> dense or CSR cheaper than CER."""
    lo = wl.random_lowentropy(m=64, n=2000, K=16, p_dom=0.9, L=1, seed=55, ratio=0.5)
    e_cer = B.cer_cost_model(B.cer_encode(lo.W, lo.codebook))["energy_pj"]
    e_csr = B.csr_cost_model(B.csr_encode(lo.W))["energy_pj"]
    e_den = B.dense_cost_model(lo.m, lo.n)["energy_pj"]
    assert e_cer < e_csr < e_den
    ss = wl.sweep_cell(256, 0.5, L=1, scale=16)
    s_cer = B.cer_cost_model(B.cer_encode(ss.W, ss.codebook))
    s_csr = B.csr_cost_model(B.csr_encode(ss.W))
    assert s_csr["storage_bits"] < B.dense_cost_model(ss.m, ss.n)["storage_bits"] * 1.6
    assert s_cer["mul"] > 0.5 * s_csr["mul"]      # hardly any sharing left: almost one multiply per element pair
