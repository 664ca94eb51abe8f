"""GPU parity: the HIP path, called through the C ABI binding, against the CPU oracle on the same
seeded inputs.  Integer arrays were already compared bit for bit on the host; here Y is compared
element by element under the bound  |Y - Y_oracle| <= 1e-5 * sum_c |W[r,c]| |X[c,l]|  (fp32 sums in
another order than the oracle's fp64 loop)."""
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


def run_matmul(fmt, W, codebook, X, stream=None, opts=None, want_path=None):
    """One product through the C ABI.  opts: a MatmulOpts for cer_matmul_ex (None: cer_matmul / cser_matmul);
    want_path: the kernel that cer_matmul_path_ex must announce for this call."""
    dev = _gpu()
    h = (B.cer_encode if fmt == "cer" else B.cser_encode)(W, codebook)
    Xd = torch.from_numpy(np.ascontiguousarray(X)).to(dev)
    Yd = torch.full((W.shape[0], X.shape[1]), float("nan"), dtype=torch.float32, device=dev)
    if want_path is not None and W.size:
        assert B.cer_matmul_path_ex(h, X.shape[1], opts) == want_path
    if opts is None:
        (B.cer_matmul if fmt == "cer" else B.cser_matmul)(h, Xd, Yd, X.shape[1], stream)
    else:
        B.cer_matmul_ex(h, Xd, Yd, X.shape[1], stream, opts)
    torch.cuda.synchronize()
    Y = Yd.cpu().numpy()
    B.cer_free(h)
    return Y


def check(Y, want, scale, what):
    assert Y.shape == want.shape, what
    assert np.isfinite(Y).all(), f"{what}: non-finite output (unwritten element?)"
    err = np.abs(Y.astype(np.float64) - want)
    bad = err > TOL * scale
    assert not bad.any(), (f"{what}: {int(bad.sum())} elements beyond tolerance; worst ratio "
                           f"{float((err / np.maximum(scale, 1e-300)).max()):.3e} at {np.argwhere(bad)[:4].tolist()}")


def full_check(w, fmts=("cer", "cser"), opts=None, want_path=None):
    """Every element of Y against the oracle's group-sum product (Algorithm 3 / 4 in fp64) of its own encoding."""
    print(f"case {w.name} m={w.m} n={w.n} L={w.L}", flush=True)
    scale = oracle.abs_dot_dense(w.W, w.X, threads=8)
    for fmt in fmts:
        A = oracle.encode(w.W, w.codebook, fmt)
        want = oracle.dot(A, w.X, threads=8)
        Y = run_matmul(fmt, w.W, w.codebook, w.X, opts=opts, want_path=want_path)
        check(Y, want, scale, f"{w.name}/{fmt}")


SMALL = {
    "c1": lambda: wl.config1(),
    "alexnet_s8_L32": lambda: wl.alexnet_fc6(L=32, scale=8),
    "vgg_s8_L1": lambda: wl.vgg_fc6(L=1, scale=8),
    "vgg_s8_L64": lambda: wl.vgg_fc6(L=64, scale=8),
    "sweep_K256_p99": lambda: wl.sweep_cell(256, 0.99, L=16, scale=4),
    "sweep_K256_p50": lambda: wl.sweep_cell(256, 0.5, L=16, scale=4),
    "sweep_K2_p70": lambda: wl.sweep_cell(2, 0.7, L=16, scale=4),
    "sweep_K64_p90_L1": lambda: wl.sweep_cell(64, 0.9, L=1, scale=4),
    "conv_s4_L200": lambda: wl.conv3x3(L=200, scale=4),
    "conv_s4_dom_L200": lambda: wl.conv3x3(L=200, nonzero_dominant=True, scale=4),
    "conv_s4_dom_L1": lambda: wl.conv3x3(L=1, nonzero_dominant=True, scale=4),
    "conv_s4_dom_L7": lambda: wl.conv3x3(L=7, nonzero_dominant=True, scale=4),
    "u8_index": lambda: wl.random_lowentropy(m=70, n=250, K=6, p_dom=0.6, L=1, seed=31),
    "u8_index_L12": lambda: wl.random_lowentropy(m=70, n=250, K=6, p_dom=0.6, L=12, seed=32),
    "u32_index_L1": lambda: wl.random_lowentropy(m=9, n=70001, K=8, p_dom=0.9, L=1, seed=33),   # X too big for LDS
    "u32_index_L5": lambda: wl.random_lowentropy(m=9, n=70001, K=8, p_dom=0.9, L=5, seed=34),
    "lds_edge": lambda: wl.random_lowentropy(m=33, n=38000, K=8, p_dom=0.95, L=1, seed=35),
    "one_row": lambda: wl.random_lowentropy(m=1, n=3000, K=16, p_dom=0.7, L=1, seed=36),
    "one_col": lambda: wl.random_lowentropy(m=300, n=1, K=3, p_dom=0.5, L=4, seed=37),
    "constant": lambda: wl.random_lowentropy(m=10, n=100, K=1, p_dom=1.0, L=3, seed=38),
    "many_groups": lambda: wl.random_lowentropy(m=40, n=9000, K=700, p_dom=0.3, L=1, seed=39, ratio=0.995),
    "many_groups_L8": lambda: wl.random_lowentropy(m=40, n=9000, K=700, p_dom=0.3, L=8, seed=40, ratio=0.995),
}


@pytest.mark.parametrize("name", list(SMALL))
def test_small_cases_all_elements(name):
    full_check(SMALL[name]())


NO_RANK_TABLE = B.MatmulOpts(flags=B.CER_OPT_NO_RANK_TABLE)


@pytest.mark.parametrize("name", [k for k in SMALL if SMALL[k]().L == 1])
def test_small_batch1_cases_without_rank_table(name):
    """Handles of at most 64 values carry a rank table for the batch-1 kernel; here the same products with the group
    boundaries read through rowPtr and OmegaPtr."""
    full_check(SMALL[name](), opts=NO_RANK_TABLE)


@pytest.mark.parametrize("L", [2, 3, 4, 5, 16, 17, 33, 63, 64, 65, 100, 256, 260, 516])
def test_ragged_batch_widths(L):
    full_check(wl.random_lowentropy(m=67, n=1500, K=16, p_dom=0.8, L=L, seed=100 + L))


def test_rows_without_entries_and_unaligned_pointers():
    w = wl.random_lowentropy(m=50, n=777, K=8, p_dom=0.9, L=4, seed=41)
    w.W[::3] = w.W[0, 0] * 0 + w.codebook[4]            # every third row holds only the dominant value
    dev = _gpu()
    scale = oracle.abs_dot_dense(w.W, w.X)
    for fmt in ("cer", "cser"):
        want = oracle.dot(oracle.encode(w.W, w.codebook, fmt), w.X)
        check(run_matmul(fmt, w.W, w.codebook, w.X), want, scale, f"empty rows/{fmt}")
    # X and Y at addresses that are only 4-byte aligned (vector paths must not be taken)
    for L in (1, 4, 7, 12, 40):
        X = wl.sample_X(np.random.Generator(np.random.PCG64(900 + L)), w.n, L)
        h = B.cer_encode(w.W, w.codebook)
        Xbuf = torch.zeros(X.size + 1, dtype=torch.float32, device=dev)
        Ybuf = torch.full((w.m * L + 1,), float("nan"), dtype=torch.float32, device=dev)
        Xbuf[1:] = torch.from_numpy(X.reshape(-1)).to(dev)
        B.cer_matmul(h, Xbuf.data_ptr() + 4, Ybuf.data_ptr() + 4, L)
        torch.cuda.synchronize()
        want = oracle.dot(oracle.encode(w.W, w.codebook, "cer"), X)
        check(Ybuf[1:].cpu().numpy().reshape(w.m, L), want, oracle.abs_dot_dense(w.W, X), f"unaligned L={L}")
        assert torch.isnan(Ybuf[0])
        B.cer_free(h)


def test_worked_example_on_the_gpu(example):
    M = example["M"].astype(np.float32)
    X = np.arange(1, 25, dtype=np.float32).reshape(12, 2)
    want = example["M"] @ X.astype(np.float64)
    for fmt in ("cer", "cser"):
        Y = run_matmul(fmt, M, np.array([0, 2, 3, 4], np.float32), X)
        assert np.array_equal(Y.astype(np.float64), want)       # small integers: exact in fp32


def test_side_stream_and_handle_reuse():
    dev = _gpu()
    w = wl.vgg_fc6(L=1, scale=16)
    A = oracle.encode(w.W, w.codebook, "cer")
    h = B.cer_encode(w.W, w.codebook)
    h2 = B.cer_clone_device(h)
    s = torch.cuda.Stream()
    outs = []
    for k in range(3):
        X = wl.sample_X(np.random.default_rng(k), w.n, 1)
        Xd = torch.from_numpy(X).to(dev)
        Yd = torch.empty((w.m, 1), dtype=torch.float32, device=dev)
        s.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(s):
            B.cer_matmul(h if k % 2 == 0 else h2, Xd, Yd, 1)        # picks up the current (side) stream
        outs.append((X, Xd, Yd))
    s.synchronize()
    for X, _, Yd in outs:
        check(Yd.cpu().numpy(), oracle.dot(A, X), oracle.abs_dot_dense(w.W, X), "side stream")
    assert B.cer_device_bytes(h) == A.nnz * 2 + (A.G + 1) * 4 + (A.m + 1) * 4 + A.K * 4
    B.cer_free(h)
    B.cer_free(h2)


@pytest.mark.parametrize("shape", [(64, 256, 1), (67, 1500, 1), (130, 999, 1), (67, 1500, 5), (200, 700, 64), (129, 515, 100),
                                   (256, 4096, 64), (300, 1000, 33), (130, 516, 200), (512, 2048, 16), (40, 37, 3), (1, 5, 2)])
def test_dense_baseline(shape):
    dev = _gpu()
    m, n, L = shape
    w = wl.random_lowentropy(m=m, n=n, K=16, p_dom=0.3, L=L, seed=77)
    Wd, Xd = torch.from_numpy(w.W).to(dev), torch.from_numpy(w.X).to(dev)
    Yd = torch.full((m, L), float("nan"), dtype=torch.float32, device=dev)
    B.dense_matmul(Wd, Xd, Yd, m, n, L)
    torch.cuda.synchronize()
    check(Yd.cpu().numpy(), oracle.dot_dense(w.W, w.X), oracle.abs_dot_dense(w.W, w.X), f"dense {shape}")


def test_stream_copy_probe():
    dev = _gpu()
    src = torch.arange(1 << 20, dtype=torch.float32, device=dev)
    dst = torch.zeros_like(src)
    B.cer_stream_copy(dst, src, src.numel() * 4)
    torch.cuda.synchronize()
    assert torch.equal(dst, src)


# ------------------------------------------------------------------ full sizes of the named workloads

# Every output element of every benchmark configuration at its full size: the oracle's group-sum product costs
# nnz.L additions (a few seconds on the host's cores even for the convolution shape), so nothing is sampled.

def test_full_vgg_fc6_gemv_all_outputs():
    full_check(wl.vgg_fc6(L=1))
    full_check(wl.vgg_fc6(L=1), opts=NO_RANK_TABLE)


def test_full_vgg_fc6_batch64_all_outputs():
    full_check(wl.vgg_fc6(L=64))


def test_full_alexnet_fc6_batch32_all_outputs():
    full_check(wl.alexnet_fc6(L=32))


@pytest.mark.parametrize("p0", wl.SWEEP_P0)
@pytest.mark.parametrize("K", wl.SWEEP_K)
def test_full_sweep_cells_all_outputs(K, p0):
    full_check(wl.sweep_cell(K, p0))


@pytest.mark.parametrize("variant", [False, True], ids=["zero_dominant", "nonzero_dominant"])
def test_full_conv_batch3136_gather_kernel_all_outputs(variant):
    """The convolution shape on the gather kernel (Algorithm 3 / 4); the library's own choice for this shape, the
    decode + dense route, is checked at full size in test_gpu_densify.py."""
    full_check(wl.conv3x3(nonzero_dominant=variant), opts=B.MatmulOpts(path=B.CER_PATH_GEMM), want_path=B.CER_PATH_GEMM)


# ------------------------------------------------------------------ CSR comparator (Algorithm 2)

CSR_CASES = {
    "c1": lambda: wl.config1(),
    "vgg_s8_L1": lambda: wl.vgg_fc6(L=1, scale=8),
    "vgg_s8_L64": lambda: wl.vgg_fc6(L=64, scale=8),
    "alexnet_s8_L32": lambda: wl.alexnet_fc6(L=32, scale=8),
    "conv_s4_dom_L7": lambda: wl.conv3x3(L=7, nonzero_dominant=True, scale=4),
    "sweep_K256_p50": lambda: wl.sweep_cell(256, 0.5, L=16, scale=4),
    "u8_index_L12": lambda: wl.random_lowentropy(m=70, n=250, K=6, p_dom=0.6, L=12, seed=32),
    "u32_index_L1": lambda: wl.random_lowentropy(m=9, n=70001, K=8, p_dom=0.9, L=1, seed=33),
    "long_rows_L1": lambda: wl.random_lowentropy(m=20, n=9000, K=8, p_dom=0.3, L=1, seed=42),
    "ragged_L100": lambda: wl.random_lowentropy(m=67, n=1500, K=16, p_dom=0.8, L=100, seed=43),
    "all_zero": lambda: wl.random_lowentropy(m=10, n=100, K=1, p_dom=1.0, L=3, seed=38),
}


@pytest.mark.parametrize("name", list(CSR_CASES))
def test_csr_matmul(name):
    dev = _gpu()
    w = CSR_CASES[name]()
    print(f"csr case {w.name}", flush=True)
    h = B.csr_encode(w.W)
    Xd = torch.from_numpy(w.X).to(dev)
    Yd = torch.full((w.m, w.L), float("nan"), dtype=torch.float32, device=dev)
    B.csr_matmul(h, Xd, Yd, w.L)
    torch.cuda.synchronize()
    want = oracle.dot_csr(oracle.csr_encode(w.W), w.X)
    check(Yd.cpu().numpy(), want, oracle.abs_dot_dense(w.W, w.X), f"csr {w.name}")
    B.csr_free(h)


@pytest.mark.parametrize("shape", [(5, 0, 1), (5, 0, 3), (0, 7, 1), (0, 7, 4), (3, 2, 1), (3, 2, 70000)])
def test_degenerate_shapes(shape):
    """No columns (Y = 0), no rows (nothing written), and a batch far wider than the matrix."""
    m, n, L = shape
    dev = _gpu()
    cb = np.array([0.0, 1.0], np.float32)
    W = np.zeros((m, n), np.float32)
    if m and n:
        W[0, 1] = 1.0
    X = torch.ones((max(n, 1), L), dtype=torch.float32, device=dev)   # a valid pointer even when n = 0
    for fmt in ("cer", "cser"):
        h = (B.cer_encode if fmt == "cer" else B.cser_encode)(W, cb)
        Y = torch.full((max(m, 1), L), float("nan"), dtype=torch.float32, device=dev)
        (B.cer_matmul if fmt == "cer" else B.cser_matmul)(h, X, Y, L)
        torch.cuda.synchronize()
        B.cer_free(h)
        if m:
            want = W @ np.ones((n, L), np.float32) if n else np.zeros((m, L), np.float32)
            assert np.array_equal(Y[:m].cpu().numpy(), want)
        else:
            assert torch.isnan(Y).all()


def test_graph_capture_and_replay():
    """A product with a zero most frequent value launches kernels only (no allocation, no memset), so a caller
    can record it into a HIP graph.  Every replay, with eager work and synchronisation in between and new
    inputs in the same buffers, must equal the eager result."""
    dev = _gpu()
    cases = [wl.vgg_fc6(L=1, scale=8), wl.alexnet_fc6(L=32, scale=8)]
    for w in cases:
        h = B.cer_encode(w.W, w.codebook)
        Xd = torch.from_numpy(w.X).to(dev)
        Yg = torch.zeros((w.m, w.L), dtype=torch.float32, device=dev)
        Ye = torch.zeros_like(Yg)
        B.cer_matmul(h, Xd, Ye, w.L)            # warm-up outside the capture (one-time kernel attributes)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            B.cer_matmul(h, Xd, Yg, w.L)        # recorded on the capture stream, which is the current stream here
        rng = np.random.default_rng(3)
        for rep in range(4):
            Xd.copy_(torch.from_numpy(rng.standard_normal(w.X.shape).astype(np.float32)))
            Yg.fill_(float("nan"))
            torch.cuda.synchronize()
            g.replay()
            B.cer_matmul(h, Xd, Ye, w.L)        # eager, same inputs
            torch.cuda.synchronize()
            assert torch.equal(Yg, Ye), f"{w.name}: replay {rep} differs from the eager product"
            scale = oracle.abs_dot_dense(w.W, Xd.cpu().numpy(), threads=8)
            want = oracle.dot_dense(w.W, Xd.cpu().numpy(), threads=8)
            check(Yg.cpu().numpy(), want, scale, f"{w.name} replay {rep}")
        B.cer_free(h)


@pytest.mark.parametrize("L", [1, 4, 8, 32])
def test_unaligned_device_pointers(L):
    """X and Y that start 4 bytes into an allocation: the 16-byte load / store paths must not be taken."""
    dev = _gpu()
    w = wl.random_lowentropy(m=77, n=1203, K=12, p_dom=0.8, L=L, seed=300 + L)
    scale = oracle.abs_dot_dense(w.W, w.X, threads=4)
    want = oracle.dot_dense(w.W, w.X, threads=4)
    xbuf = torch.zeros(w.n * L + 1, dtype=torch.float32, device=dev)
    ybuf = torch.full((w.m * L + 1,), float("nan"), dtype=torch.float32, device=dev)
    Xd, Yd = xbuf[1:], ybuf[1:]
    assert Xd.data_ptr() % 16 == 4 and Yd.data_ptr() % 16 == 4
    Xd.copy_(torch.from_numpy(w.X.reshape(-1)))
    for fmt in ("cer", "cser"):
        h = (B.cer_encode if fmt == "cer" else B.cser_encode)(w.W, w.codebook)
        for path in (B.CER_PATH_GEMM, B.CER_PATH_XTILE):      # for L = 1 neither applies: the batch-1 kernel runs
            Yd.fill_(float("nan"))
            B.cer_matmul_ex(h, Xd, Yd, L, None, B.MatmulOpts(path=path))
            torch.cuda.synchronize()
            check(Yd.cpu().numpy().reshape(w.m, L), want, scale, f"unaligned {fmt} L={L} path={path}")
        B.cer_free(h)
    Wd = torch.from_numpy(w.W).to(dev)
    Yd.fill_(float("nan"))
    B.dense_matmul(Wd, Xd, Yd, w.m, w.n, L)
    torch.cuda.synchronize()
    check(Yd.cpu().numpy().reshape(w.m, L), want, scale, f"unaligned dense L={L}")


def test_dominant_value_term_error_scale():
    """Appendix A-A1 adds Omega[0].sum_i x_i and subtracts Omega[0] inside every group's weight, so with a non-zero
    most frequent value the rounding error scales with |Omega[0]|.sum|x| as well.  A matrix of one column whose most
    frequent value is large against its other weights (one of them 0) shows it: the results stay inside
    1e-5 (sum|w||x| + |Omega[0]| sum|x|), and the rows whose weight IS the most frequent value are exact."""
    dev = _gpu()
    cb = np.array([5.0, 0.0, 0.125, -0.25], np.float32)
    W = np.full((300, 1), 5.0, np.float32)
    W[::7, 0] = 0.0
    W[3::7, 0] = 0.125
    W[5::11, 0] = -0.25
    rng = np.random.default_rng(77)
    for L in (1, 3, 8, 50):
        X = rng.standard_normal((1, L)).astype(np.float32)
        want = W.astype(np.float64) @ X.astype(np.float64)
        bound = TOL * (np.abs(W).astype(np.float64) @ np.abs(X).astype(np.float64) + 5.0 * np.abs(X).astype(np.float64).sum(axis=0))
        for fmt in ("cer", "cser"):
            Y = run_matmul(fmt, W, cb, X).astype(np.float64)
            assert np.isfinite(Y).all()
            assert (np.abs(Y - want) <= bound).all(), f"{fmt} L={L}"
            dom = W[:, 0] == 5.0
            assert (np.abs(Y[dom] - want[dom]) <= TOL * np.abs(want[dom])).all(), f"{fmt} L={L}: dominant rows"


def test_batch1_several_rows_per_wave():
    """More rows than one round of waves holds: the batch-1 kernel's loop over a wave's rows (matrices of up to 4096 -
    8192 rows run a variant without it).  10245 rows of few groups, then rows of up to 255 groups."""
    dev = _gpu()
    for w, rep in ((wl.alexnet_fc6(L=1, scale=2), 5), (wl.sweep_cell(256, 0.7, L=1, scale=1), 5)):
        W = np.vstack([w.W[::(-1) ** i] for i in range(rep)])
        X = np.ascontiguousarray(w.X[:, :1])
        want = oracle.dot_dense(W, X, threads=8)
        scale = oracle.abs_dot_dense(W, X, threads=8)
        for fmt in ("cer", "cser"):
            print(f"{w.name} x{rep} {fmt}", flush=True)
            Y = run_matmul(fmt, W, w.codebook, X, opts=B.MatmulOpts(path=B.CER_PATH_GEMV), want_path=B.CER_PATH_GEMV)
            check(Y, want, scale, f"{w.name} x{rep} {fmt}")


def test_concurrent_calls_on_one_handle():
    """Four host threads, each with its own stream and its own inputs, call every kind of product on the same
    handles at the same time (the handle is immutable, the library's one-time set-up is guarded): every result
    must match the oracle."""
    import threading
    dev = _gpu()
    cases = []
    for w, L in ((wl.alexnet_fc6(L=1, scale=8), 1), (wl.sweep_cell(256, 0.5, L=1, scale=4), 1),
                 (wl.alexnet_fc6(L=32, scale=8), 32), (wl.conv3x3(L=7, nonzero_dominant=True, scale=4), 7)):
        cases.append((w, L, B.cer_encode(w.W, w.codebook), B.cser_encode(w.W, w.codebook)))
    errors = []

    def worker(tid):
        try:
            stream = torch.cuda.Stream(device=dev)
            rng = np.random.default_rng(300 + tid)
            with torch.cuda.stream(stream):
                for rep in range(6):
                    for w, L, hc, hs in cases:
                        X = rng.standard_normal((w.n, L)).astype(np.float32)
                        Xd = torch.from_numpy(X).to(dev, non_blocking=False)
                        Yc = torch.full((w.m, L), float("nan"), dtype=torch.float32, device=dev)
                        Ys = torch.full((w.m, L), float("nan"), dtype=torch.float32, device=dev)
                        B.cer_matmul(hc, Xd, Yc, L, stream)
                        B.cser_matmul(hs, Xd, Ys, L, stream)
                        stream.synchronize()
                        want = w.W.astype(np.float64) @ X.astype(np.float64)
                        scale = np.abs(w.W).astype(np.float64) @ np.abs(X).astype(np.float64)
                        om0 = float(B.cer_get_array(hc, B.CER_ARRAY_OMEGA)[0])
                        bound = TOL * (scale + abs(om0) * np.abs(X).astype(np.float64).sum(axis=0)[None, :])
                        for Y in (Yc, Ys):
                            y = Y.cpu().numpy().astype(np.float64)
                            if not (np.isfinite(y).all() and (np.abs(y - want) <= bound).all()):
                                errors.append(f"thread {tid} rep {rep} {w.name} L={L}")
        except Exception as e:  # noqa: BLE001 - reported below
            errors.append(f"thread {tid}: {e!r}")

    threads = [threading.Thread(target=worker, args=(t,)) for t in range(4)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    for _, _, hc, hs in cases:
        B.cer_free(hc)
        B.cer_free(hs)
    assert not errors, errors[:5]
