#!/usr/bin/env python3
"""Benchmark of the CER / CSER product Y = W.X on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--format cer|cser]
                    [--warm] [--report PATH --all]

A step is one call of cer_matmul / cser_matmul (the whole hot path: group lists, index stream,
gather-add, one multiply per group, cross-lane reduction, output write) on inputs that already
reside in device memory.  By default successive steps rotate over R independent device copies of
the encoded matrix, R chosen so that the copies exceed twice the 256 MB last-level cache: every
step then streams its arrays from HBM ("cold").  --warm reuses one copy (cache-resident numbers).

Workloads: vgg_fc6_L<L> (default vgg_fc6_L1), alexnet_fc6_L<L>, conv3x3_L<L>, conv3x3_dom_L<L>, c1,
sweep_K<K>_p<p0>[_L<L>], quant<bits>_fc6_L<L> (dense Laplace weights, 4096 x 9216, through the device quantizer).  --front-end encode|quantize|decode times the device-side conversion calls instead.

Prints ONE JSON line on stdout; --report writes a table over several workloads to a file.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0            # MI355X HBM3E, published
LAST_LEVEL_CACHE_BYTES = 256 << 20

METRIC = "CER/CSER W.X dense-equiv GFLOP/s and achieved HBM GB/s (% of peak) vs dense HIP"


def make_workload(name: str):
    from paper_1805_10692_amd import workloads as wl
    m = re.fullmatch(r"vgg_fc6_L(\d+)", name)
    if m:
        return wl.vgg_fc6(L=int(m.group(1)))
    m = re.fullmatch(r"vgg_fc6_rows([0-9.]+)_L(\d+)", name)
    if m:  # log-normal row lengths (standard deviation of the logarithm), otherwise the vgg_fc6 matrix
        return wl.vgg_fc6_unequal_rows(L=int(m.group(2)), sigma=float(m.group(1)))
    m = re.fullmatch(r"alexnet_fc6_L(\d+)", name)
    if m:
        return wl.alexnet_fc6(L=int(m.group(1)))
    m = re.fullmatch(r"conv3x3(_dom)?_L(\d+)", name)
    if m:
        return wl.conv3x3(L=int(m.group(2)), nonzero_dominant=bool(m.group(1)))
    m = re.fullmatch(r"quant(\d)_fc6_L(\d+)", name)
    if m:
        # a dense Laplace layer (AlexNet-fc6 size) through the library's own uniform quantizer: the regime of the
        # paper's dense, low-entropy networks (p0 about 0.3, 3 - 4 bits of entropy)
        import torch
        from paper_1805_10692_amd import binding as B
        bits, L = int(m.group(1)), int(m.group(2))
        W0 = wl.dense_weights(4096, 9216, seed=9)
        Wd = torch.from_numpy(W0).to("cuda:0")
        Wq = torch.empty_like(Wd)
        cb = B.cer_quantize_uniform(Wd, W0.size, bits, None, Wq)
        torch.cuda.synchronize()
        X = wl.sample_X(np.random.Generator(np.random.PCG64(10)), 9216, L)
        return wl.Workload(name, Wq.cpu().numpy(), np.asarray(cb, np.float32), X, np.zeros(len(cb)), 9)
    if name == "c1":
        return wl.config1()
    m = re.fullmatch(r"sweep_K(\d+)_p([0-9.]+)(?:_L(\d+))?", name)
    if m:
        return wl.sweep_cell(int(m.group(1)), float(m.group(2)), L=int(m.group(3) or 16))
    m = re.fullmatch(r"rand_(\d+)x(\d+)_K(\d+)_p([0-9.]+)_L(\d+)", name)
    if m:  # any shape: K values, the most frequent one with the given probability, the rest uniform
        return wl.random_lowentropy(int(m.group(1)), int(m.group(2)), int(m.group(3)), float(m.group(4)),
                                    int(m.group(5)), seed=11)
    raise SystemExit(f"unknown workload {name}")


def kernel_name(fmt: str, L: int, path, K: int = 0, n: int = 0) -> str:
    """The kernel that dominates a product (cer_matmul_path's numbering for cer / cser).  Batch 1: handles of 2 - 256
    values whose X fits in LDS (every benchmark configuration) run the rank-table kernel."""
    if fmt == "csr":
        return "csr_gemv_kernel" if L == 1 else "csr_gemm_kernel"
    if path == 0 and 2 <= K <= 256 and 0 < n <= 36000:
        return "cer_gemv_tab_kernel"
    return {0: "cer_gemv_kernel",
            1: "cer_gemm_expand_kernel",
            2: "cer_xtile_kernel", 3: "decode_kernel + dense_gemm_mfma_kernel", 4: "cer_gemv_expand_kernel",
            5: "cer_strip_kernel"}[path]


def algorithmic_bytes(dims: dict, bits: dict, L: int) -> int:
    """Bytes the method itself must move per product: every format array once at its stored width
    (pointer arrays counted as 32-bit, the width the device copy uses), X once, Y once."""
    b = dims["nnz"] * bits["colI"] // 8 + 4 * (dims["groups"] + 1) + 4 * (dims["m"] + 1) + 4 * dims["K"]
    if dims["is_cser"]:
        b += dims["groups"] * bits["omegaI"] // 8
    return b + 4 * dims["n"] * L + 4 * dims["m"] * L


def read_traffic(workload: str, fmt: str):
    """(HBM bytes per launch, where they come from).  The counters are not collected in this run: the figure is the one
    recorded in the committed rocprofv3 --pmc summary of the same command, if there is one (None otherwise)."""
    rel = os.path.join("profiles", f"traffic_{fmt}_{workload}.txt")
    path = os.path.join(ROOT, rel)
    if not os.path.exists(path):
        return None, None
    txt = open(path).read()
    f = re.search(r"^fetch_bytes_per_launch:\s*([0-9.eE+]+)", txt, re.M)
    w = re.search(r"^write_bytes_per_launch:\s*([0-9.eE+]+)", txt, re.M)
    if not f or not w:
        return None, None
    return float(f.group(1)) + float(w.group(1)), rel + " (recorded rocprofv3 --pmc runs of this command; not collected in this run)"


SETTLE_S = 0.1


def time_steps(fn, steps: int, warmup: int):
    """(wall ms per step, HIP-event ms per step) over exactly `steps` calls after `warmup` calls."""
    import torch
    # The GPU raises its clocks only under sustained load (the first 10 - 20 ms after an idle phase run up to 10 %
    # slower): untimed launches of the same step for SETTLE_S seconds, then the warm-up steps, then the timed ones.
    t_settle = time.perf_counter()
    i = 0
    while time.perf_counter() - t_settle < SETTLE_S:
        for _ in range(50):
            fn(i)
            i += 1
        torch.cuda.synchronize()
    for i in range(warmup):
        fn(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        fn(i)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) * 1e3 / steps, e0.elapsed_time(e1) / steps


def probe_copy(mib: int, reps: int = 20) -> dict:
    """Runs the library's plain copy kernel on `mib` MiB: known traffic (mib read + mib written per launch)
    against which the rocprofv3 byte counters of the same run are scaled."""
    import torch
    from paper_1805_10692_amd import binding as B
    n = (mib << 20) // 4
    src = torch.ones(n, dtype=torch.float32, device="cuda:0")
    dst = torch.empty_like(src)
    wall, ev = time_steps(lambda i: B.cer_stream_copy(dst, src, n * 4), reps, 3)
    return {"MiB": mib, "us_per_launch": ev * 1e3, "GBps_read_plus_write": 2 * n * 4 / (ev * 1e-3) / 1e9}


def probe_stream(nbytes: int, steps: int = 1000) -> dict:
    """What one launch that does nothing but read `nbytes` costs here, cold (rotation over slices of a buffer
    larger than twice the last-level cache), and what a launch that reads 16 bytes costs: the ceiling and the
    floor between which a product of that size lives.  Uses the library's cer_stream_read kernel."""
    import torch
    from paper_1805_10692_amd import binding as B
    piece = (nbytes + 4095) // 4096 * 4096
    R = max(2, -(-2 * LAST_LEVEL_CACHE_BYTES // piece))
    buf = torch.zeros(R * piece, dtype=torch.uint8, device="cuda:0")
    sink = torch.zeros(16384, dtype=torch.uint8, device="cuda:0")
    base, sp = buf.data_ptr(), sink.data_ptr()
    stream = torch.cuda.current_stream().cuda_stream
    lib = B.lib()

    def big(i):
        lib.cer_stream_read(base + (i % R) * piece, nbytes, sp, stream)

    def tiny(i):
        lib.cer_stream_read(base, 16, sp, stream)

    _, ev_big = time_steps(big, steps, 50)
    _, ev_tiny = time_steps(tiny, steps, 50)
    return {"bytes": nbytes, "read_only_launch_us": ev_big * 1e3, "read_only_GBps": nbytes / (ev_big * 1e-3) / 1e9,
            "read_only_frac_of_peak": nbytes / (ev_big * 1e-3) / 1e9 / HBM_PEAK_GBS, "empty_launch_us": ev_tiny * 1e3}


def run_one(name: str, fmt: str, steps: int, warmup: int, warm: bool, with_cpu: bool, with_dense: bool, opts=None,
            cpu_timing: bool = True, strips: bool = False) -> dict:
    """with_cpu: the oracle checks sampled rows of the timed buffers (and, with cpu_timing, is timed as cpu_baseline).
    strips: the handles get the strip-major index (cer_prepare_strips), so that the library may choose its strip kernel."""
    import torch

    from paper_1805_10692_amd import binding as B

    dev = torch.device("cuda:0")
    w = make_workload(name)
    L = w.L
    if fmt == "csr":
        # the paper's sparse comparator: every element != 0 stored with its own fp32 value
        hs = B.cser_encode(w.W, w.codebook)
        stats = B.cer_get_stats(hs)
        B.cer_free(hs)
        h0 = B.csr_encode(w.W)
        mm, clone, free, dev_bytes = B.csr_matmul, B.csr_clone_device, B.csr_free, B.csr_device_bytes
        nnz = len(B.csr_get_array(h0, 0))
        dims = {"m": w.m, "n": w.n, "K": len(w.codebook), "nnz": nnz, "groups": 0, "is_cser": 0}
        idx_bytes = B.csr_get_array(h0, 1).dtype.itemsize
        alg_bytes = nnz * (4 + idx_bytes) + 4 * (w.m + 1) + 4 * w.n * L + 4 * w.m * L
    else:
        enc, mm = (B.cer_encode, B.cer_matmul) if fmt == "cer" else (B.cser_encode, B.cser_matmul)
        clone, free, dev_bytes = B.cer_clone_device, B.cer_free, B.cer_device_bytes
        h0 = enc(w.W, w.codebook)
        dims, stats = B.cer_get_dims(h0), B.cer_get_stats(h0)
        bits = {"colI": B.cer_get_array(h0, B.CER_ARRAY_COLI).dtype.itemsize * 8,
                "omegaI": B.cer_get_array(h0, B.CER_ARRAY_OMEGAI).dtype.itemsize * 8}
        alg_bytes = algorithmic_bytes(dims, bits, L)
    fmt_bytes = dev_bytes(h0)

    Xd = torch.from_numpy(w.X).to(dev)
    Yd = torch.empty((w.m, L), dtype=torch.float32, device=dev)

    # Parity on the buffers that are timed (sampled rows at full size).  The CPU leg (the only part of this
    # file that touches the oracle) supplies the reference; without it the timed product is compared with the
    # library's dense product further down.
    rows = np.sort(np.random.default_rng(0).choice(w.m, min(w.m, 32 if L > 256 else 128), replace=False))
    Wr = np.ascontiguousarray(w.W[rows])
    want = scale = None
    if with_cpu:
        import oracle
        want, scale = oracle.dot_dense(Wr, w.X, threads=8), oracle.abs_dot_dense(Wr, w.X, threads=8)
    want_strips = fmt != "csr" and L > 1 and (strips or (opts is not None and opts.path == B.CER_PATH_STRIP))
    if want_strips:
        B.cer_prepare_strips(h0)
    if opts is not None and fmt != "csr":
        B.cer_matmul_ex(h0, Xd, Yd, L, None, opts)
    else:
        mm(h0, Xd, Yd, L)
    torch.cuda.synchronize()
    y_rows = Yd.cpu().numpy()[rows].astype(np.float64)
    if with_cpu:
        err = np.abs(y_rows - want)
        if not (err <= 1e-5 * scale).all():
            raise SystemExit(f"parity check failed on {name}/{fmt}: max err {err.max():.3e}")

    # cold rotation: enough device copies to exceed twice the last-level cache
    R = 1 if warm else max(2, -(-2 * LAST_LEVEL_CACHE_BYTES // max(fmt_bytes, 1)))
    R = min(R, 256)
    handles = [h0] + [clone(h0) for _ in range(R - 1)]
    if want_strips:
        for h in handles:
            B.cer_prepare_strips(h)   # the strip-major index is per device copy
    stream = torch.cuda.current_stream().cuda_stream
    lib = B.lib()
    cfn = {"cer": lib.cer_matmul, "cser": lib.cser_matmul, "csr": lib.csr_matmul}[fmt]
    ptrs = [h.ptr for h in handles]
    xp, yp = Xd.data_ptr(), Yd.data_ptr()

    if opts is not None and fmt != "csr":   # the caller's choice of kernel instead of the library's
        import ctypes
        ex, optr = lib.cer_matmul_ex, ctypes.byref(opts)
        cfn = lambda h, x, y, l, st: ex(h, x, y, l, st, optr)  # noqa: E731

    def step(i):
        rc = cfn(ptrs[i % R], xp, yp, L, stream)
        if rc != 0:
            raise SystemExit(f"matmul failed: {rc}")

    wall_ms, ev_ms = time_steps(step, steps, warmup)
    flops = 2.0 * w.m * w.n * L
    out = {
        "workload": name, "format": fmt, "m": w.m, "n": w.n, "L": L, "K": dims["K"], "nnz": dims["nnz"],
        "groups": dims["groups"], "H_bits": round(stats["H"], 4), "p0": round(stats["p0"], 5),
        "k_bar": round(stats["k_bar"], 3), "k_tilde": round(stats["k_tilde"], 3),
        "cache_state": "warm (one copy)" if warm else f"cold (rotation over {R} device copies)",
        "ms_per_step": wall_ms, "event_ms_per_step": ev_ms,
        "dense_equiv_gflops": flops / (wall_ms * 1e-3) / 1e9,
        "algorithmic_bytes": alg_bytes, "format_bytes": fmt_bytes,
        "algorithmic_GBps": alg_bytes / (ev_ms * 1e-3) / 1e9,
        "gather_GBps_onchip": dims["nnz"] * 4.0 * L / (ev_ms * 1e-3) / 1e9,
        "dense_bytes": 4 * (w.m * w.n + w.n * L + w.m * L),
        "path": None if fmt == "csr" else B.cer_matmul_path_ex(h0, L, opts),
    }
    for h in handles[1:]:
        free(h)

    if with_dense:
        Wd = torch.from_numpy(w.W).to(dev)
        Yd2 = torch.empty_like(Yd)
        B.dense_matmul(Wd, Xd, Yd2, w.m, w.n, L)
        torch.cuda.synchronize()
        d_rows = Yd2.cpu().numpy()[rows].astype(np.float64)
        if with_cpu:
            derr = np.abs(d_rows - want)
            if not (derr <= 1e-5 * scale).all():
                raise SystemExit(f"dense baseline parity failed on {name}: {derr.max():.3e}")
        else:  # two independent fp32 kernels on the same inputs: each within 1e-5 * sum|w||x| of the exact product
            bound = 2e-5 * (np.abs(Wr).astype(np.float64) @ np.abs(w.X).astype(np.float64))
            if not (np.abs(y_rows - d_rows) <= bound).all():
                raise SystemExit(f"{name}/{fmt}: product and dense baseline disagree")
        wp = Wd.data_ptr()
        y2 = Yd2.data_ptr()

        def dstep(i):
            rc = lib.dense_matmul(wp, xp, y2, w.m, w.n, L, stream)
            if rc != 0:
                raise SystemExit(f"dense_matmul failed: {rc}")

        dsteps = max(5, min(steps, int(0.5e3 / max(out["dense_bytes"] / 4e9, 1e-3))))  # about 0.5 s at 4 TB/s
        d_wall, d_ev = time_steps(dstep, dsteps, max(2, min(warmup, dsteps // 5)))
        out["dense_hip"] = {"ms_per_step": d_wall, "event_ms_per_step": d_ev, "steps": dsteps,
                            "gflops": flops / (d_wall * 1e-3) / 1e9,
                            "GBps": out["dense_bytes"] / (d_ev * 1e-3) / 1e9}
        # rocBLAS through torch, as a cross-check that the in-house dense kernel is not a straw man
        for _ in range(3):
            torch.matmul(Wd, Xd, out=Yd2)
        t_wall, t_ev = time_steps(lambda i: torch.matmul(Wd, Xd, out=Yd2), dsteps, 2)
        out["dense_rocblas_ms_per_step"] = t_wall
        out["speedup_vs_dense_hip"] = d_wall / wall_ms
        out["speedup_vs_dense_rocblas"] = t_wall / wall_ms
        del Wd

    if with_cpu and cpu_timing:
        import oracle
        A = oracle.csr_encode(w.W) if fmt == "csr" else oracle.encode(w.W, w.codebook, fmt)
        odot = (lambda th: oracle.dot_csr(A, w.X)) if fmt == "csr" else (lambda th: oracle.dot(A, w.X, threads=th))
        cores = min(len(os.sched_getaffinity(0)), 16)
        cpu = {}
        for label, th in (("1", 1), (str(cores), cores)):
            reps, t_used = 0, 0.0
            budget = 8.0
            while t_used < budget and reps < 200:
                t0 = time.perf_counter()
                odot(th)
                t_used += time.perf_counter() - t0
                reps += 1
            cpu[label] = t_used / reps
        t0 = time.perf_counter()
        oracle.dot_dense(w.W, w.X, threads=cores)
        t_dense = time.perf_counter() - t0
        out["cpu_baseline"] = {
            "value": flops / cpu[str(cores)] / 1e9, "unit": "GFLOP/s (dense-equivalent)", "cores": cores,
            "kind": "oracle",
            "sample": f"whole {name} product ({fmt}), group-sum oracle with fp64 sums, mean over repeats within 8 s",
            "ms_per_step": cpu[str(cores)] * 1e3, "single_thread_ms_per_step": cpu["1"] * 1e3,
            "oracle_dense_ms_per_step": t_dense * 1e3,
            "cpu_speedup_over_dense_oracle": t_dense / cpu[str(cores)],
        }
    free(h0)
    return out


def run_decode(shape: str, fmt: str, steps: int, with_cpu: bool) -> dict:
    """Times cer_decode_device (handle -> dense fp32 matrix in HBM); checked bit for bit against the matrix that
    was encoded."""
    import torch

    from paper_1805_10692_amd import binding as B
    from paper_1805_10692_amd import workloads as wl

    w = {"vgg_fc6": lambda: wl.vgg_fc6(L=1), "alexnet_fc6": lambda: wl.alexnet_fc6(L=1),
         "conv3x3": lambda: wl.conv3x3(L=1)}[shape]()
    h = (B.cser_encode if fmt == "cser" else B.cer_encode)(w.W, w.codebook)
    out = torch.empty((w.m, w.n), dtype=torch.float32, device="cuda:0")
    B.cer_decode_device(h, out)
    torch.cuda.synchronize()
    if not np.array_equal(out.cpu().numpy().view(np.uint32), (w.W + np.float32(0)).view(np.uint32)):
        raise SystemExit("decode parity failed")
    lib, hp, op, stream = B.lib(), h.ptr, out.data_ptr(), torch.cuda.current_stream().cuda_stream
    wall, ev = time_steps(lambda i: lib.cer_decode_device(hp, op, stream), steps, 3)
    enc_bytes = B.cer_device_bytes(h)
    alg = 4 * w.m * w.n + enc_bytes
    res = {"metric": "decode_dense_output_GBps", "value": 4 * w.m * w.n / (wall * 1e-3) / 1e9, "unit": "GB/s of fp32 output",
           "ms_per_step": wall, "steps": steps, "n_gpus": 1, "dtype": "u16->f32", "data": "synthetic",
           "config": {"workload": f"decode_{shape}", "format": fmt, "m": w.m, "n": w.n},
           "roofline": {"bound": "hbm", "achieved": alg / (ev * 1e-3) / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": alg / (ev * 1e-3) / 1e9 / HBM_PEAK_GBS, "traffic": None,
                        "algorithmic_bytes_per_call": alg, "event_us_per_launch": ev * 1e3}}
    if with_cpu:
        import oracle
        A = oracle.encode(w.W, w.codebook, fmt)
        t0 = time.perf_counter()
        oracle.decode(A)
        t_cpu = time.perf_counter() - t0
        res["cpu_baseline"] = {"value": 4 * w.m * w.n / t_cpu / 1e9, "unit": "GB/s of fp32 output", "cores": 1, "kind": "oracle",
                               "sample": "one whole decode of the same matrix", "ms_per_step": t_cpu * 1e3}
    B.cer_free(h)
    return res


def run_front_end(kind: str, shape: str, fmt: str, bits: int, steps: int, with_cpu: bool) -> dict:
    """Times the device front-end (not part of the headline metric): `encode` converts an already quantized
    matrix that lives in HBM, `quantize` takes unquantized weights through the uniform quantizer first.
    Before the timed calls the handle is compared array by array with the CPU leg's oracle conversion of the same
    matrix (which is also what is timed as `cpu_baseline`); with --no-cpu, with the library's host encoder."""
    import torch

    from paper_1805_10692_amd import binding as B
    from paper_1805_10692_amd import workloads as wl

    dev = torch.device("cuda:0")
    if kind == "encode":
        w = {"vgg_fc6": lambda: wl.vgg_fc6(L=1), "alexnet_fc6": lambda: wl.alexnet_fc6(L=1),
             "conv3x3": lambda: wl.conv3x3(L=1)}[shape]()
        W, cb = w.W, w.codebook
        call = lambda Wd: B.cer_encode_device(Wd, W.shape[0], W.shape[1], cb, fmt)
        passes = 1
    else:
        m, n = {"vgg_fc6": (4096, 25088), "alexnet_fc6": (4096, 9216), "conv3x3": (512, 4608)}[shape]
        W = wl.dense_weights(m, n, seed=9)
        call = lambda Wd: B.cer_quantize_encode_device(Wd, m, n, bits, fmt)[0]
        passes = 2  # the range has to be known before the first element can be quantized
    m, n = W.shape
    Wd = torch.from_numpy(W).to(dev)
    h = call(Wd)
    got = {name: B.cer_get_array(h, which) for which, name in (
        (B.CER_ARRAY_OMEGA, "omega"), (B.CER_ARRAY_COLI, "colI"), (B.CER_ARRAY_OMEGAPTR, "omegaPtr"),
        (B.CER_ARRAY_ROWPTR, "rowPtr"), (B.CER_ARRAY_OMEGAI, "omegaI"))}
    t_cpu = None
    if with_cpu:
        import oracle
        t0 = time.perf_counter()
        if kind == "encode":
            A = oracle.encode(W, cb, fmt)
        else:
            from oracle import quantizer as oq
            codes, qcb = oq.uniform_quantize(W, bits)
            A = oracle.encode(qcb[codes], qcb, fmt)
        t_cpu = time.perf_counter() - t0
        ref = {"omega": A.omega, "colI": A.colI, "omegaPtr": A.omegaPtr, "rowPtr": A.rowPtr, "omegaI": A.omegaI}
    else:
        if kind == "encode":
            Wq, qcb = W, cb
        else:
            Wq_d = torch.empty_like(Wd)
            qcb = B.cer_quantize_uniform(Wd, m * n, bits, None, Wq_d)
            Wq = Wq_d.cpu().numpy().reshape(m, n)
            del Wq_d
        hh = (B.cser_encode if fmt == "cser" else B.cer_encode)(Wq, qcb)
        ref = {name: B.cer_get_array(hh, which) for which, name in (
            (B.CER_ARRAY_OMEGA, "omega"), (B.CER_ARRAY_COLI, "colI"), (B.CER_ARRAY_OMEGAPTR, "omegaPtr"),
            (B.CER_ARRAY_ROWPTR, "rowPtr"), (B.CER_ARRAY_OMEGAI, "omegaI"))}
        B.cer_free(hh)
    for name in ("colI", "omegaPtr", "rowPtr", "omegaI"):
        if fmt == "cer" and name == "omegaI":
            continue
        if not np.array_equal(got[name].astype(np.int64), np.asarray(ref[name]).astype(np.int64)):
            raise SystemExit(f"front-end parity failed on {name}")
    if got["omega"].tobytes() != np.asarray(ref["omega"], dtype=np.float32).tobytes():
        raise SystemExit("front-end parity failed on Omega")
    enc_bytes = B.cer_device_bytes(h)
    stats, K = B.cer_get_stats(h), B.cer_get_dims(h)["K"]
    B.cer_free(h)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        B.cer_free(call(Wd))
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / steps
    alg = passes * 4 * m * n + enc_bytes
    out = {"metric": "front_end_dense_input_GBps", "value": 4 * m * n / dt / 1e9, "unit": "GB/s of fp32 input",
           "ms_per_step": dt * 1e3, "steps": steps, "n_gpus": 1, "dtype": "f32->u8/u16", "data": "synthetic",
           "config": {"workload": f"{kind}_{shape}", "format": fmt, "m": m, "n": n, "bits": bits if kind == "quantize" else None,
                      "K": int(K), "H_bits": round(stats["H"], 3), "p0": round(stats["p0"], 4)},
           "roofline": {"bound": "hbm", "achieved": alg / dt / 1e9, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                        "frac": alg / dt / 1e9 / HBM_PEAK_GBS, "traffic": None,
                        "note": "whole call, allocation and synchronisation included; per-kernel times in profiles/",
                        "algorithmic_bytes_per_call": alg}}
    if with_cpu:
        out["cpu_baseline"] = {"value": 4 * m * n / t_cpu / 1e9, "unit": "GB/s of fp32 input", "cores": 1,
                               "kind": "oracle", "sample": "one whole conversion of the same matrix", "ms_per_step": t_cpu * 1e3}
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--front-end", default=None, choices=("encode", "quantize", "decode"),
                    help="time the device front-end instead of the product (shape from --shape)")
    ap.add_argument("--shape", default="vgg_fc6", choices=("vgg_fc6", "alexnet_fc6", "conv3x3"))
    ap.add_argument("--bits", type=int, default=7)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="vgg_fc6_L1")
    ap.add_argument("--format", default="cer", choices=("cer", "cser", "csr"))
    ap.add_argument("--warm", action="store_true", help="reuse one device copy (cache-resident)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-dense", action="store_true")
    ap.add_argument("--no-probe", action="store_true", help="skip the read-only stream probe of the batch-1 line")
    ap.add_argument("--no-steady", action="store_true", help="skip the HBM-bound companion measurement of the default line")
    ap.add_argument("--probe-copy", type=int, default=0, metavar="MiB",
                    help="also launch the plain copy kernel on this many MiB (calibrates byte counters)")
    ap.add_argument("--path", type=int, default=-1, help="kernel to prefer (numbering of cer_matmul_path), -1 = the library's choice")
    ap.add_argument("--strips", action="store_true",
                    help="build the strip-major index of every handle (cer_prepare_strips): the library may then choose kernel 5")
    ap.add_argument("--flags", type=int, default=0, help="CER_OPT_* bits for cer_matmul_ex")
    ap.add_argument("--tile-cols", type=int, default=0, help="batch columns per tile for cer_matmul_ex")
    ap.add_argument("--report", default=None, help="write a table over workloads/formats to this JSON file")
    ap.add_argument("--all", action="store_true", help="with --report: all named workloads and the entropy sweep")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU; this build has no multi-GPU path (--gpus must be 1)", file=sys.stderr)
        return 2

    import torch
    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        return 2

    if args.front_end:
        fe_steps = args.steps if args.steps != ap.get_default("steps") else 20
        fe_fmt = "cser" if args.format == "cser" else "cer"
        if args.front_end == "decode":
            print(json.dumps(run_decode(args.shape, fe_fmt, fe_steps, not args.no_cpu)), flush=True)
        else:
            print(json.dumps(run_front_end(args.front_end, args.shape, fe_fmt, args.bits, fe_steps, not args.no_cpu)),
                  flush=True)
        return 0

    opts = None
    if args.path != -1 or args.flags or args.tile_cols:
        from paper_1805_10692_amd import binding as B
        opts = B.MatmulOpts(path=args.path, tile_cols=args.tile_cols, flags=args.flags)
    r = run_one(args.workload, args.format, args.steps, args.warmup, args.warm, not args.no_cpu, not args.no_dense, opts,
                strips=args.strips)
    traffic, traffic_source = read_traffic(args.workload, args.format)
    line = {
        "metric": METRIC, "value": r["dense_equiv_gflops"], "unit": "GFLOP/s (dense-equivalent, 2*m*n*L/t)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": r["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {k: r[k] for k in ("workload", "format", "m", "n", "L", "K", "nnz", "groups", "H_bits", "p0",
                                     "k_bar", "k_tilde", "cache_state", "path")},
        "roofline": {"bound": "hbm", "achieved": r["algorithmic_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": r["algorithmic_GBps"] / HBM_PEAK_GBS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": kernel_name(args.format, r["L"], r["path"], r["K"], r["n"]),
                     "algorithmic_bytes_per_launch": r["algorithmic_bytes"],
                     "event_us_per_launch": r["event_ms_per_step"] * 1e3},
        "cpu_baseline": r.get("cpu_baseline"),
        "dense_hip": r.get("dense_hip"),
        "speedup_vs_dense_hip": r.get("speedup_vs_dense_hip"),
        "speedup_vs_dense_rocblas": r.get("speedup_vs_dense_rocblas"),
        "hbm_frac_of_peak": r["algorithmic_GBps"] / HBM_PEAK_GBS,
    }
    if args.probe_copy:
        line["copy_probe"] = probe_copy(args.probe_copy)
    if r["L"] == 1 and not args.warm and not args.no_probe:
        # the HBM-bound case: how fast a launch that only streams the same bytes is on this machine
        sp = probe_stream(r["algorithmic_bytes"])
        line["roofline"]["stream_probe"] = sp
        line["roofline"]["frac_of_read_only_launch"] = sp["read_only_launch_us"] / (r["event_ms_per_step"] * 1e3)
    if args.workload == ap.get_default("workload") and not args.warm and not args.no_steady and args.format != "csr":
        # The default workload is 10.6 MB, about the size of a launch.  The same kernel where HBM is the roof: a 4096 x
        # 9216 layer quantized to 7 bits (57 MB of indices), cold, with a read-only launch of the same bytes beside it.
        sname = "quant7_fc6_L1"
        rs = run_one(sname, args.format, min(args.steps, 1000), min(args.warmup, 100), False, not args.no_cpu, False, opts,
                     cpu_timing=False)
        st, st_src = read_traffic(sname, args.format)
        steady = {"workload": sname, "bound": "hbm", "achieved": rs["algorithmic_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                  "frac": rs["algorithmic_GBps"] / HBM_PEAK_GBS, "traffic": st, "traffic_source": st_src,
                  "kernel": kernel_name(args.format, rs["L"], rs["path"], rs["K"], rs["n"]),
                  "algorithmic_bytes_per_launch": rs["algorithmic_bytes"], "event_us_per_launch": rs["event_ms_per_step"] * 1e3,
                  "m": rs["m"], "n": rs["n"], "nnz": rs["nnz"], "K": rs["K"], "H_bits": rs["H_bits"], "p0": rs["p0"],
                  "cache_state": rs["cache_state"]}
        if not args.no_probe:
            sp = probe_stream(rs["algorithmic_bytes"], steps=300)
            steady["stream_probe"] = sp
            steady["frac_of_read_only_launch"] = sp["read_only_launch_us"] / (rs["event_ms_per_step"] * 1e3)
        line["roofline_steady"] = steady
    print(json.dumps(line), flush=True)

    if args.report:
        names = ["vgg_fc6_L1", "vgg_fc6_L64", "alexnet_fc6_L32", "c1"]
        if args.all:
            from paper_1805_10692_amd import workloads as wl
            names += ["conv3x3_L3136", "conv3x3_dom_L3136"]
            names += [f"sweep_K{K}_p{p0}" for K in wl.SWEEP_K for p0 in wl.SWEEP_P0]
        table = []
        for nm in names:
            for fmt in ("cer", "cser", "csr"):
                for warm in (False, True):
                    big = nm.startswith("conv")
                    rr = run_one(nm, fmt, 20 if big else 300, 3 if big else 30, warm, False, not warm)
                    table.append(rr)
                    if fmt != "csr" and rr["path"] == 3:
                        # the library chose decode + dense: the method's own number is the gather kernel's
                        from paper_1805_10692_amd import binding as B
                        rg = run_one(nm, fmt, 20 if big else 300, 3 if big else 30, warm, False, not warm,
                                     B.MatmulOpts(path=B.CER_PATH_GEMM))
                        rg["format"] = fmt + " (gather kernel)"
                        table.append(rg)
                    if fmt != "csr" and rr["L"] >= 32 and rr["L"] % 32 == 0 and rr["K"] <= 64:
                        # the same product with the strip-major index prepared: the strip kernel on request, and what
                        # the library chooses by itself once the index exists
                        from paper_1805_10692_amd import binding as B
                        rs5 = run_one(nm, fmt, 20 if big else 300, 3 if big else 30, warm, False, False,
                                      B.MatmulOpts(path=B.CER_PATH_STRIP))
                        rs5["format"] = fmt + " (strip kernel)"
                        table.append(rs5)
                        ra = run_one(nm, fmt, 20 if big else 300, 3 if big else 30, warm, False, False, strips=True)
                        ra["format"] = fmt + " (strip-major index prepared, library's choice)"
                        table.append(ra)
                    print(f"[report] {nm} {fmt} {'warm' if warm else 'cold'}: {rr['ms_per_step'] * 1e3:.2f} us/step, "
                          f"{rr['algorithmic_GBps']:.0f} GB/s alg, speedup vs dense "
                          f"{rr.get('speedup_vs_dense_hip', float('nan')):.2f}", file=sys.stderr, flush=True)
        os.makedirs(os.path.dirname(os.path.abspath(args.report)), exist_ok=True)
        with open(args.report, "w") as f:
            json.dump(table, f, indent=1)
    return 0


if __name__ == "__main__":
    sys.exit(main())
