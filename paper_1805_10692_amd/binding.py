"""Python binding of the C ABI in include/cer.h -- argument marshalling only.

Every function has the name of the C entry point it calls.  Device buffers are passed as torch
tensors (their ``data_ptr()`` is handed to the library) or as raw integer addresses; streams as
``torch.cuda.Stream`` objects, raw ``hipStream_t`` integers, or None for the current torch stream.
No step of the product runs in Python or in torch, and there is no CPU fallback: if the built
library is missing, loading fails.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
# CER_HIP_LIB selects another build of the same library (e.g. one compiled with other tuning constants)
LIB_PATH = os.environ.get("CER_HIP_LIB") or os.path.join(_PKG, "libcer_hip.so")

CER_OK = 0
CER_E_INVALID = -1
CER_E_NOT_IN_CODEBOOK = -2
CER_E_BAD_CODEBOOK = -3
CER_E_TOO_LARGE = -4
CER_E_NOMEM = -5
CER_E_HIP = -6
CER_E_FORMAT = -7

CER_ARRAY_OMEGA, CER_ARRAY_COLI, CER_ARRAY_OMEGAPTR, CER_ARRAY_ROWPTR, CER_ARRAY_OMEGAI, CER_ARRAY_COUNT = range(6)

EXPORTS = [
    "cer_encode", "cser_encode", "cer_matmul", "cser_matmul", "cer_decode", "cser_decode",
    "cer_get_array", "cer_get_dims", "cer_storage_bits", "cer_get_stats", "cer_clone_device",
    "cer_device_bytes", "cer_long_row_parts", "cer_free", "dense_matmul", "cer_stream_copy", "cer_strerror", "cer_last_hip_error",
    "csr_encode", "csr_matmul", "csr_decode", "csr_get_array", "csr_storage_bits", "csr_device_bytes",
    "csr_clone_device", "csr_free", "cer_cost_model", "csr_cost_model", "dense_cost_model",
    "cer_encode_device", "cer_quantize_uniform", "cer_quantize_encode_device", "cer_matmul_path", "cer_stream_read",
    "cer_decode_device", "cer_trim", "cer_matmul_ex", "cer_matmul_path_ex", "cer_matmul_noalloc", "cer_prepare_strips",
]

CER_FORMAT_CER, CER_FORMAT_CSER = 0, 1

CER_PATH_AUTO, CER_PATH_GEMV, CER_PATH_GEMM, CER_PATH_XTILE, CER_PATH_DENSE, CER_PATH_GEMV_EXPAND, CER_PATH_STRIP = -1, 0, 1, 2, 3, 4, 5
CER_OPT_SUM_THEN_MULTIPLY, CER_OPT_ROWS_WHOLE, CER_OPT_X_FROM_GLOBAL = 1, 2, 4
CER_OPT_ONE_COLUMN_PER_LANE, CER_OPT_SHORT_CHUNKS, CER_OPT_LONG_CHUNKS, CER_OPT_NO_RANK_TABLE = 8, 16, 32, 64

_lib = None

CER_COUNT_THEOREM, CER_COUNT_EXAMPLE = 0, 1


class CostT(ctypes.Structure):
    _fields_ = [(k, ctypes.c_int64) for k in ("read_weight", "read_omega", "read_colI", "read_omegaPtr", "read_rowPtr",
                                              "read_omegaI", "read_input", "mul", "add", "write", "storage_bits")] + [
        ("energy_pj", ctypes.c_double)]

    def as_dict(self) -> dict:
        d = {k: getattr(self, k) for k, _ in self._fields_}
        d["reads"] = sum(v for k, v in d.items() if k.startswith("read_"))
        d["ops"] = d["reads"] + d["mul"] + d["add"] + d["write"]
        return d


class MatmulOpts(ctypes.Structure):
    """cer_matmul_opts_t: preferred kernel, tile width and CER_OPT_* flags of cer_matmul_ex."""
    _fields_ = [("path", ctypes.c_int32), ("tile_cols", ctypes.c_int32), ("flags", ctypes.c_uint32),
                ("reserved", ctypes.c_uint32)]

    def __init__(self, path: int = CER_PATH_AUTO, tile_cols: int = 0, flags: int = 0):
        super().__init__(path, tile_cols, flags, 0)


class CerError(RuntimeError):
    def __init__(self, code: int, what: str):
        msg = lib().cer_strerror(code).decode()
        if code == CER_E_HIP:
            msg += f" (hipError {lib().cer_last_hip_error()})"
        super().__init__(f"{what}: {msg} [{code}]")
        self.code = code


def lib() -> ctypes.CDLL:
    """Loads paper_1805_10692_amd/libcer_hip.so (built by `python -m paper_1805_10692_amd.build`)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is not built; run `python -m paper_1805_10692_amd.build` "
                              "(there is no fallback implementation)")
        # One HIP runtime per process: PyTorch ships its own copy of it, and the tensors whose pointers this binding
        # passes live in that one.  Loaded after torch, the library binds to the copy that is already there; loaded
        # first, it would bring the system's copy, and products on torch's tensors then fail (no device).
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        vp, i64, i32 = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32
        pvp = ctypes.POINTER(vp)
        for name in ("cer_encode", "cser_encode"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [vp, i64, i64, vp, i32, pvp]
        for name in ("cer_matmul", "cser_matmul"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [vp, vp, vp, i64, vp]
        for name in ("cer_decode", "cser_decode"):
            getattr(L, name).restype = ctypes.c_int
            getattr(L, name).argtypes = [vp, vp]
        L.cer_get_array.restype = ctypes.c_int
        L.cer_get_array.argtypes = [vp, ctypes.c_int, pvp, ctypes.POINTER(i64), ctypes.POINTER(i32)]
        L.cer_get_dims.restype = ctypes.c_int
        L.cer_get_dims.argtypes = [vp, ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i32),
                                   ctypes.POINTER(i64), ctypes.POINTER(i64), ctypes.POINTER(i32)]
        L.cer_storage_bits.restype = i64
        L.cer_storage_bits.argtypes = [vp]
        L.cer_get_stats.restype = ctypes.c_int
        L.cer_get_stats.argtypes = [vp] + [ctypes.POINTER(ctypes.c_double)] * 4
        L.cer_clone_device.restype = ctypes.c_int
        L.cer_clone_device.argtypes = [vp, pvp]
        L.cer_device_bytes.restype = i64
        L.cer_device_bytes.argtypes = [vp]
        L.cer_long_row_parts.restype = i64
        L.cer_long_row_parts.argtypes = [vp]
        L.cer_free.restype = None
        L.cer_free.argtypes = [vp]
        L.dense_matmul.restype = ctypes.c_int
        L.dense_matmul.argtypes = [vp, vp, vp, i64, i64, i64, vp]
        L.csr_encode.restype = ctypes.c_int
        L.csr_encode.argtypes = [vp, i64, i64, pvp]
        L.csr_matmul.restype = ctypes.c_int
        L.csr_matmul.argtypes = [vp, vp, vp, i64, vp]
        L.csr_decode.restype = ctypes.c_int
        L.csr_decode.argtypes = [vp, vp]
        L.csr_get_array.restype = ctypes.c_int
        L.csr_get_array.argtypes = [vp, ctypes.c_int, pvp, ctypes.POINTER(i64), ctypes.POINTER(i32)]
        L.csr_storage_bits.restype = i64
        L.csr_storage_bits.argtypes = [vp]
        L.csr_device_bytes.restype = i64
        L.csr_device_bytes.argtypes = [vp]
        L.csr_clone_device.restype = ctypes.c_int
        L.csr_clone_device.argtypes = [vp, pvp]
        L.csr_free.restype = None
        L.csr_free.argtypes = [vp]
        L.cer_cost_model.restype = ctypes.c_int
        L.cer_cost_model.argtypes = [vp, ctypes.c_int, ctypes.POINTER(CostT)]
        L.csr_cost_model.restype = ctypes.c_int
        L.csr_cost_model.argtypes = [vp, ctypes.c_int, ctypes.POINTER(CostT)]
        L.dense_cost_model.restype = ctypes.c_int
        L.dense_cost_model.argtypes = [i64, i64, ctypes.c_int, ctypes.POINTER(CostT)]
        L.cer_decode_device.restype = ctypes.c_int
        L.cer_decode_device.argtypes = [vp, vp, vp]
        L.cer_stream_read.restype = ctypes.c_int
        L.cer_stream_read.argtypes = [vp, i64, vp, vp]
        L.cer_trim.restype = ctypes.c_int
        L.cer_trim.argtypes = []
        L.cer_matmul_path.restype = ctypes.c_int
        L.cer_matmul_path.argtypes = [vp, i64]
        L.cer_prepare_strips.restype = ctypes.c_int
        L.cer_prepare_strips.argtypes = [vp]
        L.cer_matmul_noalloc.restype = ctypes.c_int
        L.cer_matmul_noalloc.argtypes = [vp, vp, vp, i64, vp]
        L.cer_matmul_ex.restype = ctypes.c_int
        L.cer_matmul_ex.argtypes = [vp, vp, vp, i64, vp, ctypes.POINTER(MatmulOpts)]
        L.cer_matmul_path_ex.restype = ctypes.c_int
        L.cer_matmul_path_ex.argtypes = [vp, i64, ctypes.POINTER(MatmulOpts)]
        L.cer_encode_device.restype = ctypes.c_int
        L.cer_encode_device.argtypes = [vp, i64, i64, vp, i32, i32, vp, pvp]
        L.cer_quantize_uniform.restype = ctypes.c_int
        L.cer_quantize_uniform.argtypes = [vp, i64, i32, vp, vp, vp, ctypes.POINTER(i32), vp]
        L.cer_quantize_encode_device.restype = ctypes.c_int
        L.cer_quantize_encode_device.argtypes = [vp, i64, i64, i32, i32, vp, vp, ctypes.POINTER(i32), pvp]
        L.cer_stream_copy.restype = ctypes.c_int
        L.cer_stream_copy.argtypes = [vp, vp, i64, vp]
        L.cer_strerror.restype = ctypes.c_char_p
        L.cer_strerror.argtypes = [ctypes.c_int]
        L.cer_last_hip_error.restype = ctypes.c_int
        L.cer_last_hip_error.argtypes = []
        _lib = L
    return _lib


def _check(rc: int, what: str) -> None:
    if rc != CER_OK:
        raise CerError(rc, what)


def _dev_ptr(t) -> int:
    if isinstance(t, int):
        return t
    if not t.is_cuda or t.dtype.itemsize != 4 or not t.is_contiguous():
        raise ValueError("expected a contiguous fp32 tensor in device memory")
    return t.data_ptr()


def _stream_ptr(stream) -> int:
    if stream is None:
        import torch
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


class Handle:
    """Owns one cer_handle_t*; freed by cer_free() or when garbage-collected."""

    def __init__(self, ptr: int, fmt: str):
        self.ptr = ptr
        self.fmt = fmt

    def __del__(self):
        try:
            cer_free(self)
        except Exception:
            pass


def _encode(name: str, W: np.ndarray, codebook: np.ndarray) -> Handle:
    W = np.ascontiguousarray(W, dtype=np.float32)
    cb = np.ascontiguousarray(codebook, dtype=np.float32)
    if W.ndim != 2 or cb.ndim != 1:
        raise ValueError("W must be 2-D and the codebook 1-D")
    out = ctypes.c_void_p()
    rc = getattr(lib(), name)(W.ctypes.data, W.shape[0], W.shape[1], cb.ctypes.data, len(cb), ctypes.byref(out))
    _check(rc, name)
    return Handle(out.value, "cser" if name.startswith("cser") else "cer")


def cer_encode(W: np.ndarray, codebook: np.ndarray) -> Handle:
    return _encode("cer_encode", W, codebook)


def cser_encode(W: np.ndarray, codebook: np.ndarray) -> Handle:
    return _encode("cser_encode", W, codebook)


def _fmt_code(fmt: str) -> int:
    if fmt not in ("cer", "cser"):
        raise ValueError("format must be 'cer' or 'cser'")
    return CER_FORMAT_CSER if fmt == "cser" else CER_FORMAT_CER


def cer_encode_device(W, m: int, n: int, codebook: np.ndarray, fmt: str = "cer", stream=None) -> Handle:
    """W: fp32 device tensor (m x n, row-major) whose elements are codebook values."""
    cb = np.ascontiguousarray(codebook, dtype=np.float32)
    out = ctypes.c_void_p()
    rc = lib().cer_encode_device(_dev_ptr(W) if m * n else 0, m, n, cb.ctypes.data, len(cb), _fmt_code(fmt),
                                 _stream_ptr(stream), ctypes.byref(out))
    _check(rc, "cer_encode_device")
    return Handle(out.value, fmt)


def cer_quantize_uniform(W, count: int, bits: int, codes=None, Wq=None, stream=None) -> np.ndarray:
    """Quantizes `count` fp32 device elements; fills the optional device tensors `codes` (uint8) and
    `Wq` (fp32) and returns the codebook."""
    cb = np.zeros(1 << max(bits, 0), np.float32)
    K = ctypes.c_int32(0)
    if codes is not None and (not codes.is_cuda or codes.dtype.itemsize != 1 or not codes.is_contiguous()):
        raise ValueError("codes must be a contiguous uint8 tensor in device memory")
    rc = lib().cer_quantize_uniform(_dev_ptr(W) if count else 0, count, bits,
                                    codes.data_ptr() if codes is not None else 0,
                                    _dev_ptr(Wq) if Wq is not None else 0, cb.ctypes.data, ctypes.byref(K),
                                    _stream_ptr(stream))
    _check(rc, "cer_quantize_uniform")
    return cb[:K.value].copy()


def cer_quantize_encode_device(W, m: int, n: int, bits: int, fmt: str = "cer", stream=None):
    """Unquantized fp32 device tensor -> (handle, codebook)."""
    cb = np.zeros(1 << max(bits, 0), np.float32)
    K = ctypes.c_int32(0)
    out = ctypes.c_void_p()
    rc = lib().cer_quantize_encode_device(_dev_ptr(W) if m * n else 0, m, n, bits, _fmt_code(fmt), _stream_ptr(stream),
                                          cb.ctypes.data, ctypes.byref(K), ctypes.byref(out))
    _check(rc, "cer_quantize_encode_device")
    return Handle(out.value, fmt), cb[:K.value].copy()


def cer_matmul(h: Handle, X, Y, batch: int, stream=None) -> None:
    _check(lib().cer_matmul(h.ptr, _dev_ptr(X), _dev_ptr(Y), batch, _stream_ptr(stream)), "cer_matmul")


def cer_decode_device(h: Handle, W_out, stream=None) -> None:
    """Writes the dense m x n matrix into the fp32 device tensor W_out."""
    d = cer_get_dims(h)
    _check(lib().cer_decode_device(h.ptr, _dev_ptr(W_out) if d["m"] * d["n"] else 0, _stream_ptr(stream)),
           "cer_decode_device")


def cer_trim() -> None:
    """Releases the device memory the library keeps for its temporaries on the current device."""
    _check(lib().cer_trim(), "cer_trim")


def cer_matmul_path(h: Handle, batch: int) -> int:
    """0 = batch-1 kernel, 1 = batched kernel gathering from L2, 2 = batched kernel with X resident in LDS,
    3 = decode into a dense temporary + fp32 matrix-core product (large batches of not-so-sparse matrices),
    4 = batch-1 kernel for rows of many short groups."""
    rc = lib().cer_matmul_path(h.ptr, batch)
    if rc < 0:
        _check(rc, "cer_matmul_path")
    return rc


def cer_matmul_ex(h: Handle, X, Y, batch: int, stream=None, opts: "MatmulOpts | None" = None) -> None:
    _check(lib().cer_matmul_ex(h.ptr, _dev_ptr(X), _dev_ptr(Y), batch, _stream_ptr(stream),
                               ctypes.byref(opts) if opts is not None else None), "cer_matmul_ex")


def cer_prepare_strips(h: Handle) -> None:
    """Builds the strip-major index that cer_matmul_ex needs for CER_PATH_STRIP (once per handle)."""
    _check(lib().cer_prepare_strips(h.ptr), "cer_prepare_strips")


def cer_matmul_noalloc(h: Handle, X, Y, batch: int, stream=None) -> None:
    _check(lib().cer_matmul_noalloc(h.ptr, _dev_ptr(X), _dev_ptr(Y), batch, _stream_ptr(stream)), "cer_matmul_noalloc")


def cer_matmul_path_ex(h: Handle, batch: int, opts: "MatmulOpts | None" = None) -> int:
    rc = lib().cer_matmul_path_ex(h.ptr, batch, ctypes.byref(opts) if opts is not None else None)
    if rc < 0:
        _check(rc, "cer_matmul_path_ex")
    return rc


def cser_matmul(h: Handle, X, Y, batch: int, stream=None) -> None:
    _check(lib().cser_matmul(h.ptr, _dev_ptr(X), _dev_ptr(Y), batch, _stream_ptr(stream)), "cser_matmul")


def _decode(name: str, h: Handle) -> np.ndarray:
    m, n = cer_get_dims(h)["m"], cer_get_dims(h)["n"]
    W = np.empty((m, n), np.float32)
    _check(getattr(lib(), name)(h.ptr, W.ctypes.data), name)
    return W


def cer_decode(h: Handle) -> np.ndarray:
    return _decode("cer_decode", h)


def cser_decode(h: Handle) -> np.ndarray:
    return _decode("cser_decode", h)


def cer_get_array(h: Handle, which: int) -> np.ndarray:
    """A copy of one host array at its stored width (uint8/16/32, float32 for Omega, int64 counts)."""
    p, n, bits = ctypes.c_void_p(), ctypes.c_int64(), ctypes.c_int32()
    _check(lib().cer_get_array(h.ptr, which, ctypes.byref(p), ctypes.byref(n), ctypes.byref(bits)), "cer_get_array")
    if which == CER_ARRAY_OMEGA:
        dt = np.float32
    elif which == CER_ARRAY_COUNT:
        dt = np.int64
    else:
        dt = {8: np.uint8, 16: np.uint16, 32: np.uint32}[bits.value]
    if n.value == 0:
        return np.empty(0, dt)
    buf = (ctypes.c_char * (n.value * np.dtype(dt).itemsize)).from_address(p.value)
    return np.frombuffer(buf, dtype=dt).copy()


def cer_get_dims(h: Handle) -> dict:
    m, n, nnz, g = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    K, cs = ctypes.c_int32(), ctypes.c_int32()
    _check(lib().cer_get_dims(h.ptr, ctypes.byref(m), ctypes.byref(n), ctypes.byref(K), ctypes.byref(nnz),
                              ctypes.byref(g), ctypes.byref(cs)), "cer_get_dims")
    return {"m": m.value, "n": n.value, "K": K.value, "nnz": nnz.value, "groups": g.value, "is_cser": cs.value}


def cer_storage_bits(h: Handle) -> int:
    v = lib().cer_storage_bits(h.ptr)
    if v < 0:
        raise CerError(int(v), "cer_storage_bits")
    return int(v)


def cer_get_stats(h: Handle) -> dict:
    vals = [ctypes.c_double() for _ in range(4)]
    _check(lib().cer_get_stats(h.ptr, *[ctypes.byref(v) for v in vals]), "cer_get_stats")
    return dict(zip(("H", "p0", "k_bar", "k_tilde"), (v.value for v in vals)))


def cer_clone_device(h: Handle) -> Handle:
    out = ctypes.c_void_p()
    _check(lib().cer_clone_device(h.ptr, ctypes.byref(out)), "cer_clone_device")
    return Handle(out.value, h.fmt)


def cer_device_bytes(h: Handle) -> int:
    return int(lib().cer_device_bytes(h.ptr))


def cer_long_row_parts(h: Handle) -> int:
    """Number of further parts into which the batched product splits rows much longer than the average (0: none)."""
    return int(lib().cer_long_row_parts(h.ptr))


def cer_free(h: Handle) -> None:
    if h.ptr:
        lib().cer_free(h.ptr)
        h.ptr = None


def dense_matmul(W, X, Y, m: int, n: int, batch: int, stream=None) -> None:
    _check(lib().dense_matmul(_dev_ptr(W), _dev_ptr(X), _dev_ptr(Y), m, n, batch, _stream_ptr(stream)), "dense_matmul")


def cer_stream_copy(dst, src, nbytes: int, stream=None) -> None:
    def raw(t):
        return t if isinstance(t, int) else t.data_ptr()
    _check(lib().cer_stream_copy(raw(dst), raw(src), nbytes, _stream_ptr(stream)), "cer_stream_copy")


def cer_stream_read(src, nbytes: int, sink, stream=None) -> None:
    def raw(t):
        return t if isinstance(t, int) else t.data_ptr()
    _check(lib().cer_stream_read(raw(src), nbytes, raw(sink), _stream_ptr(stream)), "cer_stream_read")


class CsrHandle:
    """Owns one csr_handle_t*."""

    def __init__(self, ptr: int, m: int, n: int):
        self.ptr, self.m, self.n = ptr, m, n

    def __del__(self):
        try:
            csr_free(self)
        except Exception:
            pass


def csr_encode(W: np.ndarray) -> CsrHandle:
    W = np.ascontiguousarray(W, dtype=np.float32)
    out = ctypes.c_void_p()
    _check(lib().csr_encode(W.ctypes.data, W.shape[0], W.shape[1], ctypes.byref(out)), "csr_encode")
    return CsrHandle(out.value, W.shape[0], W.shape[1])


def csr_matmul(h: CsrHandle, X, Y, batch: int, stream=None) -> None:
    _check(lib().csr_matmul(h.ptr, _dev_ptr(X), _dev_ptr(Y), batch, _stream_ptr(stream)), "csr_matmul")


def csr_decode(h: CsrHandle) -> np.ndarray:
    W = np.empty((h.m, h.n), np.float32)
    _check(lib().csr_decode(h.ptr, W.ctypes.data), "csr_decode")
    return W


def csr_get_array(h: CsrHandle, which: int) -> np.ndarray:
    p, n, bits = ctypes.c_void_p(), ctypes.c_int64(), ctypes.c_int32()
    _check(lib().csr_get_array(h.ptr, which, ctypes.byref(p), ctypes.byref(n), ctypes.byref(bits)), "csr_get_array")
    dt = np.float32 if which == 0 else {8: np.uint8, 16: np.uint16, 32: np.uint32}[bits.value]
    if n.value == 0:
        return np.empty(0, dt)
    buf = (ctypes.c_char * (n.value * np.dtype(dt).itemsize)).from_address(p.value)
    return np.frombuffer(buf, dtype=dt).copy()


def csr_storage_bits(h: CsrHandle) -> int:
    return int(lib().csr_storage_bits(h.ptr))


def csr_device_bytes(h: CsrHandle) -> int:
    return int(lib().csr_device_bytes(h.ptr))


def csr_clone_device(h: CsrHandle) -> CsrHandle:
    out = ctypes.c_void_p()
    _check(lib().csr_clone_device(h.ptr, ctypes.byref(out)), "csr_clone_device")
    return CsrHandle(out.value, h.m, h.n)


def csr_free(h: CsrHandle) -> None:
    if h.ptr:
        lib().csr_free(h.ptr)
        h.ptr = None


def cer_cost_model(h: Handle, convention: int = CER_COUNT_THEOREM) -> dict:
    c = CostT()
    _check(lib().cer_cost_model(h.ptr, convention, ctypes.byref(c)), "cer_cost_model")
    return c.as_dict()


def csr_cost_model(h: CsrHandle, convention: int = CER_COUNT_THEOREM) -> dict:
    c = CostT()
    _check(lib().csr_cost_model(h.ptr, convention, ctypes.byref(c)), "csr_cost_model")
    return c.as_dict()


def dense_cost_model(m: int, n: int, convention: int = CER_COUNT_THEOREM) -> dict:
    c = CostT()
    _check(lib().dense_cost_model(m, n, convention, ctypes.byref(c)), "dense_cost_model")
    return c.as_dict()
