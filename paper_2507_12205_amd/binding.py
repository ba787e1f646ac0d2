"""Thin ctypes binding of libecspmv.so: same names as the C ABI, argument marshalling only.

Every step of the SpMV runs inside the library's HIP kernels; PyTorch is used by callers only to
own device memory and streams.  There is no CPU fallback: if the shared library is missing, loading
fails with an error that says how to build it.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_double, c_int, c_int32, c_int64, c_size_t, c_uint32, c_uint64, c_void_p

import numpy as np

from . import build as _build

OK = 0
ERR_INVALID, ERR_UNSUPPORTED, ERR_NOMEM, ERR_HIP, ERR_NOT_UPLOADED, ERR_TOO_SMALL, ERR_INTERNAL = -1, -2, -3, -4, -5, -6, -7
FLAG_GLOBAL_MATCHING = 1
FLAG_NO_REORDER = 2
FLAG_KEEP_SMALL_SETS = 4
FLAG_CLUSTER_ROWS = 8

EXPORTS = (
    "ecspmv_build_dense", "ecspmv_build_csr", "ecspmv_build_dense_f32", "ecspmv_build_csr_f32", "ecspmv_destroy",
    "ecspmv_stats", "ecspmv_decode", "ecspmv_decode_f32",
    "ecspmv_block_sets", "ecspmv_device_bytes", "ecspmv_export_image", "ecspmv_upload", "ecspmv_run", "ecspmv_run_batch", "ecspmv_run_multi",
    "ecspmv_csr_build_dense", "ecspmv_csr_destroy", "ecspmv_csr_device_bytes", "ecspmv_csr_upload",
    "ecspmv_csr_run", "ecspmv_stream_read", "ecspmv_stream_read_sliced", "ecspmv_empty_launch", "ecspmv_strerror", "ecspmv_last_hip_error",
)


class BuildOpts(Structure):
    _fields_ = [("struct_size", c_uint32), ("delta_bits", c_int32), ("max_granularity", c_int32),
                ("max_rounds", c_int32), ("num_panels", c_int32), ("num_threads", c_int32),
                ("threads_per_wg", c_int32), ("flags", c_uint64)]


class Stats(Structure):
    _fields_ = [("struct_size", c_uint32), ("m", c_int64), ("n", c_int64), ("nnz", c_int64),
                ("image_bytes", c_int64), ("value_bytes", c_int64), ("delta_bytes", c_int64),
                ("meta_bytes", c_int64), ("slack_bytes", c_int64), ("csr32_bytes", c_int64),
                ("csr16_bytes", c_int64), ("nnz_by_g", c_int64 * 5), ("units_by_g", c_int64 * 5),
                ("pad_elements", c_int64), ("gap_pad_elements", c_int64), ("num_panels", c_int32),
                ("threads_per_wg", c_int32), ("panel_stride", c_int64), ("meta_stride", c_int64),
                ("lds_bytes", c_int64), ("max_panel_bytes", c_int64), ("min_panel_bytes", c_int64),
                ("x_access_cost", c_double), ("build_seconds", c_double), ("delta_hist", c_int64 * 9),
                ("delta_bits", c_int32), ("value_bits", c_int32)]

    def as_dict(self) -> dict:
        out = {}
        for name, _ in self._fields_:
            v = getattr(self, name)
            out[name] = list(v) if hasattr(v, "__len__") else v
        return out


class EcspmvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        msg = lib().ecspmv_strerror(status).decode()
        if status == ERR_HIP:
            msg += f" [hipError {lib().ecspmv_last_hip_error()}]"
        super().__init__(f"{where}: {msg} ({status})")


_lib = None


def lib() -> ctypes.CDLL:
    """Load libecspmv.so (built in-tree by `build.build()`); never falls back to anything else."""
    global _lib
    if _lib is not None:
        return _lib
    path = _build.lib_path()
    if not os.path.exists(path):
        raise ImportError(f"{path} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(needs hipcc); there is no CPU fallback for the SpMV path")
    try:
        import torch  # noqa: F401  -- so that the process uses one HIP runtime (the one PyTorch ships)
    except Exception:
        pass
    L = ctypes.CDLL(path)
    L.ecspmv_build_dense.argtypes = [c_void_p, c_int64, c_int64, c_int64, POINTER(BuildOpts), POINTER(c_void_p)]
    L.ecspmv_build_csr.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int64, POINTER(BuildOpts), POINTER(c_void_p)]
    L.ecspmv_build_dense_f32.argtypes = [c_void_p, c_int64, c_int64, c_int64, POINTER(BuildOpts), POINTER(c_void_p)]
    L.ecspmv_build_csr_f32.argtypes = [c_void_p, c_void_p, c_void_p, c_int64, c_int64, POINTER(BuildOpts), POINTER(c_void_p)]
    L.ecspmv_decode_f32.argtypes = [c_void_p, POINTER(c_int64), c_void_p, c_void_p, c_void_p]
    L.ecspmv_destroy.argtypes = [c_void_p]
    L.ecspmv_destroy.restype = None
    L.ecspmv_stats.argtypes = [c_void_p, POINTER(Stats)]
    L.ecspmv_decode.argtypes = [c_void_p, POINTER(c_int64), c_void_p, c_void_p, c_void_p]
    L.ecspmv_block_sets.argtypes = [c_void_p, POINTER(c_int64), POINTER(c_int64), c_void_p, c_void_p, c_void_p]
    L.ecspmv_device_bytes.argtypes = [c_void_p, POINTER(c_size_t)]
    L.ecspmv_export_image.argtypes = [c_void_p, c_void_p, c_size_t]
    L.ecspmv_upload.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p]
    L.ecspmv_run.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p]
    L.ecspmv_run_batch.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_void_p]
    L.ecspmv_run_multi.argtypes = [c_void_p, c_void_p, c_void_p, c_int32, c_void_p]
    L.ecspmv_csr_build_dense.argtypes = [c_void_p, c_int64, c_int64, c_int64, POINTER(c_void_p)]
    L.ecspmv_csr_destroy.argtypes = [c_void_p]
    L.ecspmv_csr_destroy.restype = None
    L.ecspmv_csr_device_bytes.argtypes = [c_void_p, POINTER(c_size_t)]
    L.ecspmv_csr_upload.argtypes = [c_void_p, c_void_p, c_size_t, c_void_p]
    L.ecspmv_csr_run.argtypes = [c_void_p, c_void_p, c_void_p, c_void_p]
    L.ecspmv_stream_read.argtypes = [c_void_p, c_size_t, c_void_p, c_int32, c_void_p]
    L.ecspmv_stream_read_sliced.argtypes = [c_void_p, c_size_t, c_void_p, c_int32, c_int32, c_void_p]
    L.ecspmv_empty_launch.argtypes = [c_void_p, c_int32, c_int32, c_int32, c_void_p]
    L.ecspmv_strerror.argtypes = [c_int]
    L.ecspmv_strerror.restype = c_char_p
    L.ecspmv_last_hip_error.argtypes = []
    for name in EXPORTS:
        fn = getattr(L, name)
        if name not in ("ecspmv_destroy", "ecspmv_csr_destroy", "ecspmv_strerror"):
            fn.restype = c_int
    _lib = L
    return L


def _check(status: int, where: str) -> None:
    if status != OK:
        raise EcspmvError(status, where)


def make_opts(max_granularity: int = 0, num_panels: int = 0, num_threads: int = 0, threads_per_wg: int = 0,
              max_rounds: int = 0, delta_bits: int = 0, flags: int = 0) -> BuildOpts:
    o = BuildOpts()
    o.struct_size = ctypes.sizeof(BuildOpts)
    o.delta_bits, o.max_granularity, o.max_rounds = delta_bits, max_granularity, max_rounds
    o.num_panels, o.num_threads, o.threads_per_wg, o.flags = num_panels, num_threads, threads_per_wg, flags
    return o


def _as_u16_matrix(W: np.ndarray) -> np.ndarray:
    if W.dtype == np.float16:
        W = W.view(np.uint16)
    if W.dtype != np.uint16 or W.ndim != 2:
        raise TypeError("W must be a 2-D float16 / uint16 array")
    if W.strides[1] != 2 or W.strides[0] % 2 or W.strides[0] < 2 * W.shape[1]:
        W = np.ascontiguousarray(W)
    return W


class Matrix:
    """Handle of one EC-CSR matrix (wraps ecspmv_matrix*)."""

    def __init__(self, handle: int):
        self._h = c_void_p(handle)
        self.d_image = None          # whatever object owns the device buffer (kept alive here)

    def __del__(self):
        try:
            self.destroy()
        except Exception:       # interpreter shutdown: the module's globals may be gone already
            pass

    def destroy(self):
        if getattr(self, "_h", None) is not None and self._h.value:
            lib().ecspmv_destroy(self._h)
            self._h = c_void_p(0)
        self.d_image = None

    # names follow the C ABI
    def ecspmv_stats(self) -> Stats:
        st = Stats()
        st.struct_size = ctypes.sizeof(Stats)
        _check(lib().ecspmv_stats(self._h, byref(st)), "ecspmv_stats")
        return st

    def ecspmv_decode(self):
        n = c_int64(0)
        _check(lib().ecspmv_decode(self._h, byref(n), None, None, None), "ecspmv_decode")
        rows = np.empty(n.value, dtype=np.int32)
        cols = np.empty(n.value, dtype=np.int32)
        vals = np.empty(n.value, dtype=np.uint16)
        _check(lib().ecspmv_decode(self._h, byref(n), rows.ctypes.data, cols.ctypes.data, vals.ctypes.data),
               "ecspmv_decode")
        return rows, cols, vals

    def ecspmv_decode_f32(self):
        n = c_int64(0)
        _check(lib().ecspmv_decode_f32(self._h, byref(n), None, None, None), "ecspmv_decode_f32")
        rows = np.empty(n.value, dtype=np.int32)
        cols = np.empty(n.value, dtype=np.int32)
        vals = np.empty(n.value, dtype=np.uint32)            # FP32 bit patterns
        _check(lib().ecspmv_decode_f32(self._h, byref(n), rows.ctypes.data, cols.ctypes.data, vals.ctypes.data),
               "ecspmv_decode_f32")
        return rows, cols, vals

    def ecspmv_block_sets(self):
        nu, nr = c_int64(0), c_int64(0)
        _check(lib().ecspmv_block_sets(self._h, byref(nu), byref(nr), None, None, None), "ecspmv_block_sets")
        g = np.empty(nu.value, dtype=np.int32)
        rows = np.empty(nr.value, dtype=np.int32)
        cols = np.empty((nu.value, 64), dtype=np.int32)
        if nu.value:
            _check(lib().ecspmv_block_sets(self._h, byref(nu), byref(nr), g.ctypes.data, rows.ctypes.data,
                                           cols.ctypes.data), "ecspmv_block_sets")
        return g, rows, cols

    def ecspmv_device_bytes(self) -> int:
        b = c_size_t(0)
        _check(lib().ecspmv_device_bytes(self._h, byref(b)), "ecspmv_device_bytes")
        return int(b.value)

    def ecspmv_export_image(self) -> np.ndarray:
        n = self.ecspmv_device_bytes()
        out = np.empty(n, dtype=np.uint8)
        _check(lib().ecspmv_export_image(self._h, out.ctypes.data, n), "ecspmv_export_image")
        return out

    def ecspmv_upload(self, d_ptr: int, nbytes: int, stream: int = 0, keepalive=None) -> None:
        _check(lib().ecspmv_upload(self._h, c_void_p(d_ptr), nbytes, c_void_p(stream)), "ecspmv_upload")
        self.d_image = keepalive

    def ecspmv_run(self, d_x: int, d_y: int, stream: int = 0) -> None:
        _check(lib().ecspmv_run(self._h, c_void_p(d_x), c_void_p(d_y), c_void_p(stream)), "ecspmv_run")

    def ecspmv_run_multi(self, d_X: int, d_Y: int, nb: int, stream: int = 0) -> None:
        _check(lib().ecspmv_run_multi(self._h, c_void_p(d_X), c_void_p(d_Y), c_int32(nb), c_void_p(stream)),
               "ecspmv_run_multi")


class Batch:
    """Pre-marshalled argument arrays of ecspmv_run_batch (handles, x pointers, y pointers)."""

    def __init__(self, mats, d_xs, d_ys):
        assert len(mats) == len(d_xs) == len(d_ys) and len(mats) > 0
        n = len(mats)
        self.count = n
        self._mats = list(mats)                     # keep the handles alive
        self._h = (c_void_p * n)(*[m._h.value for m in mats])
        self._x = (c_void_p * n)(*[int(p) for p in d_xs])
        self._y = (c_void_p * n)(*[int(p) for p in d_ys])

    def ecspmv_run_batch(self, stream: int = 0) -> None:
        _check(lib().ecspmv_run_batch(self._h, self._x, self._y, self.count, c_void_p(stream)), "ecspmv_run_batch")


def ecspmv_run_batch(mats, d_xs, d_ys, stream: int = 0) -> None:
    Batch(mats, d_xs, d_ys).ecspmv_run_batch(stream)


def ecspmv_build_dense(W: np.ndarray, opts: BuildOpts | None = None) -> Matrix:
    Wu = _as_u16_matrix(W)
    m, n = Wu.shape
    out = c_void_p(0)
    _check(lib().ecspmv_build_dense(Wu.ctypes.data, m, n, Wu.strides[0] // 2, byref(opts) if opts else None,
                                    byref(out)), "ecspmv_build_dense")
    return Matrix(out.value)


def ecspmv_build_dense_f32(W: np.ndarray, opts: BuildOpts | None = None) -> Matrix:
    if W.dtype != np.float32 or W.ndim != 2:
        raise TypeError("W must be a 2-D float32 array")
    if W.strides[1] != 4 or W.strides[0] % 4 or W.strides[0] < 4 * W.shape[1]:
        W = np.ascontiguousarray(W)
    m, n = W.shape
    out = c_void_p(0)
    _check(lib().ecspmv_build_dense_f32(W.ctypes.data, m, n, W.strides[0] // 4, byref(opts) if opts else None,
                                        byref(out)), "ecspmv_build_dense_f32")
    return Matrix(out.value)


def ecspmv_build_csr_f32(rowptr: np.ndarray, col: np.ndarray, val: np.ndarray, m: int, n: int,
                         opts: BuildOpts | None = None) -> Matrix:
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val, dtype=np.float32)
    out = c_void_p(0)
    _check(lib().ecspmv_build_csr_f32(rowptr.ctypes.data, col.ctypes.data, val.ctypes.data, m, n,
                                      byref(opts) if opts else None, byref(out)), "ecspmv_build_csr_f32")
    return Matrix(out.value)


def ecspmv_build_csr(rowptr: np.ndarray, col: np.ndarray, val: np.ndarray, m: int, n: int,
                     opts: BuildOpts | None = None) -> Matrix:
    rowptr = np.ascontiguousarray(rowptr, dtype=np.int64)
    col = np.ascontiguousarray(col, dtype=np.int32)
    val = np.ascontiguousarray(val.view(np.uint16) if val.dtype == np.float16 else val, dtype=np.uint16)
    out = c_void_p(0)
    _check(lib().ecspmv_build_csr(rowptr.ctypes.data, col.ctypes.data, val.ctypes.data, m, n,
                                  byref(opts) if opts else None, byref(out)), "ecspmv_build_csr")
    return Matrix(out.value)


class CsrMatrix:
    """Handle of the plain-CSR comparison matrix (wraps ecspmv_csr*)."""

    def __init__(self, handle: int):
        self._h = c_void_p(handle)
        self.d_buf = None

    def __del__(self):
        try:
            if getattr(self, "_h", None) is not None and self._h.value:
                lib().ecspmv_csr_destroy(self._h)
                self._h = c_void_p(0)
        except Exception:       # interpreter shutdown: the module's globals may be gone already
            pass

    def ecspmv_csr_device_bytes(self) -> int:
        b = c_size_t(0)
        _check(lib().ecspmv_csr_device_bytes(self._h, byref(b)), "ecspmv_csr_device_bytes")
        return int(b.value)

    def ecspmv_csr_upload(self, d_ptr: int, nbytes: int, stream: int = 0, keepalive=None) -> None:
        _check(lib().ecspmv_csr_upload(self._h, c_void_p(d_ptr), nbytes, c_void_p(stream)), "ecspmv_csr_upload")
        self.d_buf = keepalive

    def ecspmv_csr_run(self, d_x: int, d_y: int, stream: int = 0) -> None:
        _check(lib().ecspmv_csr_run(self._h, c_void_p(d_x), c_void_p(d_y), c_void_p(stream)), "ecspmv_csr_run")


def ecspmv_csr_build_dense(W: np.ndarray) -> CsrMatrix:
    Wu = _as_u16_matrix(W)
    m, n = Wu.shape
    out = c_void_p(0)
    _check(lib().ecspmv_csr_build_dense(Wu.ctypes.data, m, n, Wu.strides[0] // 2, byref(out)), "ecspmv_csr_build_dense")
    return CsrMatrix(out.value)


def ecspmv_stream_read(d_buf: int, nbytes: int, d_out: int, num_wg: int, stream: int = 0) -> None:
    _check(lib().ecspmv_stream_read(c_void_p(d_buf), nbytes, c_void_p(d_out), num_wg, c_void_p(stream)),
           "ecspmv_stream_read")


def ecspmv_stream_read_sliced(d_buf: int, nbytes: int, d_out: int, num_wg: int, threads_per_wg: int,
                              stream: int = 0) -> None:
    _check(lib().ecspmv_stream_read_sliced(c_void_p(d_buf), nbytes, c_void_p(d_out), num_wg, threads_per_wg,
                                           c_void_p(stream)), "ecspmv_stream_read_sliced")


def ecspmv_empty_launch(d_out: int, num_wg: int, threads_per_wg: int, count: int = 1, stream: int = 0) -> None:
    _check(lib().ecspmv_empty_launch(c_void_p(d_out), num_wg, threads_per_wg, count, c_void_p(stream)),
           "ecspmv_empty_launch")
