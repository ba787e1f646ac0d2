"""CPU oracle for batch-1 SpMV over a dense masked FP16 matrix -- TEST INFRASTRUCTURE.

Only tests, the smoke check and the bench's cpu_baseline leg may import this module.
It shares no code with the EC-CSR encoder, the HIP kernels or their Python binding.

Defined result (paper Section 1, problem statement; Section 2.1, W is (M, K);
Section 2.2, batch size 1 turns the GEMM into a matrix-vector product):

    y[i] = sum_j W[i, j] * x[j]          S[i] = sum_j |W[i, j] * x[j]|

with W and x FP16 values converted exactly to FP64, FP64 products and sums, columns in
natural order.  `spmv_oracle` runs the C implementation in spmv_oracle.c (same
definition, threads over rows); `spmv_oracle_py` is the same definition as Python loops
for tiny cases.  `pattern_triples` states what "the nonzeros of W" means for the
format's round-trip check: entries whose FP16 bits differ from +0 and -0.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "spmv_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_spmv.so")
_lib = None


def build_oracle(force: bool = False) -> str:
    """Compile spmv_oracle.c with gcc into oracle/liboracle_spmv.so."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build_oracle()
        lib = ctypes.CDLL(_LIB)
        lib.oracle_spmv_f64.restype = ctypes.c_int
        lib.oracle_spmv_f64.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                        ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_spmv_f64_from_f32.restype = ctypes.c_int
        lib.oracle_spmv_f64_from_f32.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
                                                 ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        lib.oracle_half_to_double.restype = ctypes.c_double
        lib.oracle_half_to_double.argtypes = [ctypes.c_uint16]
        _lib = lib
    return _lib


def half_to_double(bits: int) -> float:
    """The oracle's own FP16 -> FP64 conversion of one bit pattern."""
    return float(_load().oracle_half_to_double(int(bits) & 0xFFFF))


def spmv_oracle(W: np.ndarray, x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(y_ref, S), both float64 of length m, from dense FP16 W (m, n) and FP16 x (n,)."""
    y, S, _ = spmv_oracle_threads(W, x)
    return y, S


def spmv_oracle_threads(W: np.ndarray, x: np.ndarray):
    """Same as spmv_oracle, also returning the number of threads the C loop used."""
    assert W.dtype == np.float16 and x.dtype == np.float16 and W.ndim == 2 and x.ndim == 1
    m, n = W.shape
    assert x.shape[0] == n
    Wc = np.ascontiguousarray(W)
    xc = np.ascontiguousarray(x)
    y = np.zeros(m, dtype=np.float64)
    S = np.zeros(m, dtype=np.float64)
    if m == 0:
        return y, S, 1
    t = _load().oracle_spmv_f64(Wc.ctypes.data, m, n, n, xc.ctypes.data, y.ctypes.data, S.ctypes.data)
    if t < 0:
        raise MemoryError("oracle_spmv_f64")
    return y, S, int(t)


def spmv_oracle_f32(W: np.ndarray, x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """(y_ref, S), both float64 of length m, from dense FP32 W (m, n) and FP32 x (n,): the FP32 precision of the paper."""
    assert W.dtype == np.float32 and x.dtype == np.float32 and W.ndim == 2 and x.ndim == 1
    m, n = W.shape
    assert x.shape[0] == n
    Wc = np.ascontiguousarray(W)
    xc = np.ascontiguousarray(x)
    y = np.zeros(m, dtype=np.float64)
    S = np.zeros(m, dtype=np.float64)
    if m:
        _load().oracle_spmv_f64_from_f32(Wc.ctypes.data, m, n, n, xc.ctypes.data, y.ctypes.data, S.ctypes.data)
    return y, S


def pattern_triples_f32(W: np.ndarray):
    """(rows, cols, FP32 bit patterns) of the stored entries of an FP32 W (neither +0 nor -0), sorted by (row, col)."""
    assert W.dtype == np.float32
    bits = np.ascontiguousarray(W).view(np.uint32)
    rows, cols = np.nonzero((bits & 0x7FFFFFFF) != 0)
    return rows.astype(np.int32), cols.astype(np.int32), bits[rows, cols].copy()


def spmv_oracle_py(W: np.ndarray, x: np.ndarray) -> Tuple[np.ndarray, np.ndarray]:
    """The definition as plain Python loops over FP64 scalars (tiny inputs only)."""
    assert W.dtype == np.float16 and x.dtype == np.float16
    m, n = W.shape
    y = np.zeros(m, dtype=np.float64)
    S = np.zeros(m, dtype=np.float64)
    for i in range(m):
        acc = 0.0
        mag = 0.0
        for j in range(n):
            p = float(W[i, j]) * float(x[j])      # FP16 -> Python float (FP64) is exact
            acc += p
            mag += abs(p)
        y[i] = acc
        S[i] = mag
    return y, S


def pattern_triples(W: np.ndarray):
    """(rows, cols, fp16 bit patterns) of the stored entries of W, sorted by (row, col).

    An entry is stored iff its FP16 bits are neither +0 (0x0000) nor -0 (0x8000)."""
    assert W.dtype == np.float16
    bits = np.ascontiguousarray(W).view(np.uint16)
    rows, cols = np.nonzero((bits & 0x7FFF) != 0)
    return rows.astype(np.int32), cols.astype(np.int32), bits[rows, cols].copy()


def within_band(y: np.ndarray, y_ref: np.ndarray, S: np.ndarray, rel: float = 2e-3, abs_: float = 1e-6):
    """Row-wise acceptance test |y - y_ref| <= rel * S + abs_; returns (ok, worst ratio)."""
    err = np.abs(np.asarray(y, dtype=np.float64) - y_ref)
    lim = rel * S + abs_
    ratio = float(np.max(err / lim)) if err.size else 0.0
    return bool(np.all(err <= lim)), ratio
