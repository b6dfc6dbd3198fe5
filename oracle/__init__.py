"""TEST ORACLE -- not part of the product.

Plain, slow, obviously-correct CPU implementation of what the GPU path computes:
y = A*x for a CSR matrix (paper, Section I; the operators of Table II only
re-lay-out A or re-associate the row sums, Section IV-A).  Only tests, the smoke
check and the benchmark's CPU-baseline leg may import this package.  It imports
nothing from the GPU library and shares no code with it.

  spmv(...)        working-precision, sequential left-to-right row sums
  spmv_wide(...)   wide accumulation (long double for fp64, double for fp32), float64 result
  abs_bound(...)   (|A| |x|)_i, the scale of the tolerance |y - y_ref|_i <= tau * (|A||x|)_i
  check(...)       applies that tolerance test; tau = 1e-12 (fp64) / 1e-5 (fp32)
  dense_exact(...) brute-force dense mat-vec in exact rational arithmetic (tiny inputs only)

Parity pins: every function here is pinned by tests/test_oracle_pins.py against dense
brute force, closed forms, exact integer arithmetic and SciPy.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "csr_spmv_ref.c")
_LIB = os.path.join(_HERE, "liboracle.so")

TAU = {np.dtype(np.float64): 1e-12, np.dtype(np.float32): 1e-5}


def build(force: bool = False) -> str:
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _LIB])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        for name in ("csr_spmv_f64_work", "csr_spmv_f32_work", "csr_spmv_f64_wide",
                     "csr_spmv_f32_wide", "csr_abs_f64", "csr_abs_f32"):
            fn = getattr(lib, name)
            fn.restype = None
            fn.argtypes = [ctypes.c_int64] + [ctypes.c_void_p] * 5 + [ctypes.c_int]
        _lib = lib
    return _lib


def _prep(row_ptr, col_idx, values, x):
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    values = np.ascontiguousarray(values)
    dt = values.dtype
    if dt not in TAU:
        raise TypeError("values must be float32 or float64")
    x = np.ascontiguousarray(x, dtype=dt)
    nrows = row_ptr.size - 1
    if nrows < 0 or row_ptr[0] != 0 or row_ptr[-1] != col_idx.size or col_idx.size != values.size:
        raise ValueError("inconsistent CSR arrays")
    if col_idx.size and (col_idx.min() < 0 or col_idx.max() >= x.size):
        raise ValueError("column index out of range for x")
    return nrows, row_ptr, col_idx, values, x, dt


def _call(kind, out_dtype, row_ptr, col_idx, values, x, threads):
    nrows, row_ptr, col_idx, values, x, dt = _prep(row_ptr, col_idx, values, x)
    suffix = "f64" if dt == np.float64 else "f32"
    y = np.empty(nrows, dtype=out_dtype if out_dtype is not None else dt)
    getattr(_load(), kind.format(suffix))(nrows, row_ptr.ctypes.data, col_idx.ctypes.data,
                                          values.ctypes.data, x.ctypes.data, y.ctypes.data, threads)
    return y


def spmv(row_ptr, col_idx, values, x, threads: int = 1) -> np.ndarray:
    """y = A*x accumulated in the dtype of `values` (float32 or float64)."""
    return _call("csr_spmv_{}_work", None, row_ptr, col_idx, values, x, threads)


def spmv_wide(row_ptr, col_idx, values, x, threads: int = 1) -> np.ndarray:
    """y = A*x with wide accumulation; always returns float64."""
    return _call("csr_spmv_{}_wide", np.float64, row_ptr, col_idx, values, x, threads)


def abs_bound(row_ptr, col_idx, values, x, threads: int = 1) -> np.ndarray:
    """(|A| |x|)_i as float64."""
    return _call("csr_abs_{}", np.float64, row_ptr, col_idx, values, x, threads)


def check(y, row_ptr, col_idx, values, x, tau=None, threads: int = 1):
    """Tolerance test of a computed y against the wide oracle.

    Returns (ok, worst) where worst = max_i |y_i - y_ref_i| / (tau * (|A||x|)_i) over rows with a
    non-zero bound; rows whose bound is zero must be exactly zero (either sign).
    """
    values = np.asarray(values)
    tau = TAU[values.dtype] if tau is None else tau
    ref = spmv_wide(row_ptr, col_idx, values, x, threads)
    bnd = abs_bound(row_ptr, col_idx, values, x, threads)
    y = np.asarray(y, dtype=np.float64)
    if y.shape != ref.shape:
        return False, float("inf")
    if not np.all(np.isfinite(y)):
        return False, float("inf")
    err = np.abs(y - ref)
    zero = bnd == 0
    if np.any(err[zero] != 0):
        return False, float("inf")
    ratio = np.zeros_like(err)
    np.divide(err, tau * bnd, out=ratio, where=~zero)
    worst = float(ratio.max()) if ratio.size else 0.0
    return worst <= 1.0, worst


def dense_exact(nrows, ncols, row_ptr, col_idx, values, x):
    """Brute force: build the dense matrix (duplicates add) and multiply, all in exact rational
    arithmetic.  Pure Python, for tiny inputs.  Returns a list of Fractions."""
    dense = [[Fraction(0)] * ncols for _ in range(nrows)]
    for i in range(nrows):
        for k in range(int(row_ptr[i]), int(row_ptr[i + 1])):
            dense[i][int(col_idx[k])] += Fraction(float(values[k]))
    xs = [Fraction(float(v)) for v in x]
    return [sum((dense[i][j] * xs[j] for j in range(ncols)), Fraction(0)) for i in range(nrows)]
