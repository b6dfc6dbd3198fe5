"""Seeded synthetic inputs for the SpMV workloads (CSR matrices and dense vectors).

This package only *generates data*.  It contains none of the SpMV method's
arithmetic and imports neither the test oracle nor the GPU library; both sides
of a parity test draw their inputs from here.

The five matrix families stand in for the SuiteSparse test set the paper
evaluates on (Section VII-A), which is not available offline.  Each family is a
function of its size parameters, so tests can run scaled-down versions of the
exact recipe the benchmark times at full size.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "gen.c")
_LIB = os.path.join(_HERE, "libspmvgen.so")

BASE_SEED = 20221113


def build(force: bool = False) -> str:
    """Compile the generator (gcc, OpenMP).  Returns the path of the shared library."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i64, u64, dbl, ci = ctypes.c_int64, ctypes.c_uint64, ctypes.c_double, ctypes.c_int
        vp = ctypes.c_void_p
        lib.gen_row_ptr.restype = i64
        lib.gen_row_ptr.argtypes = [ci, i64, i64, i64, i64, i64, dbl, dbl, u64, vp]
        lib.gen_fill.restype = ci
        lib.gen_fill.argtypes = [ci, i64, i64, i64, i64, i64, dbl, dbl, u64, ci, ci, vp, vp, vp]
        lib.gen_vector.restype = None
        lib.gen_vector.argtypes = [i64, u64, ci, ci, vp]
        lib.gen_hybrid_heavy_rows.restype = None
        lib.gen_hybrid_heavy_rows.argtypes = [i64, i64, u64, vp]
        _lib = lib
    return _lib


@dataclass
class CsrMatrix:
    """Plain CSR triple on the host: int32 row_ptr / col_idx, float64 values."""
    name: str
    nrows: int
    ncols: int
    row_ptr: np.ndarray
    col_idx: np.ndarray
    values: np.ndarray
    meta: dict = field(default_factory=dict)

    @property
    def nnz(self) -> int:
        return int(self.row_ptr[-1])

    def astype(self, dtype) -> "CsrMatrix":
        return CsrMatrix(self.name, self.nrows, self.ncols, self.row_ptr, self.col_idx,
                         self.values.astype(dtype), dict(self.meta))


_KINDS = {"uniform": 1, "laplace2d": 2, "powerlaw": 3, "fem3": 4, "hybrid": 5}


def _generate(name, kind, n, p=(0, 0, 0, 0), d=(0.0, 0.0), seed=BASE_SEED, integer=False, vmax=3, meta=None):
    lib = _load()
    rp64 = np.empty(n + 1, dtype=np.int64)
    nnz = lib.gen_row_ptr(kind, n, p[0], p[1], p[2], p[3], d[0], d[1], seed, rp64.ctypes.data)
    if nnz < 0:
        raise ValueError(f"bad generator parameters for {name}")
    if nnz >= 2 ** 31:
        raise ValueError("nnz does not fit int32")
    col = np.empty(nnz, dtype=np.int32)
    val = np.empty(nnz, dtype=np.float64)
    rc = lib.gen_fill(kind, n, p[0], p[1], p[2], p[3], d[0], d[1], seed, int(integer), vmax,
                      rp64.ctypes.data, col.ctypes.data, val.ctypes.data)
    if rc != 0:
        raise ValueError(f"generator failed for {name}")
    return CsrMatrix(name, n, n, rp64.astype(np.int32), col, val, meta or {})


def vector(n: int, seed: int = BASE_SEED + 100, integer: bool = False, vmax: int = 3) -> np.ndarray:
    """Dense vector: uniform in [-1, 1), or non-zero integers in [-vmax, vmax]."""
    x = np.empty(n, dtype=np.float64)
    _load().gen_vector(n, seed, int(integer), vmax, x.ctypes.data)
    return x


# --- the five configurations ----------------------------------------------------------

def uniform(n=10_000, k=10, seed=BASE_SEED + 1, **kw):
    """C1: n x n, exactly k non-zeros per row, distinct uniform columns, ascending."""
    return _generate("uniform", 1, n, (k, 0, 0, 0), seed=seed, **kw)


def laplace2d(g=1024, amp=0.01, seed=BASE_SEED + 2, **kw):
    """C2: 5-point stencil on a g x g grid without wrap-around; diagonal 4, off-diagonals -1,
    every stored entry perturbed by an independent uniform in [-amp, amp] (none in integer mode)."""
    return _generate("laplace2d", 2, g * g, (g, 0, 0, 0), (amp, 0.0), seed=seed, meta={"g": g}, **kw)


# scale of the shifted-Pareto law so that the mean row length is 16 at n = 4,194,304 with
# exponent 2.1 and cap 100,000 under this generator's random stream (found by bisection)
POWERLAW_SCALE = 2.33


def powerlaw(n=4_194_304, cap=100_000, scale=POWERLAW_SCALE, exponent=2.1, seed=BASE_SEED + 3, **kw):
    """C3: row length L = clamp(floor(scale*(U^(-1/(exponent-1)) - 1)) + 1, 1, cap); tail density
    ~ L^-exponent, minimum 1.  Columns distinct uniform, ascending."""
    return _generate("powerlaw", 3, n, (cap, 0, 0, 0), (scale, exponent), seed=seed, **kw)


def fem3(nb=1_000_000, kmin=9, kmax=27, window=2000, seed=BASE_SEED + 4, **kw):
    """C4: nb block rows of dense 3x3 blocks, emitted as scalar CSR (n = 3*nb).  Each block row has
    k ~ U{kmin..kmax} blocks: the diagonal block plus k-1 distinct block columns uniform in
    [i-window, i+window] clipped to the matrix."""
    return _generate("fem3", 4, 3 * nb, (kmin, kmax, window, 0), seed=seed,
                     meta={"nb": nb, "block": 3}, **kw)


def hybrid(n=8_388_608, n_heavy=1000, heavy_len=100_000, lo=2, hi=8, seed=BASE_SEED + 5, **kw):
    """C5: n_heavy uniformly placed rows with heavy_len non-zeros, every other row U{lo..hi};
    columns distinct uniform.  meta['heavy_rows'] holds the sorted heavy row ids."""
    ids = np.empty(n_heavy, dtype=np.int32)
    _load().gen_hybrid_heavy_rows(n, n_heavy, seed, ids.ctypes.data)
    return _generate("hybrid", 5, n, (n_heavy, heavy_len, lo, hi), seed=seed,
                     meta={"heavy_rows": ids}, **kw)


FULL = {"C1": uniform, "C2": laplace2d, "C3": powerlaw, "C4": fem3, "C5": hybrid}

# scaled-down versions of the same recipes: several tiles, ragged tails, seconds on a CPU
SMALL = {
    "C1": lambda **kw: uniform(n=10_000, k=10, **kw),
    "C2": lambda **kw: laplace2d(g=67, **kw),
    "C3": lambda **kw: powerlaw(n=70_001, cap=9_000, **kw),
    "C4": lambda **kw: fem3(nb=10_007, window=500, **kw),
    "C5": lambda **kw: hybrid(n=130_003, n_heavy=7, heavy_len=20_000, **kw),
}
