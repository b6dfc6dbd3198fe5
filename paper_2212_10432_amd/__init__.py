"""MI355X-native SpMV plan/search library: Python binding of the C ABI in include/spmv.h.

The binding only marshals arguments (ctypes); every step of the path -- census, format
construction, search, kernels -- runs inside libspmv_mi355.so.  PyTorch is used by callers for
device buffers and streams only.  There is no CPU fallback: if the shared library is missing or
cannot be loaded, importing this package's functions raises.
"""
from __future__ import annotations

import ctypes
import json
import os

import numpy as np

from . import build as _build

SPMV_F32, SPMV_F64 = 0, 1
SPMV_OK, SPMV_ERR_INVALID_ARG, SPMV_ERR_BAD_CSR, SPMV_ERR_UNSUPPORTED = 0, 1, 2, 3
SPMV_ERR_ALLOC, SPMV_ERR_HIP, SPMV_ERR_INTERNAL = 4, 5, 6
_STATUS = {0: "OK", 1: "INVALID_ARG", 2: "BAD_CSR", 3: "UNSUPPORTED", 4: "ALLOC", 5: "HIP", 6: "INTERNAL"}

EXPORTS = ["spmv_plan_create", "spmv_run", "spmv_run_noalloc", "spmv_run_multi", "spmv_plan_save", "spmv_plan_load", "spmv_cost_predict", "spmv_fit_array", "spmv_plan_jit_check", "spmv_run_timed", "spmv_plan_time", "spmv_plan_time_launches", "spmv_plan_destroy", "spmv_plan_describe",
           "spmv_plan_array_count", "spmv_plan_array_info", "spmv_plan_array_copy", "spmv_plan_bytes",
           "spmv_plan_launch_count", "spmv_plan_launch_name", "spmv_last_error", "spmv_mm_read", "spmv_mm_free", "spmv_stream_ceiling"]


class SpmvError(RuntimeError):
    def __init__(self, status: int, message: str):
        super().__init__(f"SPMV_ERR_{_STATUS.get(status, status)}: {message}")
        self.status = status
        self.message = message


_ALLOC_FN = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p)
_FREE_FN = ctypes.CFUNCTYPE(None, ctypes.c_void_p, ctypes.c_void_p)


class spmv_options_t(ctypes.Structure):
    _fields_ = [("force_plan", ctypes.c_char_p), ("search_budget_ms", ctypes.c_double),
                ("search_repeats", ctypes.c_int), ("host_threads", ctypes.c_int),
                ("dev_alloc", _ALLOC_FN), ("dev_free", _FREE_FN), ("user", ctypes.c_void_p),
                ("verbosity", ctypes.c_int), ("host_only", ctypes.c_int),
                ("cost_model_path", ctypes.c_char_p), ("cost_log_path", ctypes.c_char_p), ("search_cold", ctypes.c_int)]


# corpus of timed candidates shipped with the package: the search's cost model is trained from it
COST_CORPUS = os.path.join(os.path.dirname(os.path.abspath(__file__)), "cost_corpus.tsv")


_lib = None


def lib_path() -> str:
    return _build.LIB


def load():
    """Load libspmv_mi355.so (building it if no built library is present).  Raises on failure."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build()
    try:
        import torch  # noqa: F401  -- makes the process use the HIP runtime PyTorch ships
    except ImportError:
        pass
    lib = ctypes.CDLL(_build.LIB)
    vp, i64, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int
    P = ctypes.POINTER
    lib.spmv_plan_create.restype = ci
    lib.spmv_plan_create.argtypes = [P(vp), i64, i64, i64, vp, vp, vp, ci, P(spmv_options_t)]
    lib.spmv_run.restype = ci
    lib.spmv_run.argtypes = [vp, vp, vp, vp]
    lib.spmv_run_noalloc.restype = ci
    lib.spmv_run_noalloc.argtypes = [vp, vp, vp, vp]
    lib.spmv_run_multi.restype = ci
    lib.spmv_run_multi.argtypes = [vp, vp, i64, vp, i64, ci, vp]
    lib.spmv_plan_save.restype = ci
    lib.spmv_plan_save.argtypes = [vp, ctypes.c_char_p]
    lib.spmv_plan_load.restype = ci
    lib.spmv_plan_load.argtypes = [P(vp), ctypes.c_char_p, P(spmv_options_t)]
    lib.spmv_cost_predict.restype = ci
    lib.spmv_cost_predict.argtypes = [vp, ctypes.c_char_p, ctypes.c_char_p, P(ctypes.c_double), P(i64)]
    lib.spmv_fit_array.restype = ci
    lib.spmv_fit_array.argtypes = [vp, ci, i64, ctypes.c_char_p, ctypes.c_size_t]
    lib.spmv_plan_jit_check.restype = ci
    lib.spmv_plan_jit_check.argtypes = [vp, P(ci), ctypes.c_char_p, ctypes.c_size_t]
    lib.spmv_run_timed.restype = ci
    lib.spmv_run_timed.argtypes = [vp, vp, vp, vp, P(ctypes.c_float)]
    lib.spmv_plan_time_launches.restype = ci
    lib.spmv_plan_time_launches.argtypes = [vp, vp, vp, vp, ci, P(ctypes.c_float)]
    lib.spmv_plan_time.restype = ci
    lib.spmv_plan_time.argtypes = [vp, vp, vp, vp, ci, P(ctypes.c_double)]
    lib.spmv_plan_destroy.restype = ci
    lib.spmv_plan_destroy.argtypes = [vp]
    lib.spmv_plan_describe.restype = ci
    lib.spmv_plan_describe.argtypes = [vp, ctypes.c_char_p, ctypes.c_size_t, P(ctypes.c_size_t)]
    lib.spmv_plan_array_count.restype = ci
    lib.spmv_plan_array_count.argtypes = [vp, P(ci)]
    lib.spmv_plan_array_info.restype = ci
    lib.spmv_plan_array_info.argtypes = [vp, ci, P(ctypes.c_char_p), P(ci), P(i64)]
    lib.spmv_plan_array_copy.restype = ci
    lib.spmv_plan_array_copy.argtypes = [vp, ci, vp]
    lib.spmv_plan_bytes.restype = ci
    lib.spmv_plan_bytes.argtypes = [vp, P(i64), P(i64)]
    lib.spmv_plan_launch_count.restype = ci
    lib.spmv_plan_launch_count.argtypes = [vp, P(ci)]
    lib.spmv_plan_launch_name.restype = ci
    lib.spmv_plan_launch_name.argtypes = [vp, ci, P(ctypes.c_char_p)]
    lib.spmv_last_error.restype = ctypes.c_char_p
    lib.spmv_last_error.argtypes = []
    lib.spmv_mm_read.restype = ci
    lib.spmv_mm_read.argtypes = [ctypes.c_char_p, ci, P(i64), P(i64), P(i64), P(vp), P(vp), P(vp)]
    lib.spmv_mm_free.restype = ci
    lib.spmv_mm_free.argtypes = [vp, vp, vp]
    lib.spmv_stream_ceiling.restype = ci
    lib.spmv_stream_ceiling.argtypes = [ctypes.c_size_t, ci, vp, P(ctypes.c_double), P(ctypes.c_double)]
    _lib = lib
    return lib


def spmv_last_error() -> str:
    return load().spmv_last_error().decode()


def _check(status: int):
    if status != SPMV_OK:
        raise SpmvError(status, spmv_last_error())


def _dtype_code(dt) -> int:
    dt = np.dtype(dt)
    if dt == np.float64:
        return SPMV_F64
    if dt == np.float32:
        return SPMV_F32
    raise SpmvError(SPMV_ERR_UNSUPPORTED, f"dtype {dt} (float32 or float64 only)")


# ---- functions named after the C ABI ---------------------------------------------------------

def spmv_plan_create(nrows, ncols, row_ptr, col_idx, values, *, force_plan=None,
                     search_budget_ms=0.0, search_repeats=0, host_threads=0, verbosity=0,
                     host_only=False, nnz=None, allocator=None, cost_model="default", cost_log=None,
                     search_cold=False) -> int:
    """Returns an opaque plan handle (int).  row_ptr / col_idx / values are host NumPy arrays.
    allocator = (alloc(nbytes) -> device address or 0, free(address)): Python callables the library
    uses for every device array of the plan (kept alive until spmv_plan_destroy)."""
    lib = load()
    row_ptr = np.ascontiguousarray(row_ptr, dtype=np.int32)
    col_idx = np.ascontiguousarray(col_idx, dtype=np.int32)
    values = np.ascontiguousarray(values)
    code = _dtype_code(values.dtype)
    if nnz is None:
        nnz = int(values.size)
    # the library reads nrows + 1 offsets and nnz columns and values through raw pointers
    if nrows < 0 or row_ptr.size != nrows + 1:
        raise SpmvError(SPMV_ERR_INVALID_ARG, f"row_ptr has {row_ptr.size} entries, nrows + 1 = {nrows + 1} expected")
    if nnz < 0 or col_idx.size < nnz or values.size < nnz:
        raise SpmvError(SPMV_ERR_INVALID_ARG, f"col_idx / values hold {col_idx.size} / {values.size} entries, nnz = {nnz}")
    opts = spmv_options_t()
    opts.force_plan = force_plan.encode() if force_plan else None
    opts.search_budget_ms = float(search_budget_ms)
    opts.search_repeats = int(search_repeats)
    opts.host_threads = int(host_threads)
    opts.verbosity = int(verbosity)
    opts.host_only = int(bool(host_only))
    if cost_model == "default":
        cost_model = COST_CORPUS if os.path.exists(COST_CORPUS) else None
    opts.cost_model_path = os.fsencode(cost_model) if cost_model else None
    opts.cost_log_path = os.fsencode(cost_log) if cost_log else None
    opts.search_cold = int(bool(search_cold))
    keep = None
    if allocator is not None:
        alloc_py, free_py = allocator
        keep = (_ALLOC_FN(lambda nbytes, user: alloc_py(nbytes) or None), _FREE_FN(lambda ptr, user: free_py(ptr)))
        opts.dev_alloc, opts.dev_free = keep
    handle = ctypes.c_void_p()
    _check(lib.spmv_plan_create(ctypes.byref(handle), nrows, ncols, nnz, row_ptr.ctypes.data,
                                col_idx.ctypes.data, values.ctypes.data, code, ctypes.byref(opts)))
    if keep is not None:
        _callbacks[handle.value] = keep      # the plan calls dev_free when it is destroyed
    return handle.value


_callbacks = {}


def spmv_run(plan: int, x_dev: int, y_dev: int, stream: int = 0) -> None:
    """x_dev / y_dev are device addresses (tensor.data_ptr()); stream is a hipStream_t value."""
    _check(load().spmv_run(plan, x_dev, y_dev, stream))


def spmv_run_noalloc(plan: int, x_dev: int, y_dev: int, stream: int = 0) -> None:
    """spmv_run with the plan's scratch in the library's static device array (no allocation anywhere)."""
    _check(load().spmv_run_noalloc(plan, x_dev, y_dev, stream))


def spmv_run_multi(plan: int, x_dev: int, ldx: int, y_dev: int, ldy: int, k: int, stream: int = 0) -> None:
    """k right-hand sides: vector v of X at x_dev + v*ldx elements, of Y at y_dev + v*ldy elements."""
    _check(load().spmv_run_multi(plan, x_dev, ldx, y_dev, ldy, k, stream))


def spmv_cost_predict(plan: int, corpus_path: str, spec: str):
    """(predicted microseconds or -1, corpus lines used) for plan `spec` on the matrix of `plan`'s census."""
    us, n = ctypes.c_double(), ctypes.c_int64()
    _check(load().spmv_cost_predict(plan, os.fsencode(corpus_path), spec.encode(), ctypes.byref(us), ctypes.byref(n)))
    return us.value, n.value


def spmv_fit_array(a) -> str:
    """The index model fitted to an int32 / int64 array ("" when none is exact)."""
    a = np.ascontiguousarray(a)
    if a.dtype not in (np.int32, np.int64):
        raise SpmvError(SPMV_ERR_INVALID_ARG, "int32 or int64 arrays only")
    buf = ctypes.create_string_buffer(1024)
    _check(load().spmv_fit_array(a.ctypes.data, a.dtype.itemsize, a.size, buf, 1024))
    return buf.value.decode()


def spmv_plan_jit_check(plan: int):
    """(number of launches whose specialised kernel compiled, log of failures)."""
    n = ctypes.c_int()
    buf = ctypes.create_string_buffer(1 << 16)
    _check(load().spmv_plan_jit_check(plan, ctypes.byref(n), buf, 1 << 16))
    return n.value, buf.value.decode()


def spmv_plan_save(plan: int, path: str) -> None:
    _check(load().spmv_plan_save(plan, os.fsencode(path)))


def spmv_plan_load(path: str, *, host_only=False, allocator=None) -> int:
    """Plan handle rebuilt from a file written by spmv_plan_save (no matrix, no search needed)."""
    lib = load()
    opts = spmv_options_t()
    opts.host_only = int(bool(host_only))
    keep = None
    if allocator is not None:
        alloc_py, free_py = allocator
        keep = (_ALLOC_FN(lambda nbytes, user: alloc_py(nbytes) or None), _FREE_FN(lambda ptr, user: free_py(ptr)))
        opts.dev_alloc, opts.dev_free = keep
    handle = ctypes.c_void_p()
    _check(lib.spmv_plan_load(ctypes.byref(handle), os.fsencode(path), ctypes.byref(opts)))
    if keep is not None:
        _callbacks[handle.value] = keep
    return handle.value


def spmv_run_timed(plan: int, x_dev: int, y_dev: int, stream: int = 0):
    """Runs once, synchronises the stream, returns the per-launch durations in milliseconds."""
    lib = load()
    n = ctypes.c_int()
    _check(lib.spmv_plan_launch_count(plan, ctypes.byref(n)))
    ms = (ctypes.c_float * max(n.value, 1))()
    _check(lib.spmv_run_timed(plan, x_dev, y_dev, stream, ms))
    return [ms[i] for i in range(n.value)]


def spmv_plan_time_launches(plan: int, x_dev: int, y_dev: int, stream: int = 0, repeats: int = 10):
    """Mean duration in microseconds of each launch, repeated back to back on its own (y is scratch afterwards)."""
    lib = load()
    n = ctypes.c_int()
    _check(lib.spmv_plan_launch_count(plan, ctypes.byref(n)))
    us = (ctypes.c_float * max(n.value, 1))()
    _check(lib.spmv_plan_time_launches(plan, x_dev, y_dev, stream, repeats, us))
    return [us[i] for i in range(n.value)]


def spmv_plan_time(plan: int, x_dev: int, y_dev: int, stream: int = 0, repeats: int = 20) -> float:
    """Median time of one run in microseconds (batches of back-to-back launches, HIP events)."""
    us = ctypes.c_double()
    _check(load().spmv_plan_time(plan, x_dev, y_dev, stream, repeats, ctypes.byref(us)))
    return us.value


def spmv_plan_destroy(plan: int) -> None:
    _check(load().spmv_plan_destroy(plan))
    _callbacks.pop(plan, None)


def spmv_plan_describe(plan: int) -> dict:
    lib = load()
    need = ctypes.c_size_t()
    _check(lib.spmv_plan_describe(plan, None, 0, ctypes.byref(need)))
    buf = ctypes.create_string_buffer(need.value)
    _check(lib.spmv_plan_describe(plan, buf, need.value, None))
    return json.loads(buf.value.decode())


def spmv_stream_ceiling(nbytes: int = 2 << 30, repeats: int = 5, stream: int = 0):
    """(read GB/s, copy GB/s) of the current device: best of `repeats` launches over `nbytes` bytes."""
    r, c = ctypes.c_double(), ctypes.c_double()
    _check(load().spmv_stream_ceiling(nbytes, repeats, stream, ctypes.byref(r), ctypes.byref(c)))
    return r.value, c.value


def spmv_mm_free(row_ptr: int, col_idx: int, values: int) -> None:
    """Release the three arrays spmv_mm_read allocated (addresses as integers; 0 is fine)."""
    _check(load().spmv_mm_free(row_ptr or None, col_idx or None, values or None))


def spmv_mm_read(path: str, dtype=np.float64):
    """Matrix Market coordinate file -> (nrows, ncols, row_ptr, col_idx, values) as NumPy arrays
    (copies; the library's own arrays are released before returning)."""
    lib = load()
    code = _dtype_code(dtype)
    nrows, ncols, nnz = ctypes.c_int64(), ctypes.c_int64(), ctypes.c_int64()
    rp, ci, va = ctypes.c_void_p(), ctypes.c_void_p(), ctypes.c_void_p()
    _check(lib.spmv_mm_read(os.fsencode(path), code, ctypes.byref(nrows), ctypes.byref(ncols), ctypes.byref(nnz),
                            ctypes.byref(rp), ctypes.byref(ci), ctypes.byref(va)))
    try:
        n, z = nrows.value, nnz.value
        row_ptr = np.ctypeslib.as_array(ctypes.cast(rp, ctypes.POINTER(ctypes.c_int32)), shape=(n + 1,)).copy()
        if z:
            col_idx = np.ctypeslib.as_array(ctypes.cast(ci, ctypes.POINTER(ctypes.c_int32)), shape=(z,)).copy()
            ct = ctypes.c_double if code == SPMV_F64 else ctypes.c_float
            values = np.ctypeslib.as_array(ctypes.cast(va, ctypes.POINTER(ct)), shape=(z,)).copy()
        else:
            col_idx = np.zeros(0, np.int32)
            values = np.zeros(0, np.dtype(dtype))
    finally:
        spmv_mm_free(rp.value, ci.value, va.value)
    return n, ncols.value, row_ptr, col_idx, values


def spmv_plan_array_count(plan: int) -> int:
    n = ctypes.c_int()
    _check(load().spmv_plan_array_count(plan, ctypes.byref(n)))
    return n.value


def spmv_plan_array_info(plan: int, i: int):
    name, eb, cnt = ctypes.c_char_p(), ctypes.c_int(), ctypes.c_int64()
    _check(load().spmv_plan_array_info(plan, i, ctypes.byref(name), ctypes.byref(eb), ctypes.byref(cnt)))
    return name.value.decode(), eb.value, cnt.value


def spmv_plan_array_copy(plan: int, i: int, value_dtype=np.float64) -> np.ndarray:
    name, eb, cnt = spmv_plan_array_info(plan, i)
    if name.endswith("vals"):
        dt = np.dtype(value_dtype)
    elif name.endswith("mask"):
        dt = np.dtype(np.uint64)
    elif name.endswith("dcols") or name.endswith("lane_meta"):
        dt = np.dtype(np.uint32)      # packed bytes / bit fields
    else:
        dt = {1: np.dtype(np.uint8), 2: np.dtype(np.uint16), 4: np.dtype(np.int32), 8: np.dtype(np.int64)}[eb]
    assert dt.itemsize == eb, (name, dt, eb)
    out = np.empty(cnt, dtype=dt)
    _check(load().spmv_plan_array_copy(plan, i, out.ctypes.data))
    return out


def spmv_plan_bytes(plan: int):
    a, b = ctypes.c_int64(), ctypes.c_int64()
    _check(load().spmv_plan_bytes(plan, ctypes.byref(a), ctypes.byref(b)))
    return a.value, b.value


def spmv_plan_launch_names(plan: int):
    lib = load()
    n = ctypes.c_int()
    _check(lib.spmv_plan_launch_count(plan, ctypes.byref(n)))
    out = []
    for i in range(n.value):
        s = ctypes.c_char_p()
        _check(lib.spmv_plan_launch_name(plan, i, ctypes.byref(s)))
        out.append(s.value.decode())
    return out


# ---- a small convenience wrapper over the handle -----------------------------------------------

class Plan:
    """Owns one plan handle.  `run` takes torch tensors on the plan's device."""

    def __init__(self, nrows, ncols, row_ptr, col_idx, values, **kw):
        self.nrows, self.ncols = int(nrows), int(ncols)
        self.value_dtype = np.dtype(np.asarray(values).dtype)
        self.handle = spmv_plan_create(nrows, ncols, row_ptr, col_idx, values, **kw)

    def run(self, x, y, stream=None, noalloc=False):
        if x.numel() != self.ncols or y.numel() != self.nrows:
            raise SpmvError(SPMV_ERR_INVALID_ARG, "x / y have the wrong length")
        if not (x.is_cuda and y.is_cuda and x.is_contiguous() and y.is_contiguous()):
            raise SpmvError(SPMV_ERR_INVALID_ARG, "x / y must be contiguous device tensors")
        want = "float64" if self.value_dtype == np.float64 else "float32"
        if str(x.dtype) != "torch." + want or str(y.dtype) != "torch." + want:
            raise SpmvError(SPMV_ERR_INVALID_ARG, "x / y dtype differs from the plan's")
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        (spmv_run_noalloc if noalloc else spmv_run)(self.handle, x.data_ptr(), y.data_ptr(), int(stream))
        return y

    @classmethod
    def load(cls, path, value_dtype=np.float64, **kw):
        """A plan read back from a file written by save()."""
        self = cls.__new__(cls)
        self.handle = spmv_plan_load(path, **kw)
        d = spmv_plan_describe(self.handle)
        self.nrows, self.ncols = int(d["nrows"]), int(d["ncols"])
        self.value_dtype = np.dtype(np.float64 if d["dtype"] == "f64" else np.float32)
        return self

    def save(self, path):
        spmv_plan_save(self.handle, path)

    def run_multi(self, X, Y, stream=None):
        """X: (k, ncols) and Y: (k, nrows) contiguous device tensors, one right-hand side per row."""
        if X.dim() != 2 or Y.dim() != 2 or X.shape[0] != Y.shape[0] or X.shape[1] != self.ncols or Y.shape[1] != self.nrows:
            raise SpmvError(SPMV_ERR_INVALID_ARG, "X must be (k, ncols) and Y (k, nrows)")
        if not (X.is_cuda and Y.is_cuda and X.is_contiguous() and Y.is_contiguous()):
            raise SpmvError(SPMV_ERR_INVALID_ARG, "X / Y must be contiguous device tensors")
        want = "float64" if self.value_dtype == np.float64 else "float32"
        if str(X.dtype) != "torch." + want or str(Y.dtype) != "torch." + want:
            raise SpmvError(SPMV_ERR_INVALID_ARG, "X / Y dtype differs from the plan's")
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        spmv_run_multi(self.handle, X.data_ptr(), self.ncols, Y.data_ptr(), self.nrows, int(X.shape[0]), int(stream))
        return Y

    def run_timed(self, x, y, stream=None):
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        return spmv_run_timed(self.handle, x.data_ptr(), y.data_ptr(), int(stream))

    def time_launches(self, x, y, stream=None, repeats=10):
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        return spmv_plan_time_launches(self.handle, x.data_ptr(), y.data_ptr(), int(stream), repeats)

    def time(self, x, y, stream=None, repeats=20) -> float:
        if stream is None:
            import torch
            stream = torch.cuda.current_stream().cuda_stream
        return spmv_plan_time(self.handle, x.data_ptr(), y.data_ptr(), int(stream), repeats)

    def describe(self) -> dict:
        return spmv_plan_describe(self.handle)

    def arrays(self) -> dict:
        return {spmv_plan_array_info(self.handle, i)[0]: spmv_plan_array_copy(self.handle, i, self.value_dtype)
                for i in range(spmv_plan_array_count(self.handle))}

    def bytes(self):
        return spmv_plan_bytes(self.handle)

    def launch_names(self):
        return spmv_plan_launch_names(self.handle)

    def destroy(self):
        if self.handle:
            spmv_plan_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass
