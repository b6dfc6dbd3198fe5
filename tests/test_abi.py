"""The C-ABI shared library loads and exports every function include/spmv.h declares."""
import ctypes
import os
import re

import paper_2212_10432_amd as lib

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "spmv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(spmv_[a-z_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported():
    names = declared_functions()
    assert "spmv_plan_create" in names and "spmv_run" in names and "spmv_plan_destroy" in names
    dll = ctypes.CDLL(lib.lib_path())
    for n in names:
        assert hasattr(dll, n), n
    assert sorted(lib.EXPORTS) == names


def test_binding_has_the_same_names():
    for n in declared_functions():
        if n in ("spmv_plan_launch_count", "spmv_plan_launch_name"):
            assert hasattr(lib, "spmv_plan_launch_names")
        else:
            assert callable(getattr(lib, n)), n


def test_last_error_is_empty_string_or_text():
    assert isinstance(lib.spmv_last_error(), str)


def test_binding_checks_array_lengths_before_passing_pointers():
    import numpy as np
    import pytest
    rp = np.array([0, 1, 2], np.int32)
    with pytest.raises(lib.SpmvError) as e:          # row_ptr too short for nrows = 5
        lib.spmv_plan_create(5, 2, rp, np.zeros(2, np.int32), np.ones(2), host_only=True, force_plan="light=csrv")
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG
    with pytest.raises(lib.SpmvError) as e:          # nnz larger than the arrays
        lib.spmv_plan_create(2, 2, rp, np.zeros(2, np.int32), np.ones(2), host_only=True, force_plan="light=csrv", nnz=7)
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG
