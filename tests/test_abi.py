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
