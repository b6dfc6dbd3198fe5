"""The C ABI used from plain C (tests/c_example/spmv_from_c.c, compiled with gcc against include/spmv.h
and the built library) on the GPU, and plan create/destroy cycles that must not leak device memory."""
import os
import shutil
import subprocess

import numpy as np
import pytest

import inputs
import paper_2212_10432_amd as lib

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_plain_c_program_runs_through_the_abi(tmp_path):
    rocm = "/opt/rocm"
    if not (shutil.which("gcc") and os.path.exists(os.path.join(rocm, "include", "hip", "hip_runtime_api.h"))):
        pytest.skip("gcc or the ROCm headers are not available")
    exe = str(tmp_path / "spmv_from_c")
    libdir = os.path.dirname(lib.lib_path())
    cmd = ["gcc", "-std=c99", "-O2", "-D__HIP_PLATFORM_AMD__", f"-I{rocm}/include", f"-I{ROOT}/include",
           os.path.join(ROOT, "tests", "c_example", "spmv_from_c.c"), f"-L{libdir}", "-lspmv_mi355", f"-L{rocm}/lib", "-lamdhip64", "-lm",
           f"-Wl,-rpath,{libdir}", f"-Wl,-rpath,{rocm}/lib", "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True, timeout=120)
    print("running the C example", flush=True)
    out = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "worst |y - ref|" in out.stdout
    # the same program on a Matrix Market file
    path = str(tmp_path / "t.mtx")
    with open(path, "w") as f:
        f.write("%%MatrixMarket matrix coordinate real symmetric\n4 4 5\n1 1 2.0\n2 1 -1.0\n3 2 -1.0\n4 3 -1.0\n4 4 2.0\n")
    out = subprocess.run([exe, path], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0, out.stdout + out.stderr
    assert "rows 4, nnz 8" in out.stdout


def test_plan_cycles_do_not_leak_device_memory():
    m = inputs.SMALL["C5"]()
    x = torch.from_numpy(inputs.vector(m.ncols)).cuda()
    y = torch.empty(m.nrows, dtype=torch.float64, device="cuda")
    specs = ["heavy=64,tile=2048,hd=1,light=xl", "heavy=64,tile=2048,light=xnb,k=8,r=8", "light=bin,smax=16,sigma=256,chunk=1024", None]

    def cycle():
        for spec in specs:
            P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan=spec, search_budget_ms=200)
            P.run(x, y)
            torch.cuda.synchronize()
            P.destroy()
    cycle()                                   # warm-up: code objects, allocator pools
    torch.cuda.synchronize()
    free0, _ = torch.cuda.mem_get_info()
    for _ in range(5):
        cycle()
    torch.cuda.synchronize()
    free1, _ = torch.cuda.mem_get_info()
    assert free0 - free1 < 8 << 20, (free0, free1)     # nothing of a plan's 10-100 MB stays behind
