"""The host side of the library (format builder, census, spec parser, Matrix Market reader, C ABI)
compiled with AddressSanitizer and UndefinedBehaviorSanitizer and driven over host-only plans of
every design on ragged seeded matrices (tests/host_asan/driver.cc).  No GPU code is involved: the
device side is replaced by stubs (tests/host_asan/kernels_stub.cc); host-only plans launch nothing."""
import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CSRC = os.path.join(ROOT, "paper_2212_10432_amd", "csrc")
HOST_SOURCES = ["util.cc", "census.cc", "builder.cc", "search.cc", "cost.cc", "fit.cc", "jit.cc", "mmio.cc", "serialize.cc", "api.cc"]


def test_host_side_is_clean_under_asan_and_ubsan(tmp_path):
    gxx = shutil.which("g++")
    if gxx is None or not os.path.isdir("/opt/rocm/include"):
        pytest.skip("needs g++ and the ROCm headers")
    from paper_2212_10432_amd import build as libbuild
    sources = [s for s in libbuild.SOURCES if s.endswith(".cc")]
    assert sorted(sources) == sorted(HOST_SOURCES)          # every host source of the library is covered
    libbuild.generate_jit_source()
    exe = str(tmp_path / "host_asan")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-static-libasan", "-static-libubsan", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           *[os.path.join(CSRC, s) for s in sources],
           os.path.join(ROOT, "tests", "host_asan", "kernels_stub.cc"), os.path.join(ROOT, "tests", "host_asan", "driver.cc"),
           "-o", exe, "-L/opt/rocm/lib", "-lamdhip64", "-lhiprtc", "-lpthread", "-Wl,-rpath,/opt/rocm/lib"]
    proc = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert proc.returncode == 0, proc.stdout[-4000:]
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:verify_asan_link_order=0:abort_on_error=0",
               UBSAN_OPTIONS="print_stacktrace=1:halt_on_error=1")
    run = subprocess.run([exe, str(tmp_path)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True, env=env, timeout=600)
    assert run.returncode == 0, run.stdout[-6000:]
    assert run.stdout.strip().splitlines()[-1].startswith("OK "), run.stdout[-2000:]
