"""Model-driven compression of index arrays and run-time kernel generation, on the CPU: the fitter's
models reproduce every element of the arrays they claim to describe (re-evaluated here from their
printed form), refuse arrays they cannot describe, and the specialised kernel source of every
launch compiles with hipRTC for gfx950 (no device needed for compiling)."""
import re

import numpy as np
import pytest

import inputs
import paper_2212_10432_amd as lib


def evaluate(text, n):
    """value(i) for i < n of a model printed as kind(base=..,step=..[,period=..][,inner=..][,if[i]=v..])."""
    f = {k: int(v) for k, v in re.findall(r"(base|step|period|inner)=(-?\d+)", text)}
    i = np.arange(n, dtype=np.int64)
    p = f.get("period", 1)
    out = f["base"] + f["step"] * (i // p) + f.get("inner", 0) * (i % p)
    for k, v in re.findall(r"if\[(\d+)\]=(-?\d+)", text):
        out[int(k)] = int(v)
    return out


@pytest.mark.parametrize("dt", [np.int32, np.int64])
def test_fitter_models(dt):
    i = np.arange(1000)
    cases = {
        "linear": 17 + 640 * i, "step": 5 - 3 * (i // 16), "periodic-linear": 100 * (i // 8) + 3 * (i % 8),
    }
    for kind, a in cases.items():
        a = a.astype(dt)
        t = lib.spmv_fit_array(a)
        assert t.startswith(kind + "("), (kind, t)
        assert np.array_equal(evaluate(t, a.size), a)
        b = a.copy()
        b[[7, 500, 999]] += 11                      # three outliers: patched by "if" branches
        t = lib.spmv_fit_array(b)
        assert t.startswith(kind + "(") and t.count("if[") == 3 and np.array_equal(evaluate(t, b.size), b)
        b[[3, 4, 5, 6, 8]] -= 1                     # too many outliers: no model
        assert lib.spmv_fit_array(b) == "" or np.array_equal(evaluate(lib.spmv_fit_array(b), b.size), b)
    rng = np.random.default_rng(3)
    assert lib.spmv_fit_array(np.cumsum(rng.integers(1, 9, 500)).astype(dt)) == ""     # a ragged offset array
    assert lib.spmv_fit_array(np.zeros(0, dt)) == "" and lib.spmv_fit_array(np.zeros(1, dt)) == ""
    assert lib.spmv_fit_array(np.array([4, 9], dt)) == "linear(base=4,step=5)"
    short = np.array([0, 10, 20, 31, 40, 50, 60], dt)                                  # 7 elements: no patch allowed
    assert lib.spmv_fit_array(short) == ""


def periodic_matrix(nrows=64 * 12, ncols=500, seed=5, run=64):
    """Runs of `run` rows with 4 entries alternate with runs of `run` rows with 8: with run = 64 the slice
    offsets, with run = 1 the row offsets follow a periodic-linear model, not a linear one."""
    rng = np.random.default_rng(seed)
    lens = np.where((np.arange(nrows) // run) % 2 == 0, 4, 8)
    rp = np.zeros(nrows + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    ci = np.concatenate([np.sort(rng.choice(ncols, L, replace=False)) for L in lens]).astype(np.int32)
    va = rng.integers(-3, 4, rp[-1]).astype(np.float64)
    va[va == 0] = 1
    return nrows, ncols, rp, ci, va


def test_models_of_plan_arrays_are_exact_and_reach_the_kernel_source():
    found = {}
    plans = [(inputs.SMALL["C1"](), "light=csrv,jit=1"), (inputs.SMALL["C1"](), "light=sell,sigma=0,jit=1"),
             (inputs.SMALL["C3"](), "heavy=1024,tile=2048,light=bin,smax=8,sigma=256,chunk=512,jit=1"),
             (inputs.SMALL["C5"](), "heavy=64,tile=2048,light=xl,w=2048,rb=4096,jit=1"),
             (inputs.SMALL["C4"](), "light=bsell,block=3,sigma=0,jit=1")]
    for m, spec in plans:
        P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan=spec, host_only=True)
        arrays, d = P.arrays(), P.describe()
        for a in d["arrays"]:
            if a["model"]:
                assert np.array_equal(evaluate(a["model"], a["count"]), arrays[a["name"]].astype(np.int64)), a
                found[a["name"]] = a["model"]
        P.destroy()
    assert found["csrv.seg_ptr"] == "linear(base=0,step=10)" and found["sell.slice_ptr"] == "linear(base=0,step=640)"
    # periodic structure: the fitted expression replaces the offset loads of the specialised kernel
    for spec, arr, macro, run in (("light=sell,sigma=0,jit=1", "sell.slice_ptr", "SPMV_JIT_SLICE_PTR(i)", 64),
                                  ("light=csrv,lpr=4,sigma=1,jit=1", "csrv.seg_ptr", "SPMV_JIT_SEG_PTR(i)", 1)):
        n, nc, rp, ci, va = periodic_matrix(run=run)
        P = lib.Plan(n, nc, rp, ci, va, force_plan=spec, host_only=True)
        d = P.describe()
        model = {a["name"]: a["model"] for a in d["arrays"]}[arr]
        assert model.startswith("periodic-linear(") and np.array_equal(evaluate(model, P.arrays()[arr].size), P.arrays()[arr])
        assert macro in d["parts"][0]["jit_defines"]
        ok, log = lib.spmv_plan_jit_check(P.handle)
        assert ok == 1, log
        P.destroy()


@pytest.mark.parametrize("name,spec", [
    ("C1", "light=csrv,jit=1"), ("C2", "dia=1,drows=2,light=sell,jit=1"), ("C3", "heavy=1024,tile=2048,hd=1,light=xl,jit=1"),
    ("C3", "rows(64){light=sell,sigma=128,jit=1}{heavy=64,tile=1024,light=csrv}"), ("C4", "light=bsell,block=3,sigma=2048,xwin=1,remap=1,jit=1"),
    ("C5", "heavy=64,tile=2048,light=xnb,k=8,r=8,jit=1"),
])
def test_specialised_kernel_source_compiles_for_gfx950(name, spec):
    m = inputs.SMALL[name]()
    for dt in (np.float64, np.float32):
        P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values.astype(dt), force_plan=spec, host_only=True)
        d = P.describe()
        assert d["jit_note"].startswith("host-only")
        want = [p for p in d["parts"] if p["jit_kernel"]]
        assert want and all("spmv::dev::k_" in p["jit_kernel"] and ("double" if dt == np.float64 else "float") in p["jit_kernel"] for p in want)
        ok, log = lib.spmv_plan_jit_check(P.handle)
        assert ok == len(want), log
        P.destroy()
