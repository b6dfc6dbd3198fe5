"""Run-time specialised kernels on the GPU: plans built with jit=1 compile their kernels with hipRTC
(constants and fitted index models baked in), launch them in place of the ahead-of-time ones, and
match the oracle to the same bar: bit-exact on integer-valued data, the tolerance otherwise."""
import numpy as np
import pytest

import inputs
import oracle
import paper_2212_10432_amd as lib
from test_jit_and_models import periodic_matrix

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

SPECS = {
    "C1": ["light=csrv,jit=1", "light=sell,sigma=256,remap=1,jit=1", "light=csrv,lpr=16,sigma=128,jit=1"],
    "C2": ["dia=1,light=sell,jit=1", "dia=1,dia_fill=0.999,drows=2,light=csrv,lpr=1,jit=1", "dia=1,dia_fill=0.999,drows=4,light=xl,w=64,rb=64,jit=1"],
    "C3": ["heavy=1024,tile=2048,light=xl,jit=1", "heavy=1024,tile=2048,hd=1,light=xl,w=16384,rb=16384,chunk=20000,jit=1",
           "heavy=1024,tile=2048,light=bin,smax=8,sigma=256,chunk=512,jit=1", "light=csrv,chunk=512,jit=1",
           "rows(64:512){light=xl,w=4096,rb=8192,jit=1}{heavy=64,tile=2048,light=csrv}{heavy=512,tile=2048,light=csrv}"],
    "C4": ["light=bsell,block=3,sigma=2048,xwin=1,remap=1,jit=1", "light=bsell,block=3,sigma=256,jit=1", "light=sell,sigma=512,jit=1"],
    "C5": ["heavy=64,tile=2048,hd=1,light=xl,jit=1", "heavy=64,tile=8192,light=xl,w=8192,rb=16384,jit=1", "heavy=1000,tile=4096,light=csrv,lpr=2,jit=1"],
}
CASES = [(n, s) for n in SPECS for s in SPECS[n]]
JIT_KINDS = ("dia", "csrv", "sell", "bsell", "heavy", "heavy.reduce", "xl", "xl.reduce", "bin0.sell", "bin1.csrv8", "bin2.csrv64")


def run(m, vals, x, spec):
    dev = torch.device("cuda:0")
    tdt = torch.float64 if vals.dtype == np.float64 else torch.float32
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, vals, force_plan=spec)
    xd = torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    yd = torch.full((m.nrows,), float("nan"), dtype=tdt, device=dev)
    P.run(xd, yd)
    torch.cuda.synchronize()
    d = P.describe()
    P.destroy()
    return yd.cpu().numpy(), d


@pytest.mark.parametrize("name,spec", CASES)
@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_jit_plans_match_oracle(name, spec, dt):
    print(f"jit {name} {spec} {np.dtype(dt).name}", flush=True)
    mi = inputs.SMALL[name](integer=True)
    vi, xi = mi.values.astype(dt), inputs.vector(mi.ncols, integer=True).astype(dt)
    y, d = run(mi, vi, xi, spec)
    assert np.array_equal(y, oracle.spmv(mi.row_ptr, mi.col_idx, vi, xi, threads=8))
    # every launch that has a specialisation runs it (the note lists what stayed ahead-of-time and why)
    for p in d["parts"]:
        leaf = p["name"].split(".", 1)[1] if p["name"][0] in "rbpc" and p["name"][1].isdigit() else p["name"]
        if leaf in JIT_KINDS and p["jit_kernel"]:
            assert p["jit"] or p["name"] in d["jit_note"], (p, d["jit_note"])
    assert any(p["jit"] for p in d["parts"]), d["jit_note"]
    m = inputs.SMALL[name]()
    vals, x = m.values.astype(dt), inputs.vector(m.ncols).astype(dt)
    y, _ = run(m, vals, x, spec)
    ok, worst = oracle.check(y, m.row_ptr, m.col_idx, vals, x, threads=8)
    assert ok, (spec, worst)


def test_fitted_offset_models_replace_the_loads():
    for spec, arr, run_len in (("light=sell,sigma=0,jit=1", "sell.slice_ptr", 64), ("light=csrv,lpr=4,sigma=1,jit=1", "csrv.seg_ptr", 1)):
        n, nc, rp, ci, va = periodic_matrix(run=run_len)
        x = np.random.default_rng(1).integers(-3, 4, nc).astype(np.float64)

        class M:
            nrows, ncols, row_ptr, col_idx = n, nc, rp, ci
        y, d = run(M, va, x, spec)
        assert d["parts"][0]["jit"] and "periodic-linear" in {a["name"]: a["model"] for a in d["arrays"]}[arr]
        assert "SPMV_JIT_S" in d["parts"][0]["jit_defines"]
        assert np.array_equal(y, oracle.spmv(rp, ci, va, x))


def test_searched_plan_may_choose_jit_and_loaded_plans_recompile(tmp_path):
    m = inputs.SMALL["C3"](integer=True)
    x = inputs.vector(m.ncols, integer=True)
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan="heavy=1024,tile=2048,light=xl,jit=1")
    path = str(tmp_path / "p.bin")
    P.save(path)
    P.destroy()
    Q = lib.Plan.load(path)
    assert any(p["jit"] for p in Q.describe()["parts"])
    dev = torch.device("cuda:0")
    xd = torch.from_numpy(x).to(dev)
    yd = torch.full((m.nrows,), float("nan"), dtype=torch.float64, device=dev)
    Q.run(xd, yd)
    Q.run(xd, yd, noalloc=True)
    torch.cuda.synchronize()
    assert np.array_equal(yd.cpu().numpy(), oracle.spmv(m.row_ptr, m.col_idx, m.values, x, threads=8))
    Q.destroy()
