"""GPU parity at the benchmark's full sizes, with the plan the search picks (the launch
configuration bench.py times).  The C oracle computes every output element in well under a
second per matrix, so the whole y vector is compared, not a sample."""
import json
import os

import numpy as np
import pytest

import inputs
import oracle
import paper_2212_10432_amd as lib

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def run(m, vals, x, **kw):
    dev = torch.device("cuda:0")
    tdt = torch.float64 if vals.dtype == np.float64 else torch.float32
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, vals, **kw)
    xd = torch.from_numpy(x).to(dev)
    yd = torch.full((m.nrows,), float("nan"), dtype=tdt, device=dev)
    P.run(xd, yd)
    torch.cuda.synchronize()
    y = yd.cpu().numpy()
    spec = P.describe()["spec"]
    P.destroy()
    del xd, yd
    torch.cuda.empty_cache()
    return y, spec


CASES = [("C1", "C1", np.float64), ("C2", "C2", np.float64), ("C3", "C3", np.float64), ("C4", "C4", np.float64),
         ("C5", "C5", np.float64), ("C5f32", "C5", np.float32)]


def benchmarked_plans():
    """The plan specs of the run whose numbers are quoted (written by bench.py --save-plans)."""
    path = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "profiles", "plans.json")
    return json.load(open(path))


@pytest.mark.parametrize("cfg,name,dt", CASES)
def test_full_size_searched_and_benchmarked_plans(cfg, name, dt):
    print(f"full size {cfg} {np.dtype(dt).name}: generating", flush=True)
    m = inputs.FULL[name]()
    vals = m.values.astype(dt)
    x = inputs.vector(m.ncols).astype(dt)
    mi = inputs.FULL[name](integer=True)
    vi = mi.values.astype(dt)
    xi = inputs.vector(mi.ncols, integer=True).astype(dt)
    want_i = oracle.spmv(mi.row_ptr, mi.col_idx, vi, xi, threads=16)
    print("  search + run", flush=True)
    y, searched = run(m, vals, x, search_budget_ms=6000)
    specs = [("searched", searched, y)]
    quoted = benchmarked_plans()[cfg]
    if quoted != searched:
        print("  benchmarked plan differs from this search's: forcing it too", flush=True)
        yq, got = run(m, vals, x, force_plan=quoted)
        assert got == quoted
        specs.append(("benchmarked", quoted, yq))
    for what, spec, yy in specs:
        print(f"  {what} plan: {spec}", flush=True)
        ok, worst = oracle.check(yy, m.row_ptr, m.col_idx, vals, x, threads=16)
        assert ok, (cfg, what, spec, worst)
        print(f"    worst error / tolerance = {worst:.3g}", flush=True)
        # the same plan on integer-valued data of the same structure: bit-exact
        yi, _ = run(mi, vi, xi, force_plan=spec)
        assert np.array_equal(yi, want_i), (cfg, what, spec)
