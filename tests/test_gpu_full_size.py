"""GPU parity at the benchmark's full sizes, with the plan the search picks (the launch
configuration bench.py times).  The C oracle computes every output element in well under a
second per matrix, so the whole y vector is compared, not a sample."""
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


@pytest.mark.parametrize("name,dt", [("C1", np.float64), ("C2", np.float64), ("C3", np.float64), ("C4", np.float64),
                                     ("C5", np.float64), ("C5", np.float32)])
def test_full_size_searched_plan(name, dt):
    print(f"full size {name} {np.dtype(dt).name}: generating", flush=True)
    m = inputs.FULL[name]()
    vals = m.values.astype(dt)
    x = inputs.vector(m.ncols).astype(dt)
    print("  plan + run", flush=True)
    y, spec = run(m, vals, x, search_budget_ms=6000)
    print("  plan:", spec, flush=True)
    ok, worst = oracle.check(y, m.row_ptr, m.col_idx, vals, x, threads=16)
    assert ok, (name, spec, worst)
    print(f"  worst error / tolerance = {worst:.3g}", flush=True)
    # the same plan on integer-valued data of the same structure: bit-exact
    mi = inputs.FULL[name](integer=True)
    vi = mi.values.astype(dt)
    xi = inputs.vector(mi.ncols, integer=True).astype(dt)
    yi, _ = run(mi, vi, xi, force_plan=spec)
    assert np.array_equal(yi, oracle.spmv(mi.row_ptr, mi.col_idx, vi, xi, threads=16)), (name, spec)
