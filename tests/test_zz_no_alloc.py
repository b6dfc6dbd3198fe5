"""spmv_run_noalloc (the plan's scratch in the library's static device array) against spmv_run, the
entry point it is a variant of: two calls in a row through the C ABI, the second with a smaller
input, so that whatever the first call left in the shared array lies under and beyond what the
second one uses.  Bar: bit-exact on integer-valued data (every summation order is exact there),
within the oracle's tolerance on real-valued data."""
import numpy as np
import pytest

import inputs
import oracle
import paper_2212_10432_amd as lib

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

# plans whose launches hand partial sums or products to a later launch through scratch
SPECS = ["heavy=64,tile=2048,light=xl,w=2048,rb=4096", "heavy=64,tile=2048,hd=1,light=xnb,k=8,r=8",
         "heavy=64,tile=2048,light=xs,k=8,sigma=256"]


def both(m, vals, x, spec):
    dev = torch.device("cuda:0")
    tdt = torch.float64 if vals.dtype == np.float64 else torch.float32
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, vals, force_plan=spec)
    assert P.describe()["scratch_bytes"] > 0
    xd = torch.from_numpy(x).to(dev)
    ya = torch.full((m.nrows,), float("nan"), dtype=tdt, device=dev)
    yb = torch.full((m.nrows,), float("nan"), dtype=tdt, device=dev)
    P.run(xd, ya)
    P.run(xd, yb, noalloc=True)
    torch.cuda.synchronize()
    P.destroy()
    return ya.cpu().numpy(), yb.cpu().numpy()


@pytest.mark.parametrize("spec", SPECS)
@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_noalloc_matches_run_twice_in_a_row(spec, dt):
    print(f"noalloc {spec} {np.dtype(dt).name}", flush=True)
    big = inputs.SMALL["C5"]
    small = lambda **kw: inputs.hybrid(n=20011, n_heavy=5, heavy_len=5000, **kw)
    for make in (big, small):            # second call: a smaller matrix, same static array
        mi = make(integer=True)
        vi, xi = mi.values.astype(dt), inputs.vector(mi.ncols, integer=True).astype(dt)
        ya, yb = both(mi, vi, xi, spec)
        want = oracle.spmv(mi.row_ptr, mi.col_idx, vi, xi, threads=8)
        assert np.array_equal(ya, want) and np.array_equal(yb, want)
        m = make()
        vals, x = m.values.astype(dt), inputs.vector(m.ncols).astype(dt)
        ya, yb = both(m, vals, x, spec)
        for y in (ya, yb):
            ok, worst = oracle.check(y, m.row_ptr, m.col_idx, vals, x, threads=8)
            assert ok, (spec, worst)


def test_noalloc_rejects_plans_beyond_the_static_array():
    # one fp64 product per stored entry: 5 M entries need 40 MB of scratch, the array holds 32 MiB
    m = inputs.uniform(n=500_000, k=10, integer=True)
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan="light=xl")
    assert P.describe()["scratch_bytes"] > (32 << 20)
    dev = torch.device("cuda:0")
    x = inputs.vector(m.ncols, integer=True)
    xd = torch.from_numpy(x).to(dev)
    yd = torch.full((m.nrows,), float("nan"), dtype=torch.float64, device=dev)
    with pytest.raises(lib.SpmvError) as e:
        P.run(xd, yd, noalloc=True)
    assert e.value.status == lib.SPMV_ERR_UNSUPPORTED and "static" in e.value.message
    assert torch.all(torch.isnan(yd))          # nothing was launched
    P.run(xd, yd)                               # the plan itself is fine
    torch.cuda.synchronize()
    assert np.array_equal(yd.cpu().numpy(), oracle.spmv(m.row_ptr, m.col_idx, m.values, x, threads=8))
    P.destroy()
