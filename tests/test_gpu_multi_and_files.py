"""GPU parity of (i) plans read back from plan files and (ii) the multi-vector entry point
spmv_run_multi: every result vector element by element against one oracle call per vector.
Bar: bit-exact on integer-valued data, the oracle's tolerance on real-valued data."""
import numpy as np
import pytest

import inputs
import oracle
import paper_2212_10432_amd as lib

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

MULTI = [
    ("C1", "light=csrv"), ("C1", "light=csrv,lpr=16,sigma=128"), ("C1", "light=sell,sigma=256,remap=1"),
    ("C2", "dia=1,light=sell"), ("C2", "dia=1,dia_fill=0.999,light=csrv,lpr=1"), ("C2", "dia=1,dia_fill=0.999,drows=2,light=xl,w=64,rb=64"),
    ("C3", "light=csrv,chunk=512"), ("C3", "heavy=1024,tile=2048,light=bin,smax=8,sigma=256,chunk=512"),
    ("C3", "heavy=1024,tile=2048,hd=1,light=xl"), ("C4", "light=bsell,block=3,sigma=2048,xwin=1,remap=1"),
    ("C5", "heavy=64,tile=2048,light=xnb,k=32,r=4"), ("C5", "heavy=64,tile=2048,light=sell,sigma=1024"),
]


@pytest.mark.parametrize("name,spec", MULTI)
@pytest.mark.parametrize("dt", [np.float64, np.float32])
@pytest.mark.parametrize("k", [1, 3, 8, 15])
def test_multi_vector_matches_k_oracle_calls(name, spec, dt, k):
    print(f"multi {name} {spec} {np.dtype(dt).name} k={k}", flush=True)
    dev = torch.device("cuda:0")
    tdt = torch.float64 if dt == np.float64 else torch.float32
    for integer in (True, False):
        m = inputs.SMALL[name](integer=integer)
        vals = m.values.astype(dt)
        X = np.stack([inputs.vector(m.ncols, seed=inputs.BASE_SEED + 200 + v, integer=integer).astype(dt) for v in range(k)])
        P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, vals, force_plan=spec)
        Xd = torch.from_numpy(X).to(dev)
        Yd = torch.full((k, m.nrows), float("nan"), dtype=tdt, device=dev)
        P.run_multi(Xd, Yd)
        torch.cuda.synchronize()
        Y = Yd.cpu().numpy()
        P.destroy()
        for v in range(k):
            if integer:
                assert np.array_equal(Y[v], oracle.spmv(m.row_ptr, m.col_idx, vals, X[v], threads=8)), (spec, v)
            else:
                ok, worst = oracle.check(Y[v], m.row_ptr, m.col_idx, vals, X[v], threads=8)
                assert ok, (spec, v, worst)


def test_multi_vector_with_padded_leading_dimensions_and_bad_arguments():
    dev = torch.device("cuda:0")
    m = inputs.SMALL["C1"](integer=True)
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan="light=csrv")
    k, ldx, ldy = 5, m.ncols + 37, m.nrows + 11
    X = np.zeros((k, ldx))
    for v in range(k):
        X[v, : m.ncols] = inputs.vector(m.ncols, seed=inputs.BASE_SEED + 300 + v, integer=True)
    Xd = torch.from_numpy(X).to(dev)
    Yd = torch.full((k, ldy), -7.0, dtype=torch.float64, device=dev)
    lib.spmv_run_multi(P.handle, Xd.data_ptr(), ldx, Yd.data_ptr(), ldy, k, torch.cuda.current_stream().cuda_stream)
    torch.cuda.synchronize()
    Y = Yd.cpu().numpy()
    for v in range(k):
        assert np.array_equal(Y[v, : m.nrows], oracle.spmv(m.row_ptr, m.col_idx, m.values, X[v, : m.ncols], threads=8))
    assert np.all(Y[:, m.nrows:] == -7.0)            # nothing written between the vectors
    for bad in ((m.ncols - 1, ldy, 2), (ldx, m.nrows - 1, 2), (ldx, ldy, -1), (ldx, ldy, 5000)):
        with pytest.raises(lib.SpmvError) as e:
            lib.spmv_run_multi(P.handle, Xd.data_ptr(), bad[0], Yd.data_ptr(), bad[1], bad[2], 0)
        assert e.value.status == lib.SPMV_ERR_INVALID_ARG
    lib.spmv_run_multi(P.handle, Xd.data_ptr(), ldx, Yd.data_ptr(), ldy, 0, 0)    # k = 0: nothing to do
    P.destroy()


@pytest.mark.parametrize("name,spec", [("C3", "heavy=1024,tile=2048,hd=1,light=xl"), ("C4", "light=bsell,block=3,sigma=2048,xwin=1,remap=1"),
                                       ("C5", "heavy=64,tile=2048,light=xnb,k=32,r=4"), ("C2", "dia=1,light=sell"), ("C3", None)])
@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_plan_read_back_from_a_file_runs_like_the_original(tmp_path, name, spec, dt):
    print(f"plan file {name} {spec} {np.dtype(dt).name}", flush=True)
    dev = torch.device("cuda:0")
    tdt = torch.float64 if dt == np.float64 else torch.float32
    m = inputs.SMALL[name](integer=True)
    vals, x = m.values.astype(dt), inputs.vector(m.ncols, integer=True).astype(dt)
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, vals, force_plan=spec, search_budget_ms=500)
    path = str(tmp_path / "plan.bin")
    P.save(path)
    want_arrays, want_desc = P.arrays(), P.describe()
    P.destroy()
    Q = lib.Plan.load(path)                       # device plan, no matrix, no search
    got = Q.arrays()
    assert list(got) == list(want_arrays) and all(np.array_equal(got[k], want_arrays[k]) for k in got)
    assert Q.describe() == want_desc
    xd = torch.from_numpy(x).to(dev)
    yd = torch.full((m.nrows,), float("nan"), dtype=tdt, device=dev)
    Q.run(xd, yd)
    torch.cuda.synchronize()
    assert np.array_equal(yd.cpu().numpy(), oracle.spmv(m.row_ptr, m.col_idx, vals, x, threads=8))
    Q.destroy()
    Qh = lib.Plan.load(path, host_only=True)      # the same file read on the host
    assert all(np.array_equal(Qh.arrays()[k], want_arrays[k]) for k in want_arrays)
    Qh.destroy()
