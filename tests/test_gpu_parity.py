"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bar (from the benchmark spec): bit-exact on integer-valued inputs; otherwise
|y - y_ref|_i <= tau * (|A||x|)_i with tau = 1e-12 (fp64) / 1e-5 (fp32), y_ref accumulated wide.
Plans that reduce through atomics may differ between runs in the last bits on real data (the
summation order changes); on integer data every order is exact, so two runs must be identical.
"""
import numpy as np
import pytest

import inputs
import oracle
import paper_2212_10432_amd as lib

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

SPECS = {
    "C1": ["light=wbm", "light=csrv,lpr=256", "light=xl,w=1024,rb=2048,chunk=4096", "light=xl", "light=coo", "light=xnb,k=8,r=4", "light=nnzb,r=4", "light=xs,k=8,sigma=256", "light=xs,k=32,sigma=0", "light=csrv", "light=csrv,lpr=1", "light=csrv,lpr=64,sigma=128", "light=sell", "light=sell,sigma=256,remap=1",
           "light=bin,smax=4,sigma=128"],
    "C2": ["dia=1,dia_fill=0.999,light=wbm", "dia=1,dia_fill=0.999,light=xl,w=64,rb=64", "light=xl,w=512,rb=1024", "dia=1,dia_fill=0.999,light=coo", "dia=1,dia_fill=0.999,light=xnb,k=8,r=4", "light=xnb,k=24,r=16", "dia=1,dia_fill=0.999,light=nnzb,r=4", "light=nnzb,r=16", "dia=1,dia_fill=0.999,light=xs,k=8,sigma=64", "light=xs,k=24,sigma=4096", "dia=1,light=sell", "light=sell,sigma=64", "light=csrv,lpr=2,remap=1", "dia=1,dia_fill=0.999,light=csrv,lpr=1",
           "dia=1,drows=2,light=sell", "dia=1,dia_fill=0.999,drows=4,light=csrv,lpr=1"],
    "C3": ["heavy=1024,tile=16384,piece=32,light=sell,sigma=128", "heavy=1024,tile=2048,piece=32,light=xl", "heavy=512,tile=4096,hd=1,piece=64,light=csrv,lpr=8", "light=wbm", "heavy=1024,tile=2048,light=wbm", "light=bin,smax=16,sigma=512,chunk=256,wg=1", "heavy=1024,tile=2048,light=bin,smax=8,sigma=256,chunk=0,wg=1", "light=csrv,lpr=256,chunk=512", "light=xl,w=4096,rb=8192", "heavy=1024,tile=2048,light=xl,w=16384,rb=16384,chunk=20000", "heavy=1024,tile=2048,light=xl", "light=xnb,k=16,r=8", "heavy=1024,tile=2048,light=xnb,k=8,r=16", "light=nnzb,r=8", "light=nnzb,r=16", "heavy=1024,tile=2048,light=nnzb,r=4", "light=xs,k=16,sigma=512", "heavy=1024,tile=2048,light=xs,k=8,sigma=8192", "light=csrv,chunk=512", "light=csrv,lpr=32", "light=bin,smax=16,sigma=512,chunk=256",
           "heavy=1024,tile=2048,light=bin,smax=8,sigma=256,chunk=512", "heavy=600,tile=1024,light=csrv,lpr=8",
           "heavy=256,tile=512,light=sell,sigma=128", "heavy=2048,tile=8192,light=bin,chunk=1024", "heavy=1024,tile=2048,hd=1,light=xl", "heavy=256,tile=512,hd=1,light=sell,sigma=128"],
    "C4": ["light=bsell,block=3,sigma=256", "light=bsell,block=3,sigma=0,remap=1", "light=bsell,block=3,sigma=2048,xwin=1,remap=1", "light=sell,sigma=512",
           "light=csrv,lpr=16"],
    "C5": ["heavy=64,tile=16384,hd=1,light=csrv", "heavy=64,tile=2048,piece=16,light=xl", "heavy=64,tile=8192,hd=1,piece=128,light=sell,sigma=1024", "heavy=64,tile=2048,light=wbm", "light=bin,smax=16,sigma=256,chunk=1024,wg=1", "heavy=64,tile=2048,light=xl,w=8192,rb=16384", "light=xl,w=2048,rb=4096,chunk=100000", "heavy=64,tile=2048,light=coo", "heavy=64,tile=2048,light=xnb,k=32,r=4", "heavy=64,tile=2048,light=nnzb,r=8", "heavy=64,tile=2048,light=xs,k=16,sigma=1024", "heavy=64,tile=2048,light=sell,sigma=1024", "light=bin,smax=16,sigma=256,chunk=1024",
           "heavy=1000,tile=4096,light=csrv,lpr=2", "heavy=100,tile=8192,light=bin,sigma=8192,remap=1", "heavy=64,tile=2048,hd=1,light=xl", "heavy=64,tile=8192,hd=1,light=csrv"],
}
# plan trees: ROW_DIV by length class, power-of-two BIN, the ratio cut after SORT, COL_DIV, nested
TREES = {
    "C1": ["cols(4){light=sell,sigma=256}", "bin2(3){light=sell}{light=csrv,lpr=4}"],
    "C3": ["rows(8:64:1024){light=sell,sigma=128}{light=csrv,lpr=8}{light=csrv,lpr=64}{heavy=1024,tile=512,light=csrv}",
           "rows(16:256){light=xl,w=512,rb=1024}{light=nnzb,r=8}{heavy=256,tile=1024,hd=1,light=csrv}",
           "bin2(6){light=sell}{light=wbm}", "cut(2:64){light=sell,sigma=0}",
           "rows(64){cols(2){light=sell}{light=xl,w=256,rb=512}}{light=csrv,lpr=64,chunk=512}",
           "cols(3){rows(32){light=xl,w=256,rb=256}{light=csrv,lpr=16}}",
           "rows(100){light=xs,k=8,sigma=256}{light=xnb,k=8,r=4}",
           "rows(64:512){light=xl,w=4096,rb=8192}{heavy=64,tile=2048,light=csrv}{heavy=512,tile=2048,light=csrv}"],
    "C5": ["cut(8:100){light=sell,sigma=0}", "rows(8){light=xl,w=2048,rb=4096}{heavy=8,tile=2048,hd=1,light=csrv}",
           "rows(4:8){light=sell}{light=coo}{cols(2){heavy=8,tile=1024,light=csrv}}"],
}
for _n in TREES:
    SPECS[_n] = SPECS[_n] + TREES[_n]
CASES = [(n, s) for n in SPECS for s in SPECS[n]]


def _check_kept(kept, timed):
    """The first pass keeps the earlier of two near-ties (a later one must be 0.5 % faster); up to three candidates
    within 3 % of that one meet the kept plan again, one after the other, in a play-off that a challenger wins
    only by more than 0.5 % (the times of different turns scatter by a percent or so among themselves)."""
    assert all(kept["run_us"] <= 1.03 / 0.995 * c["run_us"] for c in timed)
    field = [c for c in timed if c["playoff_us"] > 0]
    if field:
        assert kept["playoff_us"] > 0 and len(field) <= 4 and all(0.97 * kept["playoff_us"] <= c["playoff_us"] for c in field)
    else:
        assert all(0.995 * kept["run_us"] <= c["run_us"] for c in timed)


def gpu_spmv(m, vals, x, spec=None, runs=1, **kw):
    """Returns (list of y as NumPy arrays, one per run; plan description)."""
    dev = torch.device("cuda:0")
    tdt = torch.float64 if vals.dtype == np.float64 else torch.float32
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, vals, force_plan=spec, **kw)
    xd = torch.from_numpy(np.ascontiguousarray(x.astype(vals.dtype))).to(dev)
    out = []
    for _ in range(runs):
        yd = torch.full((m.nrows,), float("nan"), dtype=tdt, device=dev)   # every element must be overwritten
        P.run(xd, yd)
        torch.cuda.synchronize()
        out.append(yd.cpu().numpy())
    d = P.describe()
    P.destroy()
    return out, d


@pytest.mark.parametrize("name,spec", CASES)
@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_forced_plans_match_oracle(name, spec, dt):
    print(f"case {name} {spec} {np.dtype(dt).name}", flush=True)
    # real-valued: tolerance
    m = inputs.SMALL[name]()
    vals, x = m.values.astype(dt), inputs.vector(m.ncols).astype(dt)
    (y1, y2), d = gpu_spmv(m, vals, x, spec, runs=2)
    for y in (y1, y2):
        ok, worst = oracle.check(y, m.row_ptr, m.col_idx, vals, x, threads=8)
        assert ok, (name, spec, worst)
    # integer-valued: bit-exact, run to run identical
    mi = inputs.SMALL[name](integer=True)
    vi, xi = mi.values.astype(dt), inputs.vector(mi.ncols, integer=True).astype(dt)
    (y1, y2), _ = gpu_spmv(mi, vi, xi, spec, runs=2)
    want = oracle.spmv(mi.row_ptr, mi.col_idx, vi, xi, threads=8)
    assert np.array_equal(y1, want) and np.array_equal(y2, want)


@pytest.mark.parametrize("name", ["C1", "C2", "C3", "C4", "C5"])
def test_searched_plan_matches_oracle(name):
    print(f"search {name}", flush=True)
    m = inputs.SMALL[name](integer=True)
    x = inputs.vector(m.ncols, integer=True)
    (y,), d = gpu_spmv(m, m.values, x, None, search_budget_ms=1500)
    assert np.array_equal(y, oracle.spmv(m.row_ptr, m.col_idx, m.values, x, threads=8))
    timed = [c for c in d["search"] if c["run_us"] >= 0]
    kept = [c for c in timed if c["note"] == "kept"]
    assert len(kept) == 1 and kept[0]["spec"] == d["spec"]
    _check_kept(kept[0], timed)


def test_device_arrays_equal_host_only_arrays():
    m = inputs.SMALL["C3"]()
    spec = "heavy=1024,tile=2048,light=bin,smax=8,sigma=256,chunk=512"
    Pd = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan=spec)
    Ph = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan=spec, host_only=True)
    a, b = Pd.arrays(), Ph.arrays()
    assert sorted(a) == sorted(b)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    Pd.destroy(); Ph.destroy()


def test_edge_cases():
    rng = np.random.default_rng(11)
    dev = torch.device("cuda:0")
    # empty matrix, matrix of empty rows, single entry
    for nrows, ncols in ((0, 0), (5, 7), (130, 3)):
        rp = np.zeros(nrows + 1, np.int32)
        for spec in ("light=csrv", "light=sell", "light=bin", "heavy=4,light=sell", "light=xs", "light=nnzb", "light=wbm", "light=csrv,lpr=256", "light=bin,wg=1", "light=xnb", "light=xl", "light=coo", None):
            P = lib.Plan(nrows, ncols, rp, np.zeros(0, np.int32), np.zeros(0), force_plan=spec, search_budget_ms=200)
            x = torch.ones(max(ncols, 1), dtype=torch.float64, device=dev)[:ncols]
            y = torch.full((max(nrows, 1),), float("nan"), dtype=torch.float64, device=dev)[:nrows]
            P.run(x, y)
            torch.cuda.synchronize()
            assert torch.all(y == 0)
            P.destroy()
    # ragged: many empty rows, duplicates, unsorted columns, rectangular
    nrows, ncols = 777, 1234
    lens = rng.integers(0, 40, nrows)
    lens[rng.random(nrows) < 0.4] = 0
    lens[5] = 3000
    rp = np.zeros(nrows + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    ci = rng.integers(0, ncols, rp[-1]).astype(np.int32)
    va = rng.integers(-3, 4, rp[-1]).astype(np.float64)
    x = rng.integers(-3, 4, ncols).astype(np.float64)
    want = oracle.spmv(rp, ci, va, x)

    class M:
        pass
    m = M()
    m.nrows, m.ncols, m.row_ptr, m.col_idx = nrows, ncols, rp, ci
    for spec in ("light=csrv", "light=csrv,lpr=64,chunk=256", "light=sell,sigma=64", "light=bin,sigma=32,chunk=512",
                 "heavy=100,tile=256,light=sell,sigma=64", "heavy=100,tile=64,light=bin", "heavy=100,tile=64,light=xs,k=8,sigma=64", "light=xs,k=16", "light=nnzb,r=4", "heavy=100,tile=64,light=nnzb,r=16", "light=xnb,k=8,r=4", "heavy=100,tile=64,light=xnb,k=16,r=8", "light=xl,w=64,rb=64", "heavy=100,tile=64,light=xl,w=256,rb=128,chunk=64", "heavy=100,tile=1024,hd=1,light=sell", "light=wbm", "heavy=100,tile=64,light=wbm", "light=csrv,lpr=256,chunk=512", "light=bin,sigma=32,chunk=512,wg=1", "light=coo", None):
        for dt in (np.float64, np.float32):
            (y,), _ = gpu_spmv(m, va.astype(dt), x.astype(dt), spec, search_budget_ms=300)
            assert np.array_equal(y.astype(np.float64), want), (spec, dt)
    # banded with duplicates: DIA and block plans must add repeated positions
    n = 600
    lens = rng.integers(0, 12, n)
    rp = np.zeros(n + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    r = np.repeat(np.arange(n), lens)
    ci = np.clip(r + rng.integers(-3, 4, rp[-1]), 0, n - 1).astype(np.int32)
    va = rng.integers(-3, 4, rp[-1]).astype(np.float64)
    x = rng.integers(-3, 4, n).astype(np.float64)
    want = oracle.spmv(rp, ci, va, x)
    m.nrows = m.ncols = n
    m.row_ptr, m.col_idx = rp, ci
    for spec in ("dia=1,light=sell", "dia=1,light=wbm", "dia=1,drows=4,light=csrv,lpr=256", "dia=1,light=xs,k=8", "dia=1,light=csrv,lpr=2", "light=bsell,block=3", "light=bsell,block=2,sigma=32,xwin=1",
                 "light=bsell,block=4,sigma=-1,remap=1"):
        (y,), _ = gpu_spmv(m, va, x, spec)
        assert np.array_equal(y, want), spec


def test_run_argument_errors():
    m = inputs.SMALL["C1"]()
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan="light=csrv")
    x = torch.zeros(m.ncols, dtype=torch.float64, device="cuda:0")
    with pytest.raises(lib.SpmvError) as e:
        lib.spmv_run(P.handle, x.data_ptr(), x.data_ptr(), 0)        # aliasing
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG
    with pytest.raises(lib.SpmvError):
        lib.spmv_run(P.handle, 0, x.data_ptr(), 0)
    with pytest.raises(lib.SpmvError):
        P.run(x[:-1], x)
    P.destroy()


def test_row_permutation_invariance():
    """P (A x) == (P A) x: permuting the rows of A permutes y, whatever plan is chosen."""
    m = inputs.SMALL["C5"](integer=True)
    x = inputs.vector(m.ncols, integer=True)
    rng = np.random.default_rng(2)
    perm = rng.permutation(m.nrows)
    lens = np.diff(m.row_ptr)[perm]
    rp = np.zeros(m.nrows + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    idx = np.concatenate([np.arange(m.row_ptr[r], m.row_ptr[r + 1]) for r in perm])

    class M:
        pass
    pm = M()
    pm.nrows, pm.ncols, pm.row_ptr, pm.col_idx = m.nrows, m.ncols, rp, m.col_idx[idx]
    spec = "heavy=100,tile=8192,light=bin,sigma=8192"
    (y,), _ = gpu_spmv(m, m.values, x, spec)
    (yp,), _ = gpu_spmv(pm, m.values[idx], x, spec)
    assert np.array_equal(yp, y[perm])


def test_timing_and_launch_introspection():
    """spmv_run_timed / spmv_plan_time / launch names and per-launch bytes agree with the plan."""
    m = inputs.SMALL["C3"]()
    x = inputs.vector(m.ncols)
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan="heavy=1024,tile=2048,light=xnb,k=8,r=8")
    d = P.describe()
    names = P.launch_names()
    assert names == [p["name"] for p in d["parts"]] == ["xnb.zero", "xnb", "xnb.reduce", "heavy", "heavy.reduce"]
    assert d["scratch_bytes"] > 0 and all(p["bytes"] > 0 for p in d["parts"])
    b_plan, b_csr = P.bytes()
    assert b_plan == sum(p["bytes"] for p in d["parts"])
    xd = torch.from_numpy(x).to("cuda:0")
    yd = torch.full((m.nrows,), float("nan"), dtype=torch.float64, device="cuda:0")
    ms = P.run_timed(xd, yd)
    assert len(ms) == len(names) and all(t >= 0 for t in ms)
    ok, worst = oracle.check(yd.cpu().numpy(), m.row_ptr, m.col_idx, m.values, x)
    assert ok, worst
    us = P.time(xd, yd, repeats=5)
    assert 0 < us < 1e5
    # a plan with scratch gives the same result on repeated runs into the same y (integer data: exact)
    mi = inputs.SMALL["C3"](integer=True)
    xi = inputs.vector(mi.ncols, integer=True)
    Pi = lib.Plan(mi.nrows, mi.ncols, mi.row_ptr, mi.col_idx, mi.values, force_plan="heavy=1024,tile=2048,light=xnb,k=8,r=8")
    xid = torch.from_numpy(xi).to("cuda:0")
    want = oracle.spmv(mi.row_ptr, mi.col_idx, mi.values, xi)
    for _ in range(3):
        Pi.run(xid, yd)
    torch.cuda.synchronize()
    assert np.array_equal(yd.cpu().numpy(), want)
    P.destroy(); Pi.destroy()


def test_graph_replay_matches_eager():
    """spmv_run enqueues kernels only, so a captured HIP graph of runs replays to the same result."""
    m = inputs.SMALL["C5"](integer=True)
    x = inputs.vector(m.ncols, integer=True)
    want = oracle.spmv(m.row_ptr, m.col_idx, m.values, x)
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, search_budget_ms=500)
    xd = torch.from_numpy(x).to("cuda:0")
    yd = torch.zeros(m.nrows, dtype=torch.float64, device="cuda:0")
    s = torch.cuda.Stream()
    with torch.cuda.stream(s):
        P.run(xd, yd, s.cuda_stream)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g, stream=s):
        for _ in range(3):
            P.run(xd, yd, s.cuda_stream)
    for _ in range(3):
        yd.fill_(-1.0)
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(yd.cpu().numpy(), want)
    P.destroy()


def test_caller_supplied_allocator_and_allocation_failure():
    """dev_alloc / dev_free: every device array of a plan comes from the caller's allocator (here backed
    by torch tensors) and goes back through it; a failing allocator yields SPMV_ERR_ALLOC with nothing
    left allocated."""
    m = inputs.SMALL["C5"](integer=True)
    x = inputs.vector(m.ncols, integer=True)
    want = oracle.spmv(m.row_ptr, m.col_idx, m.values, x)
    live, stats = {}, {"allocs": 0, "frees": 0, "fail_at": None}

    def alloc(nbytes):
        stats["allocs"] += 1
        if stats["fail_at"] is not None and stats["allocs"] >= stats["fail_at"]:
            return 0
        t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device="cuda:0")
        live[t.data_ptr()] = t
        return t.data_ptr()

    def free(ptr):
        stats["frees"] += 1
        del live[ptr]

    spec = "heavy=64,tile=2048,light=xnb,k=8,r=8"
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan=spec, allocator=(alloc, free))
    n_arrays = lib.spmv_plan_array_count(P.handle)
    assert len(live) >= n_arrays and stats["frees"] == 0
    xd = torch.from_numpy(x).to("cuda:0")
    yd = torch.empty(m.nrows, dtype=torch.float64, device="cuda:0")
    P.run(xd, yd)
    torch.cuda.synchronize()
    assert np.array_equal(yd.cpu().numpy(), want)
    P.destroy()
    assert not live and stats["frees"] == stats["allocs"]
    # the search allocates and frees candidate after candidate through the same pair
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, search_budget_ms=300, allocator=(alloc, free))
    P.run(xd, yd)
    torch.cuda.synchronize()
    assert np.array_equal(yd.cpu().numpy(), want)
    P.destroy()
    assert not live
    # failure on the n-th allocation: error code, message, and everything handed back
    for fail_at in (1, 3, 6):
        stats.update(allocs=0, frees=0, fail_at=fail_at)
        with pytest.raises(lib.SpmvError) as e:
            lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, force_plan=spec, allocator=(alloc, free))
        assert e.value.status == lib.SPMV_ERR_ALLOC and "allocation" in e.value.message
        assert not live and stats["frees"] == fail_at - 1
    stats["fail_at"] = None


def test_matrix_market_file_to_gpu_result(tmp_path):
    """The path a user of the paper's tool takes: a Matrix Market file in, y out."""
    m = inputs.hybrid(n=20011, n_heavy=5, heavy_len=5000, integer=True)
    path = str(tmp_path / "h.mtx")
    rows = np.repeat(np.arange(m.nrows), np.diff(m.row_ptr))
    with open(path, "w") as f:
        f.write("%%MatrixMarket matrix coordinate integer general\n")
        f.write(f"{m.nrows} {m.ncols} {m.nnz}\n")
        for r, c, v in zip(rows, m.col_idx, m.values):
            f.write(f"{r + 1} {c + 1} {int(v)}\n")
    nrows, ncols, rp, ci, va = lib.spmv_mm_read(path, np.float64)
    assert np.array_equal(rp, m.row_ptr) and np.array_equal(ci, m.col_idx) and np.array_equal(va, m.values)

    class M:
        pass
    mm = M()
    mm.nrows, mm.ncols, mm.row_ptr, mm.col_idx = nrows, ncols, rp, ci
    x = inputs.vector(ncols, integer=True)
    (y,), d = gpu_spmv(mm, va, x, None, search_budget_ms=500)
    assert np.array_equal(y, oracle.spmv(rp, ci, va, x))


def _random_spec(rng):
    light = rng.choice(["csrv", "sell", "bin", "nnzb", "xs", "xnb", "xl", "xl", "coo", "wbm"])
    parts = []
    if rng.random() < 0.5:
        parts.append(f"heavy={int(rng.choice([8, 16, 40, 100]))},tile={int(rng.choice([64, 128, 512, 4096]))}")
        if rng.random() < 0.5:
            parts.append("hd=1")
        if rng.random() < 0.4:
            parts.append(f"piece={int(rng.choice([4, 8, 32]))}")
    parts.append(f"light={light}")
    if light == "csrv":
        parts.append(f"lpr={int(rng.choice([0, 1, 2, 8, 64]))},chunk={int(rng.choice([0, 64, 200]))},sigma={int(rng.choice([0, 64, -1]))}")
    elif light == "sell":
        parts.append(f"sigma={int(rng.choice([0, 64, 300, -1]))}")
    elif light == "bin":
        parts.append(f"smax={int(rng.choice([2, 8, 16]))},sigma={int(rng.choice([0, 128]))},chunk={int(rng.choice([0, 128]))}")
    elif light == "nnzb":
        parts.append(f"r={int(rng.choice([4, 8, 16]))}")
    elif light == "xs":
        parts.append(f"k={int(rng.choice([8, 16, 24, 32]))},sigma={int(rng.choice([0, 64, 1024]))}")
    elif light == "xnb":
        parts.append(f"k={int(rng.choice([8, 16, 24, 32]))},r={int(rng.choice([4, 8, 16]))}")
    elif light == "xl":
        parts.append(f"w={int(rng.choice([64, 128, 1024, 0]))},rb={int(rng.choice([64, 256, 4096, 16384]))},chunk={int(rng.choice([0, 64, 1000]))}")
    if rng.random() < 0.3:
        parts.append("remap=1")
    return ",".join(parts)


def test_random_matrices_random_plans():
    """Differential test: random shapes (rectangular, empty rows and columns, repeated and unsorted
    columns, a few long rows) under random legal plan specs; integer data, so bit-exact."""
    rng = np.random.default_rng(20221113)

    class M:
        pass
    for case in range(150):
        nrows, ncols = int(rng.integers(1, 3000)), int(rng.integers(1, 3000))
        lens = rng.integers(0, int(rng.choice([3, 12, 60])), nrows)
        lens[rng.random(nrows) < 0.3] = 0
        for _ in range(int(rng.integers(0, 4))):
            lens[int(rng.integers(0, nrows))] = int(rng.integers(100, 4000))
        rp = np.zeros(nrows + 1, np.int32)
        np.cumsum(lens, out=rp[1:])
        span = ncols if rng.random() < 0.5 else max(1, ncols // 7)      # scattered or clustered columns
        ci = rng.integers(0, span, rp[-1]).astype(np.int32)
        va = rng.integers(-3, 4, rp[-1]).astype(np.float64)
        x = rng.integers(-3, 4, ncols).astype(np.float64)
        m = M()
        m.nrows, m.ncols, m.row_ptr, m.col_idx = nrows, ncols, rp, ci
        want = oracle.spmv(rp, ci, va, x)
        for _ in range(3):
            spec = _random_spec(rng)
            dt = np.float64 if rng.random() < 0.5 else np.float32
            print(f"case {case}: {nrows}x{ncols} nnz {rp[-1]} {spec} {np.dtype(dt).name}", flush=True)
            try:
                (y,), _ = gpu_spmv(m, va.astype(dt), x.astype(dt), spec)
            except lib.SpmvError as e:
                assert e.status == lib.SPMV_ERR_UNSUPPORTED, (spec, e)      # e.g. too many heavy rows
                continue
            assert np.array_equal(y.astype(np.float64), want), (case, spec, dt)


def test_stream_ceiling_is_plausible():
    read, copy = lib.spmv_stream_ceiling(1 << 30, 3)
    assert 2000 < read < 8000 and 2000 < copy < 8000, (read, copy)      # GB/s on an MI355X (peak 8000)
    with pytest.raises(lib.SpmvError) as e:
        lib.spmv_stream_ceiling(1000, 3)
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG


@pytest.mark.parametrize("dt", [np.float64, np.float32])
def test_many_heavy_rows_with_narrow_slices(dt):
    """Several hundred heavy rows whose entries per column stripe are few: the heavy kernel then
    walks many narrow slices (taken four at a time when their widths agree) besides a few wide ones."""
    rng = np.random.default_rng(3)
    nrows, ncols = 3000, 40000
    lens = rng.integers(1, 6, nrows)
    heavy_rows = rng.choice(nrows, 700, replace=False)
    lens[heavy_rows] = rng.integers(120, 400, heavy_rows.size)
    lens[heavy_rows[:5]] = 6000                      # a few really long rows: wide slices too
    rp = np.zeros(nrows + 1, np.int32)
    np.cumsum(lens, out=rp[1:])
    ci = rng.integers(0, ncols, rp[-1]).astype(np.int32)
    va = rng.integers(-3, 4, rp[-1]).astype(np.float64)
    x = rng.integers(-3, 4, ncols).astype(np.float64)
    want = oracle.spmv(rp, ci, va, x)

    class M:
        pass
    m = M()
    m.nrows, m.ncols, m.row_ptr, m.col_idx = nrows, ncols, rp, ci
    for spec in ("heavy=100,tile=512,light=csrv", "heavy=100,tile=2048,light=xl,w=1024,rb=512", "heavy=100,tile=1024,hd=1,light=sell,sigma=64",
                 "heavy=100,tile=64,light=coo"):
        (y,), d = gpu_spmv(m, va.astype(dt), x.astype(dt), spec)
        assert np.array_equal(y.astype(np.float64), want), (spec, dt)
        heavy = [p for p in d["parts"] if p["name"] == "heavy"][0]
        assert heavy["rows"] == 700


def test_random_block_banded_matrices_blocked_and_diagonal_plans():
    """Differential test for the plans that need structure: random block-banded matrices (block edge
    2-4, partly filled blocks, repeated positions summed) under blocked-SELL plans with and without
    the LDS x window and sort, diagonal extraction with several remainders, and the search."""
    import scipy.sparse as sp
    rng = np.random.default_rng(1)

    class M:
        pass
    ran = 0
    for case in range(30):
        b = int(rng.choice([2, 3, 4]))
        nb = int(rng.integers(1, 5000))
        band = int(rng.choice([1, 3, 40, 700]))
        per = rng.integers(1, 8, nb)
        br = np.repeat(np.arange(nb), per)
        bc = np.clip(br + rng.integers(-band, band + 1, br.size), 0, nb - 1)
        keep = rng.random((br.size, b, b)) < float(rng.choice([1.0, 0.9, 0.5]))
        rr = (br[:, None, None] * b + np.arange(b)[None, :, None] + np.zeros((1, 1, b), int))[keep]
        cc = (bc[:, None, None] * b + np.zeros((1, b, 1), int) + np.arange(b)[None, None, :])[keep]
        vv = rng.integers(-3, 4, rr.size).astype(np.float64)
        n = nb * b
        A = sp.coo_matrix((vv, (rr, cc)), shape=(n, n)).tocsr()
        A.sort_indices()
        rp, ci, va = A.indptr.astype(np.int32), A.indices.astype(np.int32), A.data.astype(np.float64)
        x = rng.integers(-3, 4, n).astype(np.float64)
        m = M()
        m.nrows, m.ncols, m.row_ptr, m.col_idx = n, n, rp, ci
        want = oracle.spmv(rp, ci, va, x)
        specs = [f"light=bsell,block={b},sigma={int(rng.choice([0, 64, 2048, -1]))},xwin={int(rng.integers(0, 2))},remap={int(rng.integers(0, 2))}",
                 f"light=bsell,block={b},sigma=2048,xwin=1,remap=1",
                 "dia=1,dia_fill=0.3,light=" + str(rng.choice(["sell,sigma=64", "csrv", "xl,w=64,rb=64", "xnb,k=8,r=4", "coo"])), None]
        for spec in specs:
            dt = np.float64 if rng.random() < 0.5 else np.float32
            print(f"case {case}: n {n} block {b} band {band} nnz {rp[-1]} {spec} {np.dtype(dt).name}", flush=True)
            try:
                (y,), _ = gpu_spmv(m, va.astype(dt), x.astype(dt), spec, search_budget_ms=100)
            except lib.SpmvError as e:
                assert e.status == lib.SPMV_ERR_UNSUPPORTED, (spec, e)     # no diagonal dense enough, window too wide
                continue
            ran += 1
            assert np.array_equal(y.astype(np.float64), want), (case, spec, dt)
    assert ran > 60


@pytest.mark.gpu
@pytest.mark.parametrize("extra_rows,extra_cols", [(1, 1), (2, 0), (0, 1)])
def test_blocked_plans_on_dimensions_with_a_ragged_edge(extra_rows, extra_cols):
    """A block-structured matrix whose dimensions are not multiples of 3: the blocked part takes the whole
    blocks, a CSR part the last rows and columns; forced and searched plans against the oracle, bit-exact
    on integer values."""
    import scipy.sparse as sp
    m = inputs.SMALL["C4"](integer=True)
    rng = np.random.default_rng(11)
    ints = lambda k: rng.integers(1, 4, k).astype(np.float64)
    A = sp.csr_matrix((m.values, m.col_idx, m.row_ptr), shape=(m.nrows, m.ncols))
    if extra_cols:
        A = sp.hstack([A, sp.random(m.nrows, extra_cols, density=0.2, random_state=1, data_rvs=ints)])
    if extra_rows:
        A = sp.vstack([A, sp.random(extra_rows, A.shape[1], density=0.01, random_state=2, data_rvs=ints)])
    A = A.tocsr(); A.sort_indices()
    nr, nc = A.shape
    rp, ci, va = A.indptr.astype(np.int32), A.indices.astype(np.int32), A.data.astype(np.float64)
    x = inputs.vector(nc, integer=True)
    want = oracle.spmv(rp, ci, va, x)
    dev = torch.device("cuda:0")
    xd = torch.from_numpy(x).to(dev)
    for spec in ("light=bsell,block=3,sigma=256", "light=bsell,block=3,sigma=2048,xwin=1,remap=1", None):
        print(f"case ragged {extra_rows} {extra_cols} {spec}", flush=True)
        P = lib.Plan(nr, nc, rp, ci, va, force_plan=spec, search_budget_ms=1500)
        yd = torch.full((nr,), float("nan"), dtype=torch.float64, device=dev)
        P.run(xd, yd)
        torch.cuda.synchronize()
        d = P.describe()
        P.destroy()
        assert np.array_equal(yd.cpu().numpy(), want), (spec, d["spec"])
        if spec is None:   # the census sees the blocks despite the edge: blocked candidates were built and timed
            assert any("bsell" in c["spec"] and c["run_us"] > 0 for c in d["search"]), d["search"]
