"""The search's learned cost model (regression tree over census and plan features), on the CPU:
it reproduces the corpus it was fitted to, orders designs as the corpus does for a matrix it has
not seen, skips lines it cannot parse, and says so when the corpus is too small."""
import numpy as np
import pytest

import inputs
import paper_2212_10432_amd as lib


def census_fields(m, dtype_code=1):
    L = np.diff(m.row_ptr).astype(np.int64)
    return [dtype_code, m.nrows, m.ncols, m.nnz, repr(float(L.mean())), repr(float(L.var())), int(L.max()),
            int(L[L > 64].sum()), int(L[L > 1024].sum()), int((L > 1024).sum()), 0, 0.0]


# a made-up machine: microseconds per stored entry of each design, slower for irregular matrices
RATE = {"light=sell,sigma=4096": 1.0e-3, "light=csrv": 2.5e-3, "light=nnzb,r=8": 1.6e-3, "light=xl": 4.0e-3,
        "light=bin,smax=16,sigma=8192,chunk=8192": 1.3e-3}


def fake_us(m, spec):
    L = np.diff(m.row_ptr)
    irregular = L.var() > 100
    rate = RATE[spec] * (3.0 if irregular and spec.startswith("light=sell") else 1.0)
    return 2.0 + rate * m.nnz


def write_corpus(path, mats):
    with open(path, "w") as f:
        f.write("# test corpus\n")
        f.write("v0\tan old line format that must be skipped\n")
        f.write("v1\t1\t10\t10\t10\t1\t0\t1\t0\t0\t0\t0\t0\tlight=no_such_design\t5.0\n")
        for m in mats:
            for spec in RATE:
                f.write("\t".join(["v1"] + [str(v) for v in census_fields(m)] + [spec, repr(fake_us(m, spec))]) + "\n")


def test_tree_reproduces_its_corpus_and_ranks_designs_for_an_unseen_matrix(tmp_path):
    train = [inputs.uniform(n=n, k=k) for n, k in ((2000, 6), (8000, 10), (30000, 14), (60000, 8))]
    train += [inputs.powerlaw(n=n, cap=c) for n, c in ((3000, 500), (9000, 2000), (40000, 5000))]
    path = str(tmp_path / "corpus.tsv")
    write_corpus(path, train)
    for m in train:
        P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True, force_plan="light=csrv")
        for spec in RATE:
            us, n = lib.spmv_cost_predict(P.handle, path, spec)
            assert n == len(train) * len(RATE)                       # the two foreign lines were skipped
            assert us == pytest.approx(fake_us(m, spec), rel=0.35)   # leaves hold a few neighbouring samples
        P.destroy()
    # unseen sizes: the regular matrix must prefer SELL, the irregular one must not
    reg, irr = inputs.uniform(n=15000, k=9), inputs.powerlaw(n=20000, cap=3000)
    for m, best in ((reg, "light=sell,sigma=4096"), (irr, "light=bin,smax=16,sigma=8192,chunk=8192")):
        P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True, force_plan="light=csrv")
        pred = {spec: lib.spmv_cost_predict(P.handle, path, spec)[0] for spec in RATE}
        assert min(pred, key=pred.get) == best, pred
        assert pred["light=xl"] == max(pred.values())
        P.destroy()


def test_small_or_missing_corpus_gives_no_prediction(tmp_path):
    m = inputs.SMALL["C1"]()
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True, force_plan="light=csrv")
    path = str(tmp_path / "tiny.tsv")
    write_corpus(path, [])
    assert lib.spmv_cost_predict(P.handle, path, "light=sell") == (-1.0, 0)
    assert lib.spmv_cost_predict(P.handle, str(tmp_path / "missing.tsv"), "light=sell") == (-1.0, 0)
    with pytest.raises(lib.SpmvError) as e:
        lib.spmv_cost_predict(P.handle, path, "light=no_such_design")
    assert e.value.status == lib.SPMV_ERR_INVALID_ARG
    P.destroy()


def test_tree_specs_are_features_too(tmp_path):
    """Lines with plan trees load, and a tree is told apart from its first leaf."""
    mats = [inputs.powerlaw(n=n, cap=c) for n, c in ((3000, 500), (9000, 2000), (20000, 3000), (40000, 5000))]
    flat, tree = "light=xl,w=0,rb=16384,chunk=0,remap=0", "rows(64:1024){light=xl}{light=xl,rb=4096}{heavy=1024,tile=4096,light=csrv,lpr=1}"
    path = str(tmp_path / "corpus.tsv")
    with open(path, "w") as f:
        for m in mats:
            for spec, rate in ((flat, 4e-3), (tree, 2e-3)):
                f.write("\t".join(["v1"] + [str(v) for v in census_fields(m)] + [spec, repr(rate * m.nnz)]) + "\n")
    m = inputs.powerlaw(n=12000, cap=2500)
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True, force_plan="light=csrv")
    a, n = lib.spmv_cost_predict(P.handle, path, flat)
    b, _ = lib.spmv_cost_predict(P.handle, path, tree)
    assert n == 8 and 1.5 < a / b < 2.6
    P.destroy()


@pytest.mark.parametrize("name,make", [("powerlaw-70k", lambda: inputs.powerlaw(n=70_001, cap=9_000)),
                                       ("hybrid-130k", lambda: inputs.hybrid(n=130_003, n_heavy=7, heavy_len=20_000))])
def test_shipped_corpus_carries_over_to_a_matrix_left_out(tmp_path, name, make):
    """Leave one matrix out of the shipped corpus (measured on the MI355X), train on the rest, predict the
    candidates that were timed on that matrix: the predicted order must follow the measured one, and the
    best of the model's first three must be close to the best measured."""
    from scipy.stats import spearmanr
    m = make()
    lines = [l.rstrip("\n") for l in open(lib.COST_CORPUS) if l.startswith("v1")]
    same = lambda t: t[2] == str(m.nrows) and t[4] == str(m.nnz)
    mine = [l.split("\t") for l in lines if same(l.split("\t")) and l.split("\t")[1] == "1"]
    rest = [l for l in lines if not same(l.split("\t"))]
    assert len(mine) >= 10 and len(rest) > 500
    path = str(tmp_path / "rest.tsv")
    with open(path, "w") as f:
        f.write("\n".join(rest) + "\n")
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True, force_plan="light=csrv")
    pred = np.array([lib.spmv_cost_predict(P.handle, path, t[13])[0] for t in mine])
    meas = np.array([float(t[14]) for t in mine])
    P.destroy()
    assert spearmanr(pred, meas).correlation > 0.5
    assert meas[np.argsort(pred)[:3]].min() <= 1.25 * meas.min()
    assert meas[pred <= 3 * pred.min()].min() <= 1.05 * meas.min()      # what the search's pruning rule would keep
