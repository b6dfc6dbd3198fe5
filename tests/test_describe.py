"""The plan description (JSON) a host-only plan reports: schema, operator chain in the paper's
vocabulary, byte model, and the deterministic candidate order of the census-pruned search."""
import numpy as np

import inputs
import paper_2212_10432_amd as lib


def test_schema_and_operator_names():
    m = inputs.SMALL["C3"]()
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True,
                 force_plan="heavy=1024,tile=2048,light=xnb,k=16,r=8")
    d = P.describe()
    for key in ("spec", "operators", "dtype", "nrows", "ncols", "nnz", "bytes_plan", "bytes_csr", "census", "parts",
                "arrays", "scratch_bytes", "search"):
        assert key in d, key
    assert d["dtype"] == "f64" and d["nnz"] == m.nnz
    for op in ("COMPRESS", "ROW_DIV", "COL_DIV", "BMT_NNZ_BLOCK", "THREAD_BITMAP_RED", "WARP_SEG_RED"):
        assert op in d["operators"], op
    c = d["census"]
    L = np.diff(m.row_ptr)
    assert c["max_len"] == L.max() and c["min_len"] == L.min() and abs(c["mean_len"] - L.mean()) < 1e-9 * L.mean()
    assert c["irregular"] is True and abs(c["var_len"] - L.var()) < 1e-9 * L.var()
    assert d["search"] == [{"spec": d["spec"], "build_ms": 0, "run_us": -1, "pred_us": -1, "playoff_us": -1, "note": "forced"}]
    # the spec string round-trips
    P2 = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True, force_plan=d["spec"])
    assert P2.describe()["spec"] == d["spec"]
    P.destroy(); P2.destroy()


def test_census_prunes_the_candidates():
    """Structure pruning by sparsity pattern (paper, Section VI-B): what the census sees decides
    which designs are even tried; with no timing the first candidate is taken."""
    first = {}
    for name in ("C1", "C2", "C3", "C4", "C5"):
        m = inputs.SMALL[name]()
        P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values, host_only=True, search_budget_ms=-1)
        first[name] = P.describe()
        P.destroy()
    assert first["C1"]["spec"].startswith("light=sell")                      # short even rows
    assert first["C2"]["spec"].startswith("dia=1")                           # five full diagonals
    assert first["C2"]["census"]["diag_offsets"] == [-67, -1, 0, 1, 67]
    assert "light=bsell,block=3" in first["C4"]["spec"]                      # 3x3 blocks, fill 1
    assert abs(first["C4"]["census"]["block_fill"]["3"] - 1.0) < 1e-12
    for name in ("C3", "C5"):                                                 # irregular: heavy split
        assert first[name]["census"]["irregular"] is True
        assert first[name]["spec"].startswith("heavy=")


def test_block_census_does_not_need_sorted_columns():
    """A block-structured matrix whose rows list their columns in any order still gets the blocked design."""
    import numpy as np
    m = inputs.SMALL["C4"]()
    rng = np.random.default_rng(0)
    ci, va = m.col_idx.copy(), m.values.copy()
    for r in range(0, m.nrows, 7):
        s, e = m.row_ptr[r], m.row_ptr[r + 1]
        p = rng.permutation(e - s)
        ci[s:e], va[s:e] = ci[s:e][p], va[s:e][p]
    P = lib.Plan(m.nrows, m.ncols, m.row_ptr, ci, va, host_only=True, search_budget_ms=-1)
    d = P.describe()
    assert d["census"]["cols_sorted"] is False and abs(d["census"]["block_fill"]["3"] - 1.0) < 1e-12
    assert "light=bsell,block=3" in d["spec"]
    P.destroy()
