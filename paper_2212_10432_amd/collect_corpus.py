"""Writes the corpus the search's cost model is trained from (paper_2212_10432_amd/cost_corpus.tsv).

Runs the search, without a model, on seeded synthetic matrices of the five benchmark families at
several sizes and in both value types, on the GPU of this machine; every candidate the searches time
is appended to the corpus (census features, plan spec, microseconds).  Usage, from the repository root:

    python -m paper_2212_10432_amd.collect_corpus [--more] [--full] [--out FILE] [--budget-ms MS]

--more adds the families at other sizes, densities and exponents; --full adds the five matrices at
their benchmark sizes (minutes instead of seconds)."""
import argparse
import os
import sys

import numpy as np


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--out", default=None)
    ap.add_argument("--full", action="store_true")
    ap.add_argument("--more", action="store_true")
    ap.add_argument("--budget-ms", type=float, default=20000.0)
    args = ap.parse_args()
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    if root not in sys.path:
        sys.path.insert(0, root)
    import inputs
    import paper_2212_10432_amd as lib

    out = args.out or lib.COST_CORPUS
    makers = [
        ("uniform-10k", lambda: inputs.uniform(n=10_000, k=10)), ("uniform-200k", lambda: inputs.uniform(n=200_000, k=12)),
        ("uniform-2m", lambda: inputs.uniform(n=2_000_000, k=6)),
        ("laplace-67", lambda: inputs.laplace2d(g=67)), ("laplace-400", lambda: inputs.laplace2d(g=400)),
        ("powerlaw-70k", lambda: inputs.powerlaw(n=70_001, cap=9_000)), ("powerlaw-500k", lambda: inputs.powerlaw(n=500_000, cap=30_000)),
        ("fem-10k", lambda: inputs.fem3(nb=10_007, window=500)), ("fem-100k", lambda: inputs.fem3(nb=100_000, window=1000)),
        ("hybrid-130k", lambda: inputs.hybrid(n=130_003, n_heavy=7, heavy_len=20_000)),
        ("hybrid-1m", lambda: inputs.hybrid(n=1_000_000, n_heavy=100, heavy_len=50_000)),
    ]
    if args.more:   # the same families at other sizes, densities and exponents
        makers += [
            ("uniform-50k-k30", lambda: inputs.uniform(n=50_000, k=30)), ("uniform-1m-k3", lambda: inputs.uniform(n=1_000_000, k=3)),
            ("uniform-4m-k16", lambda: inputs.uniform(n=4_000_000, k=16)),
            ("laplace-150", lambda: inputs.laplace2d(g=150)), ("laplace-1500", lambda: inputs.laplace2d(g=1500)),
            ("powerlaw-200k-e1.8", lambda: inputs.powerlaw(n=200_000, cap=20_000, exponent=1.8)),
            ("powerlaw-2m", lambda: inputs.powerlaw(n=2_000_000, cap=60_000)),
            ("powerlaw-1m-e2.6", lambda: inputs.powerlaw(n=1_000_000, cap=10_000, exponent=2.6)),
            ("fem-30k-w100", lambda: inputs.fem3(nb=30_000, window=100)), ("fem-400k", lambda: inputs.fem3(nb=400_000, window=3000)),
            ("hybrid-400k", lambda: inputs.hybrid(n=400_000, n_heavy=30, heavy_len=100_000)),
            ("hybrid-4m", lambda: inputs.hybrid(n=4_000_000, n_heavy=400, heavy_len=60_000, lo=1, hi=12)),
        ]
    if args.full:
        makers += [(f"full-{k}", inputs.FULL[k]) for k in ("C1", "C2", "C3", "C4", "C5")]
    for name, make in makers:
        m = make()
        for dt in (np.float64, np.float32):
            P = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, m.values.astype(dt), search_budget_ms=args.budget_ms,
                         cost_model=None, cost_log=out)
            d = P.describe()
            timed = [c for c in d["search"] if c["run_us"] >= 0]
            print(f"{name} {np.dtype(dt).name}: {len(timed)} candidates timed, kept {d['spec']}", flush=True)
            P.destroy()
        del m
    print("corpus:", out, sum(1 for _ in open(out)), "lines")


if __name__ == "__main__":
    main()
