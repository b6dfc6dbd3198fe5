"""Command line: a Matrix Market file in, the machine-chosen plan and its measured speed out
(the usage the paper describes for its tool: Section III and the artifact description).

    python -m paper_2212_10432_amd matrix.mtx [--dtype f64|f32] [--plan SPEC] [--budget-ms MS]
                                              [--host-only] [--json]

Without --host-only the plan is searched (or built from --plan) and timed on the GPU; with it the
forced plan is only built in host memory and described.  Nothing here computes on the CPU."""
import argparse
import json
import sys

import numpy as np

from . import Plan, spmv_mm_read


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(prog="python -m paper_2212_10432_amd", description=__doc__.split("\n")[0])
    ap.add_argument("matrix", help="Matrix Market coordinate file (.mtx)")
    ap.add_argument("--dtype", choices=["f64", "f32"], default="f64")
    ap.add_argument("--plan", default="", help="plan-spec string: skip the search")
    ap.add_argument("--budget-ms", type=float, default=0.0, help="search budget (0 = library default)")
    ap.add_argument("--host-only", action="store_true", help="build the forced plan in host memory, do not run")
    ap.add_argument("--json", action="store_true", help="print the full plan description as JSON")
    args = ap.parse_args(argv)
    dt = np.float64 if args.dtype == "f64" else np.float32
    nrows, ncols, row_ptr, col_idx, values = spmv_mm_read(args.matrix, dt)
    print(f"{args.matrix}: {nrows} x {ncols}, {values.size} stored entries, {args.dtype}", file=sys.stderr)
    if args.host_only:
        if not args.plan:
            ap.error("--host-only needs --plan")
        plan = Plan(nrows, ncols, row_ptr, col_idx, values, force_plan=args.plan, host_only=True)
        d = plan.describe()
        print(json.dumps(d) if args.json else f"plan: {d['spec']}\noperators: {d['operators']}\nbytes: plan {d['bytes_plan']}, csr {d['bytes_csr']}")
        plan.destroy()
        return 0
    import torch
    if not torch.cuda.is_available():
        print("no GPU: use --host-only --plan SPEC to inspect a plan", file=sys.stderr)
        return 2
    plan = Plan(nrows, ncols, row_ptr, col_idx, values, force_plan=args.plan or None, search_budget_ms=args.budget_ms)
    tdt = torch.float64 if dt == np.float64 else torch.float32
    x = torch.ones(ncols, dtype=tdt, device="cuda")
    y = torch.empty(nrows, dtype=tdt, device="cuda")
    us = plan.time(x, y)
    d = plan.describe()
    if args.json:
        d["run_us"] = us
        print(json.dumps(d))
    else:
        credited = min(d["bytes_plan"], d["bytes_csr"])
        print(f"plan: {d['spec']}\noperators: {d['operators']}\nlaunches: {', '.join(plan.launch_names())}\n"
              f"time: {us:.2f} us per SpMV, {2.0 * values.size / us / 1e3:.1f} GFLOP/s, "
              f"{credited / us / 1e3:.1f} GB/s of credited bytes")
    plan.destroy()
    return 0


if __name__ == "__main__":
    sys.exit(main())
