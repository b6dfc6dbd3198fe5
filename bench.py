#!/usr/bin/env python3
"""Benchmark: SpMV throughput of the searched plans on the five synthetic matrices, on one MI355X.

One "step" is one spmv_run on each configured matrix (inputs and plans resident in HBM before the
timed region).  Prints ONE JSON line: whole-job GFLOP/s (2 * sum(nnz) / sum(time)), per-matrix
GFLOP/s and achieved bandwidth as a fraction of the 8 TB/s HBM peak, the roofline record of the
dominant kernel (timed live with HIP events on the launch stream), and the CPU oracle timed on the
host cores as a baseline.
"""
import argparse
import json
import math
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK = 8.0e12   # bytes/s, MI355X published peak

CONFIGS = {
    "C1": ("uniform 10k x 10k, 10 nnz/row, fp64", "C1", "float64"),
    "C2": ("2D 5-point Laplacian 1024x1024 grid, fp64", "C2", "float64"),
    "C3": ("power-law 4.19M rows, mean 16 nnz/row, fp64", "C3", "float64"),
    "C4": ("FEM-like 3x3 blocks, 1M block rows, fp64", "C4", "float64"),
    "C5": ("hybrid 8.39M rows: 1000 rows x 100k + rows of 2-8, fp64", "C5", "float64"),
    "C5f32": ("hybrid 8.39M rows: 1000 rows x 100k + rows of 2-8, fp32", "C5", "float32"),
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--configs", default="C1,C2,C3,C4,C5,C5f32")
    ap.add_argument("--budget-ms", type=float, default=12000.0, help="search budget per matrix")
    ap.add_argument("--plan", default="", help="force this plan spec for every matrix (skips the search)")
    ap.add_argument("--plan-json", default="", help="JSON file {config: plan spec}: skip the search for those matrices")
    ap.add_argument("--save-plans", default="", help="write the chosen plan specs to this JSON file")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-jit", action="store_true", help="skip the comparison of run-time specialised against ahead-of-time kernels")
    ap.add_argument("--no-spmm", action="store_true", help="skip the multi-vector figure of the launch-bound matrices")
    ap.add_argument("--no-parity", action="store_true", help="skip the full-size check of every timed plan against the oracle")
    ap.add_argument("--verbose", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; SpMV here is a single-device kernel path and no "
              "multi-GPU figure exists (--gpus must be 1)", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import inputs
    import paper_2212_10432_amd as lib

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    dev = torch.device("cuda:0")
    lib.load()
    names = [c for c in args.configs.split(",") if c]
    log = (lambda *a: print(*a, file=sys.stderr, flush=True)) if args.verbose else (lambda *a: None)

    # Every device array of every plan comes from torch's caching allocator (the library's dev_alloc /
    # dev_free hooks): what the searches free goes back to torch's pool, not to the driver.  Returning
    # gigabytes to the driver shortly before a timed region was measured to slow the kernels that
    # follow by 3-4 % for seconds (C4: 225 instead of 217 us).
    live = {}

    def dev_alloc(nbytes):
        t = torch.empty(max(int(nbytes), 1), dtype=torch.uint8, device=dev)
        live[t.data_ptr()] = t
        return t.data_ptr()

    def dev_free(ptr):
        live.pop(ptr, None)

    torch_mem = (dev_alloc, dev_free)
    forced = json.load(open(args.plan_json)) if args.plan_json else {}
    # achievable streaming ceiling of this device (2 GiB read, 1 GiB copied to 1 GiB): the second
    # reference, beside the 8 TB/s peak, that achieved bandwidths are read against
    ceil_read, ceil_copy = lib.spmv_stream_ceiling(2 << 30, 5, torch.cuda.current_stream().cuda_stream)
    log(f"stream ceiling: read {ceil_read:.0f} GB/s, copy {ceil_copy:.0f} GB/s")
    items = []
    cpu = {"seconds": 0.0, "seconds_1t": 0.0, "flops": 0.0, "cores": 0, "sample": []}
    cache = {}
    for name in names:
        desc, fam, dt = CONFIGS[name]
        dt = np.dtype(dt)
        t0 = time.time()
        if fam not in cache:
            cache.clear()
            cache[fam] = inputs.FULL[fam]()
        m = cache[fam]
        vals = m.values.astype(dt)
        x = inputs.vector(m.ncols).astype(dt)
        t_gen = time.time() - t0
        t0 = time.time()
        plan = lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, vals, force_plan=args.plan or forced.get(name) or None,
                        search_budget_ms=args.budget_ms, verbosity=int(args.verbose), allocator=torch_mem,
                        search_cold=True)   # cache-sized matrices are timed cold below, so the search times them cold too
        t_plan = time.time() - t0
        d = plan.describe()
        b_plan, b_csr = plan.bytes()
        tdt = torch.float64 if dt == np.float64 else torch.float32
        footprint = b_plan
        # matrices that fit the 256 MB Infinity Cache are rotated over independent copies so that the
        # steady state streams from HBM; tiny ones (launch-latency bound) are left alone
        copies = 1
        if 16e6 < footprint < 512e6:
            copies = int(math.ceil(640e6 / footprint))
        plans = [plan] + [lib.Plan(m.nrows, m.ncols, m.row_ptr, m.col_idx, vals, force_plan=d["spec"], allocator=torch_mem)
                          for _ in range(copies - 1)]
        xs = [torch.from_numpy(x).to(dev) for _ in range(copies)]
        ys = [torch.empty(m.nrows, dtype=tdt, device=dev) for _ in range(copies)]
        # parity of the very plan that is timed, at full size (outside the timed region): one run,
        # every y element against the oracle's tolerance |y - y_ref| <= tau (|A||x|)
        parity = None
        if not args.no_parity or not args.no_cpu:
            import oracle
        if not args.no_parity:
            ys[0].fill_(float("nan"))
            plan.run(xs[0], ys[0])
            torch.cuda.synchronize()
            ok, worst = oracle.check(ys[0].cpu().numpy(), m.row_ptr, m.col_idx, vals, x, threads=len(os.sched_getaffinity(0)))
            parity = dict(parity_ok=bool(ok), worst_err_over_tol=float(worst))
            log(f"{name}: parity_ok={ok} worst error / tolerance = {worst:.3g}")
        if not args.no_cpu:
            threads = len(os.sched_getaffinity(0))
            for nt, key in ((threads, "seconds"), (1, "seconds_1t")):
                oracle.spmv(m.row_ptr, m.col_idx, vals, x, threads=nt)          # warm-up
                ts = []
                for _ in range(5):
                    t0 = time.perf_counter()
                    oracle.spmv(m.row_ptr, m.col_idx, vals, x, threads=nt)
                    ts.append(time.perf_counter() - t0)
                cpu[key] += sorted(ts)[2]
            cpu["flops"] += 2.0 * m.nnz
            cpu["cores"] = threads
            cpu["sample"].append(name)
        items.append(dict(name=name, desc=desc, nnz=m.nnz, nrows=m.nrows, dtype=dt.name, plans=plans, xs=xs, ys=ys,
                          copies=copies, b_plan=b_plan, b_csr=b_csr, spec=d["spec"], operators=d["operators"],
                          launches=plan.launch_names(), launch_bytes=[p["bytes"] for p in d["parts"]],
                          gen_s=t_gen, plan_s=t_plan, parity=parity, matrix=(m, vals),
                          search=[(c["spec"], c["run_us"], c["pred_us"], c["note"]) for c in d["search"]]))
        log(f"{name}: nnz={m.nnz} gen {t_gen:.1f}s plan {t_plan:.1f}s -> {d['spec']} (copies={copies})")
        del x
    cache.clear()

    # All launches go to one side stream.  A step is captured once into a HIP graph (kernel nodes
    # only: the library enqueues nothing else) and replayed, so that the launch-bound matrices are
    # not timed through the Python call overhead of this script.
    stream = torch.cuda.Stream()
    ncopies = max(it["copies"] for it in items)

    def step(k, only=None):
        for it in items:
            if only is not None and it is not only:
                continue
            i = k % it["copies"]
            it["plans"][i].run(it["xs"][i], it["ys"][i], stream.cuda_stream)

    def capture(nsteps, only=None):
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=stream):
            for k in range(nsteps):
                step(k, only)
        return g

    with torch.cuda.stream(stream):
        for k in range(max(args.warmup, 1)):
            step(k)
    torch.cuda.synchronize()
    # the timed region: exactly --steps steps, bracketed by synchronisation
    block = ncopies                                    # one graph = one rotation over the copies
    g_all = capture(block)
    g_all.replay()
    torch.cuda.synchronize()
    nblocks, rest = divmod(args.steps, block)
    t0 = time.perf_counter()
    for _ in range(nblocks):
        g_all.replay()
    with torch.cuda.stream(stream):
        for k in range(rest):
            step(k)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # per-matrix times (graph of `reps` runs, HIP events on the launch stream) and per-launch times
    for it in items:
        reps = max(20, it["copies"] * 2)
        reps -= reps % it["copies"]
        g = capture(reps, it)
        g.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        nrep = max(1, min(50, int(math.ceil(args.steps / reps))))
        with torch.cuda.stream(stream):
            e0.record(stream)
            for _ in range(nrep):
                g.replay()
            e1.record(stream)
        e1.synchronize()
        it["ms"] = e0.elapsed_time(e1) / (reps * nrep)
        it["ms_graph"] = it["ms"]
        if it["copies"] == 1:
            # back-to-back launches from the library's own timing loop (what a C caller sees)
            it["ms_loop"] = it["plans"][0].time(it["xs"][0], it["ys"][0], stream.cuda_stream, 25) * 1e-3   # reported beside, never used
        # warm (cache-resident) figure for rotated matrices: the same copy every time
        if it["copies"] > 1:
            gw = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gw, stream=stream):
                for k in range(reps):
                    it["plans"][0].run(it["xs"][0], it["ys"][0], stream.cuda_stream)
            gw.replay()
            torch.cuda.synchronize()
            with torch.cuda.stream(stream):
                e0.record(stream)
                for _ in range(nrep):
                    gw.replay()
                e1.record(stream)
            e1.synchronize()
            it["ms_warm"] = e0.elapsed_time(e1) / (reps * nrep)
        # per launch: each launch repeated back to back between two HIP events on the launch stream
        # (rotated over the copies for the cache-sized matrices)
        per = np.zeros(len(it["launches"]))
        for i in range(it["copies"]):
            per += np.array(it["plans"][i].time_launches(it["xs"][i], it["ys"][i], stream.cuda_stream, 10 if it["copies"] == 1 else 1))
        it["launch_ms"] = (per / it["copies"] * 1e-3).tolist()

    # side records, after every timing above is done (they build further plans and buffers)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for it in items:
        # run-time specialised kernels on / off for this plan, both timed the same way (the library's
        # loop of back-to-back launches on the same copy: cache-warm for the small matrices)
        if not args.no_jit:
            spec = it["spec"]
            if ",jit=1" in spec:
                other = spec.replace(",jit=1", "")
            elif "}" in spec:
                other = spec.replace("}", ",jit=1}", 1)
            else:
                other = spec + ",jit=1"
            m_, vals_ = it["matrix"]
            alt = lib.Plan(m_.nrows, m_.ncols, m_.row_ptr, m_.col_idx, vals_, force_plan=other, allocator=torch_mem)
            t_this = it["plans"][0].time(it["xs"][0], it["ys"][0], stream.cuda_stream, 25)
            t_alt = alt.time(it["xs"][0], it["ys"][0], stream.cuda_stream, 25)
            on, off = (t_this, t_alt) if ",jit=1" in spec else (t_alt, t_this)
            it["jit"] = dict(jit_on_us=on, jit_off_us=off, timed_plan_uses_jit=",jit=1" in spec,
                             launches_specialised=sum(1 for q in (alt if ",jit=1" not in spec else it["plans"][0]).describe()["parts"] if q["jit"]))
            alt.destroy()
        # several right-hand sides through one plan (the launch-bound matrices are where it pays)
        if it["name"] in ("C1", "C2") and not args.no_spmm:
            k = 8
            tdt_ = it["xs"][0].dtype
            X = torch.stack([it["xs"][0]] * k).contiguous()
            Y = torch.empty((k, it["nrows"]), dtype=tdt_, device=dev)
            with torch.cuda.stream(stream):
                for _ in range(3):
                    it["plans"][0].run_multi(X, Y, stream.cuda_stream)
                e0.record(stream)
                for _ in range(50):
                    it["plans"][0].run_multi(X, Y, stream.cuda_stream)
                e1.record(stream)
            e1.synchronize()
            it["spmm"] = dict(k=k, us_per_call=e0.elapsed_time(e1) / 50 * 1e3, us_per_vector=e0.elapsed_time(e1) / 50 / k * 1e3)
            del X, Y

    per_config = []
    tot_ms = sum(it["ms"] for it in items)
    tot_nnz = sum(it["nnz"] for it in items)
    for it in items:
        credited = min(it["b_plan"], it["b_csr"])
        t = it["ms"] * 1e-3
        rec = dict(config=it["name"], workload=it["desc"], dtype=it["dtype"], nnz=it["nnz"], us=it["ms"] * 1e3,
                   gflops=2.0 * it["nnz"] / t / 1e9, bytes_csr=it["b_csr"], bytes_plan=it["b_plan"],
                   gbps_credited=credited / t / 1e9, hbm_frac=credited / t / HBM_PEAK,
                   frac_of_read_ceiling=credited / t / 1e9 / ceil_read,
                   gbps_csr=it["b_csr"] / t / 1e9, gbps_plan=it["b_plan"] / t / 1e9,
                   plan=it["spec"], operators=it["operators"], launches=it["launches"],
                   launch_us=[v * 1e3 for v in it["launch_ms"]], launch_bytes=it["launch_bytes"],
                   rotated_copies=it["copies"],
                   # what this plan's own bytes would take at the read ceiling measured in this run:
                   # the time below which only a plan that moves fewer bytes can go
                   design_floor_us=it["b_plan"] / (ceil_read * 1e9) * 1e6,
                   csr_floor_us=it["b_csr"] / (ceil_read * 1e9) * 1e6,
                   plan_create_s=it["plan_s"], search=it["search"])
        if it["parity"] is not None:
            rec.update(it["parity"])
        if "jit" in it:
            rec["jit"] = it["jit"]
        if "spmm" in it:
            rec["spmm"] = it["spmm"]
        if "ms_warm" in it:
            rec["us_cache_warm"] = it["ms_warm"] * 1e3
        rec["us_graph_replay"] = it["ms_graph"] * 1e3
        if "ms_loop" in it:
            rec["us_stream_loop"] = it["ms_loop"] * 1e3
        per_config.append(rec)

    def geomean(v):
        return float(np.exp(np.mean(np.log(v)))) if len(v) else None

    # one score per configured matrix: the fp64 and fp32 runs of the hybrid matrix count as one
    # (their geometric mean), so that the mean below is over the five matrices
    by_matrix = {}
    for r in per_config:
        by_matrix.setdefault(CONFIGS[r["config"]][1], []).append(r["hbm_frac"])
    matrix_frac = {k: geomean(v) for k, v in by_matrix.items()}

    # dominant kernel: the launch with the largest share of a step; its algorithmic bytes are the
    # format arrays it reads plus the x, scratch and y elements it touches (plan description)
    dit, di = max(((it, i) for it in items for i in range(len(it["launches"]))), key=lambda p: p[0]["launch_ms"][p[1]])
    dom_bytes = dit["launch_bytes"][di]
    achieved = dom_bytes / (dit["launch_ms"][di] * 1e-3) / 1e9
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get(f"{dit['name']}:{dit['launches'][di]}")
        except Exception:
            traffic = None
    roofline = dict(bound="hbm", achieved=achieved, peak=HBM_PEAK / 1e9, unit="GB/s", frac=achieved / (HBM_PEAK / 1e9),
                    frac_of_read_ceiling=achieved / ceil_read,
                    traffic=traffic, kernel=f"{dit['name']}:{dit['launches'][di]}",
                    launch_us=dit["launch_ms"][di] * 1e3, algorithmic_bytes=dom_bytes)
    if args.save_plans:
        json.dump({it["name"]: it["spec"] for it in items}, open(args.save_plans, "w"), indent=1)

    out = {
        "metric": "SpMV GFLOP/s (2*nnz/time) and achieved HBM GB/s (fraction of 8 TB/s peak) per matrix, 1 MI355X",
        "value": 2.0 * tot_nnz / (wall_ms * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall_ms, "sum_of_per_matrix_ms": tot_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64" if all(it["dtype"] == "float64" for it in items) else "f64+f32",
        "data": "synthetic",
        "config": {"workload": "+".join(names) + " (seeded synthetic stand-ins for SuiteSparse), one spmv_run per matrix per step"},
        "geomean_gflops": geomean([r["gflops"] for r in per_config]),
        "hbm_frac_per_matrix": matrix_frac,
        "geomean_hbm_frac": geomean(list(matrix_frac.values())),
        "geomean_hbm_frac_without_C1": geomean([v for k, v in matrix_frac.items() if k != "C1"]),
        "parity_ok": (all(r["parity_ok"] for r in per_config) if all("parity_ok" in r for r in per_config) else None),
        "stream_ceiling": {"read_gbps": ceil_read, "copy_gbps": ceil_copy, "bytes": 2 << 30,
                           "note": "measured at start-up with the library's spmv_stream_ceiling"},
        "per_config": per_config,
        "roofline": roofline,
    }
    if not args.no_cpu and cpu["seconds"] > 0:
        model = ""
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        out["cpu_baseline"] = dict(value=cpu["flops"] / cpu["seconds"] / 1e9, unit="GFLOP/s", cores=cpu["cores"],
                                   kind="oracle", value_1_thread=cpu["flops"] / cpu["seconds_1t"] / 1e9, cpu_model=model,
                                   sample="one full oracle SpMV (median of 5 after a warm-up; rows split over all cores, and on "
                                          "one thread) on each of " + ",".join(cpu["sample"]))
    for it in items:
        for p in it["plans"]:
            p.destroy()
    print(json.dumps(out))


if __name__ == "__main__":
    main()
