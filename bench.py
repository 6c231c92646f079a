#!/usr/bin/env python3
"""Benchmark of the ADMM sweep on one MI355X.

A "step" is one full ADMM iteration (W-update, Z-update for every layer and community, last-layer
solve, dual step) on a synthetic SBM workload already resident in HBM.  Prints ONE JSON line:
ADMM iterations/s for the whole job, the roofline of the dominant kernel class measured live with
HIP events on the library's stream, the aggregation's own roofline and its measured gather ceiling,
a short leg on the GEMM-heavy configuration that prices the wide products against the matrix-core
peak of the dtype they issue (both product paths), and the CPU oracle timed on two bounded samples
of the same recipe.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..5] [--scale S]
"""
import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# published MI355X peaks
HBM_PEAK_GBS = 8000.0
MFMA_FP32_PEAK_TFLOPS = 157.3
MFMA_BF16_PEAK_TFLOPS = 2500.0
SPLIT_PRODUCTS = 6      # bf16 MFMA products issued per fp32 product in the split kernels

# A kernel class is priced against the MFMA roofline if its arithmetic intensity (algorithmic flops per
# algorithmic byte over the timed region) is above the machine balance, else against HBM bandwidth.
MACHINE_BALANCE = MFMA_FP32_PEAK_TFLOPS * 1e12 / (HBM_PEAK_GBS * 1e9)      # flop per byte

DTYPE = ("f32 state and accumulation; products wider than 32 columns issued as 6 bf16 MFMA terms of exactly split fp32 "
         "operands (fp32 MFMA with gemm_split=0), narrower ones as fp32 MFMA; search decisions and reductions in f64")

# Bytes per launch group that crossed the L2 -> fabric boundary (FETCH_SIZE + WRITE_SIZE of rocprofv3 --pmc, each scaled
# by what a plain copy of known size reads) are not measured here: traffic_table.py writes them from the counter runs
# into this file, together with the commit and a hash of the kernel sources they were measured at.
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "sweep_memory_traffic_powerlaw_dcsbm_2M.json")
KERNEL_SOURCES = ["cadmm_api.hip", "spmm.hip", "gemm.hip", "elementwise.hip", "kernels.h", "host_graph.cpp", "host_graph.h"]

# CPU-oracle samples: two (scale of N, iterations) per workload, together sized for about 20-30 s of host time
ORACLE_SAMPLES = {1: ((0.5, 10), (1.0, 10)), 2: ((0.125, 4), (0.25, 4)), 3: ((0.01, 3), (0.02, 3)),
                  4: ((0.002, 6), (0.004, 6)), 5: ((0.002, 2), (0.004, 2)), 6: ((0.05, 3), (0.1, 3)),
                  7: ((0.1, 3), (0.2, 3))}


def kernel_source_hash():
    h = hashlib.sha256()
    for name in KERNEL_SOURCES:
        with open(os.path.join(ROOT, "paper_2112_09335_amd", "csrc", name), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def load_traffic(workload):
    """Measured traffic per kernel class for the default workload, or nothing if no table was written for it."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f)
    except (OSError, ValueError):
        return {}, None
    if t.get("workload") != workload:
        return {}, None
    src = dict(file=os.path.relpath(TRAFFIC_FILE, ROOT), commit=t.get("commit"), measured=t.get("date"),
               kernel_source_hash=t.get("kernel_source_hash"),
               stale=t.get("kernel_source_hash") != kernel_source_hash())
    return t.get("classes", {}), src


def roofline_entry(name, p):
    sec = p["ms"] * 1e-3
    if sec <= 0 or p["records"] == 0:
        return None
    per_launch_ms = p["ms"] / p["records"]
    if name.startswith(("gemm_nn_split", "gemm_tn_split")) and p["bytes"] > 0 and p["flops"] / p["bytes"] > MACHINE_BALANCE:
        # fp32-exact product issued as six bf16 MFMA products: priced in issued bf16 flops against the bf16 peak
        ach = SPLIT_PRODUCTS * p["flops"] / sec / 1e12
        return dict(kernel=name, bound="mfma", achieved=ach, peak=MFMA_BF16_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=ach / MFMA_BF16_PEAK_TFLOPS, traffic=None, avg_launch_ms=per_launch_ms,
                    launches=p["records"], share_of_step=None, fp32_product_TFLOPs=p["flops"] / sec / 1e12,
                    issued="bf16 x6")
    if name.startswith("gemm") and p["bytes"] > 0 and p["flops"] / p["bytes"] > MACHINE_BALANCE:
        ach = p["flops"] / sec / 1e12
        return dict(kernel=name, bound="mfma", achieved=ach, peak=MFMA_FP32_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=ach / MFMA_FP32_PEAK_TFLOPS, traffic=None, avg_launch_ms=per_launch_ms,
                    launches=p["records"], share_of_step=None, issued="fp32")
    ach = p["bytes"] / sec / 1e9
    return dict(kernel=name, bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS,
                traffic=None, avg_launch_ms=per_launch_ms, launches=p["records"], share_of_step=None)


def timed_run(solver, steps, warmup):
    """(seconds of a plain run of `steps` iterations, per-class profile of a second, event-timed run, its seconds)."""
    import torch
    solver.run(warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    solver.run(steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    solver.profile(True)
    t0 = time.perf_counter()
    solver.run(steps)
    prof = solver.get_profile()          # synchronises
    dt_prof = time.perf_counter() - t0
    solver.profile(False)
    return dt, prof, dt_prof


def class_entries(prof):
    total_ms = sum(p["ms"] for p in prof.values())
    entries = []
    for name, p in prof.items():
        e = roofline_entry(name, p)
        if e is not None:
            e["share_of_step"] = p["ms"] / total_ms if total_ms > 0 else None
            entries.append(e)
    entries.sort(key=lambda e: -e["share_of_step"])
    return entries


def mfma_leg(steps, warmup):
    """The wide products on the GEMM-heavy configuration (8 layers of 512 units, N = 500 000), both product paths:
    achieved rate per kernel class against the matrix-core peak of the dtype it issues."""
    import torch
    from paper_2112_09335_amd import binding, synth
    w = synth.config(5)
    solver = binding.Solver.from_workload(w, 0)
    out = {"workload": f"configs[4] {w.name}", "N": w.N, "widths": w.dims, "steps": steps, "paths": {}}
    try:
        for split in (1, 0):
            solver.tune("gemm_split", split)
            dt, prof, _ = timed_run(solver, steps, warmup)
            kernels = [{k: e[k] for k in ("kernel", "issued", "achieved", "peak", "unit", "frac", "avg_launch_ms", "launches",
                                          "share_of_step") if k in e}
                       | ({"fp32_product_TFLOPs": e["fp32_product_TFLOPs"]} if "fp32_product_TFLOPs" in e else {})
                       for e in class_entries(prof) if e["bound"] == "mfma"]
            out["paths"]["bf16_split" if split else "fp32"] = dict(gemm_split=split, iterations_per_s=steps / dt,
                                                                  ms_per_step=1e3 * dt / steps, kernels=kernels)
        # what the matrix cores issue from registers alone on this machine: the ceiling the fractions above are read against
        out["calibration"] = {
            "fp32_mfma_TFLOPs": solver.op_calibrate("mfma", 20000, 3),
            "bf16_mfma_TFLOPs": solver.op_calibrate("mfma_bf16", 20000, 3),
            "bf16_mfma_TFLOPs_with_6_vector_instructions_each": solver.op_calibrate("mfma_bf16_valu6", 20000, 3),
        }
    finally:
        solver.tune("gemm_split", 1)
        solver.close()
        torch.cuda.empty_cache()
    return out


def cpu_baseline(index, full_N, full_nnz, communities=None, schedule=0, step_policy=0):
    """The oracle as it stands, timed on two smaller instances of the same recipe with a pinned thread count; the
    full-size figure extrapolates with the exponent measured between the two (rate ~ nnz^-exponent)."""
    import math
    import psutil
    from threadpoolctl import threadpool_limits
    from oracle.admm import make_oracle
    from paper_2112_09335_amd import synth
    threads = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    threads = max(1, min(threads, int(os.environ.get("OMP_NUM_THREADS", threads))))
    points = []
    with threadpool_limits(limits=threads):
        for scale, iters in ORACLE_SAMPLES[index]:
            w = synth.config(index, scale, communities)
            w.hyper["schedule"] = schedule
            w.hyper["step_policy"] = step_policy
            orc = make_oracle(w)
            orc.iterate(1)               # first iteration is atypical (zero gradients at the forward-pass start)
            t0 = time.perf_counter()
            orc.iterate(iters)
            dt = time.perf_counter() - t0
            points.append(dict(N=w.N, M=w.M, nnz=orc.g.nnz, iterations=iters, seconds=dt, iterations_per_s=iters / dt))
    # the smaller sample once more on ONE thread (the oracle is numpy: at these sizes most of its time is the plain
    # Python loops over communities, which no thread count changes)
    scale1, _ = ORACLE_SAMPLES[index][0]
    with threadpool_limits(limits=1):
        w = synth.config(index, scale1, communities)
        w.hyper["schedule"] = schedule
        w.hyper["step_policy"] = step_policy
        orc = make_oracle(w)
        orc.iterate(1)
        t0 = time.perf_counter()
        orc.iterate(2)
        single = dict(N=w.N, threads=1, iterations=2, seconds=time.perf_counter() - t0)
        single["iterations_per_s"] = 2 / single["seconds"]
    a, b = points
    # seconds per iteration = fixed + per_entry * nnz: the fixed part is the per-block overhead of the plain Python loops
    # over communities, the rest grows with the graph
    ta, tb = 1.0 / a["iterations_per_s"], 1.0 / b["iterations_per_s"]
    per_entry = (tb - ta) / float(b["nnz"] - a["nnz"]) if b["nnz"] > a["nnz"] else tb / b["nnz"]
    per_entry = max(per_entry, 0.0)
    fixed = max(tb - per_entry * b["nnz"], 0.0)
    exponent = math.log(tb / ta) / math.log(b["nnz"] / a["nnz"]) if b["nnz"] > a["nnz"] and ta > 0 else 1.0
    at_full = b["nnz"] >= full_nnz
    value = b["iterations_per_s"] if at_full else 1.0 / (fixed + per_entry * float(full_nnz))
    return dict(value=value, unit="iterations/s", cores=threads, kind="oracle",
                physical_cores=psutil.cpu_count(logical=False), logical_cores=psutil.cpu_count(logical=True),
                sample=(f"oracle iterations timed at N={a['N']} ({a['iterations_per_s']:.3f} it/s) and N={b['N']} "
                        f"({b['iterations_per_s']:.3f} it/s) of the same recipe, {threads} threads; "
                        + ("value = the rate at the larger sample, which is the full size" if at_full else
                           f"value = 1 / (fixed + per_entry * nnz_full) with fixed = {fixed:.3f} s and per_entry = "
                           f"{per_entry:.3e} s fitted through the two samples (extrapolation to N={full_N}, "
                           f"nnz={full_nnz}); the power law through the same two points has exponent {exponent:.2f}")),
                samples=points, single_thread_sample=single, seconds_per_iteration_fixed=fixed, seconds_per_iteration_per_entry=per_entry,
                scaling_exponent=exponent, extrapolated=not at_full)


def full_size_oracle_forms(w, solver, stats):
    """The oracle's full-graph forms timed at the FULL size of the workload, on the library's own state: Eq. 1 once
    (`stats_full_graph`: every layer's aggregation, product and penalty) and two evaluations of phi_l per layer (what a
    W step that accepts its first candidate evaluates besides its gradient).  Not an iteration -- the oracle's iteration
    works in the message form over M x M community blocks and is far slower -- but a measured full-size anchor next to
    the extrapolated figure, and a check of the library's readout at the size the benchmark times."""
    import numpy as np
    from threadpoolctl import threadpool_limits
    from oracle.admm import AdmmOracle
    from oracle.graph import OracleGraph
    threads = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    threads = max(1, min(threads, int(os.environ.get("OMP_NUM_THREADS", threads))))
    h = w.hyper
    with threadpool_limits(limits=threads):
        t0 = time.perf_counter()
        g = OracleGraph(w.N, w.src, w.dst, w.M, w.comm, split=False)
        o = AdmmOracle(g, w.dims, nu=h["nu"], rho=h["rho"], tau0=h["tau0"], theta0=h["theta0"], eta=h["eta"],
                       max_backtrack=h["max_backtrack"], fista_iters=h["fista_iters"], risk=h["risk"])
        o.set_data(w.X, w.labels)
        L = w.L
        W = [None] + [solver.get_W(l).astype(np.float64) for l in range(1, L + 1)]
        Z = [o.Z[0]] + [g.to_new(solver.get_Z(l).astype(np.float64)) for l in range(1, L + 1)]
        U = g.to_new(solver.get_U().astype(np.float64))
        o.phi_full_graph(1, W[1], Z[0], Z[1], U)          # forms and keeps A~ Z_0, as the library does at set-up
        t_setup = time.perf_counter() - t0
        t0 = time.perf_counter()
        so = o.stats_full_graph(W, Z, U)
        t_eq1 = time.perf_counter() - t0
        t_phi = []
        for l in range(1, L + 1):
            t0 = time.perf_counter()
            o.phi_full_graph(l, W[l], Z[l - 1], Z[l], U)
            o.phi_full_graph(l, W[l], Z[l - 1], Z[l], U)
            t_phi.append(time.perf_counter() - t0)
    return dict(what="oracle full-graph forms at full size on the library's state: Eq. 1 once, and two evaluations of "
                     "phi_l per layer; a lower bound on the CPU time of an iteration, not an iteration",
                N=w.N, threads=threads, seconds_setup=t_setup, seconds_eq1=t_eq1, seconds_two_phi_per_layer=t_phi,
                seconds_total=t_eq1 + sum(t_phi), iterations_per_s_upper_bound=1.0 / (t_eq1 + sum(t_phi)),
                objective_oracle=so["objective"], objective_library=stats["objective"],
                objective_rel_diff=abs(so["objective"] - stats["objective"]) / abs(so["objective"]))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # 32 = two periods of the exact re-evaluation of the carried pre-activations (every 16 iterations), so the
    # timed region holds its share of them
    ap.add_argument("--steps", type=int, default=32)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", type=int, default=4, help="benchmark configuration 1..5; 6, 7: shapes of the "
                    "paper's speed-up experiment (synth.config)")
    ap.add_argument("--communities", type=int, default=None, help="override the number of communities M")
    ap.add_argument("--schedule", type=int, default=0, help="0 = Algorithm 1, 1 = layer by layer (serial baseline)")
    ap.add_argument("--step-policy", type=int, default=0, help="0 = step parameters never shrink, 1 = a search "
                    "starts one notch below the last accepted value")
    ap.add_argument("--fista-mode", type=int, default=0, help="last layer: 0 = FISTA per row with the constant step, "
                    "1 = FISTA with backtracking on the blocks Z_{L,m}")
    ap.add_argument("--partition", choices=["planted", "builtin"], default="planted",
                    help="communities: the generator's planted blocks, or the library's own partitioner")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink N (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-mfma-leg", action="store_true", help="skip the short leg on the GEMM-heavy configuration "
                    "and the fp32-MFMA run of the headline workload")
    ap.add_argument("--mfma-steps", type=int, default=3)
    ap.add_argument("--no-full-size-oracle", action="store_true", help="skip timing the oracle's full-graph forms at "
                    "the full size of the workload (about a minute of host work)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding or collectives are part of it); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2112_09335_amd import binding, synth

    t0 = time.perf_counter()
    w = synth.config(args.workload, args.scale, args.communities)
    w.hyper["schedule"] = args.schedule
    w.hyper["step_policy"] = args.step_policy
    w.hyper["fista_mode"] = args.fista_mode
    t_gen = time.perf_counter() - t0
    if args.partition == "builtin":
        t0 = time.perf_counter()
        host = binding.Solver(device=-1)
        w.comm = host.partition(w.N, w.src, w.dst, w.M)
        host.close()
        print(f"# built-in partitioner: {time.perf_counter() - t0:.2f} s on the host", file=sys.stderr, flush=True)
    t0 = time.perf_counter()
    solver = binding.Solver.from_workload(w, 0)
    torch.cuda.synchronize()
    t_setup = time.perf_counter() - t0
    nnz, nseg, nhalo = solver.graph_sizes()
    print(f"# workload {w.name}: N={w.N} M={w.M} E={w.E} nnz={nnz} segments={nseg} halo_rows={nhalo} "
          f"dims={w.dims}; generated in {t_gen:.1f} s, built+uploaded+initialised in {t_setup:.1f} s, "
          f"workspace {solver.workspace_bytes() / 2**30:.2f} GiB", file=sys.stderr, flush=True)

    # timed region 1: the plain run, nothing but the sweep on the stream; region 2: the same number of steps with
    # every launch group bracketed by HIP events on the library's stream
    dt, prof, dt_prof = timed_run(solver, args.steps, args.warmup)
    stats = solver.eval()

    entries = class_entries(prof)
    workload_key = f"configs[{args.workload - 1}] {w.name}" + ("" if args.scale == 1.0 else f" scale {args.scale}")
    traffic, traffic_source = load_traffic(workload_key) if args.scale == 1.0 else ({}, None)
    for e in entries:
        e["traffic"] = traffic.get(e["kernel"])
    dominant = dict(entries[0]) if entries else None
    spmm_keys = [k for k in prof if k.startswith("spmm")]
    spmm_ms = sum(prof[k]["ms"] for k in spmm_keys)
    spmm_bytes = sum(prof[k]["bytes"] for k in spmm_keys)
    spmm_flops = sum(prof[k]["flops"] for k in spmm_keys)
    rows_entry = next((e for e in entries if e["kernel"] == "spmm_rows_kernel[rows]"), None)

    # what the memory system serves to this graph's gathers at the narrowest aggregation width of the sweep, with no
    # row structure around them (cadmm_op_calibrate kinds 2, 3): the measured ceiling of the aggregation kernels
    gather_width = min(c for c in w.dims[1:] if c % 4 == 0) if any(c % 4 == 0 for c in w.dims[1:]) else None
    gather = None
    if gather_width and gather_width <= 256:
        pw = 4
        while pw < gather_width:
            pw *= 2
        rate_rows = solver.op_calibrate("gather", pw, 3)
        rate_segs = solver.op_calibrate("gather_segments", pw, 3)
        per_gather = 8.0 + 4.0 * pw
        gather = dict(row_floats=pw, rows_requested_GBs=rate_rows, rows_G_gathers_per_s=rate_rows / per_gather,
                      segments_requested_GBs=rate_segs, segments_G_gathers_per_s=rate_segs / per_gather,
                      copy_GBs=solver.op_calibrate("copy", 1 << 28, 3))
        if rows_entry is not None and gather_width == pw:
            # the row aggregation of that width issues nnz gathers (plus padding) per launch
            rows_entry["G_gathers_per_s"] = nnz / (rows_entry["avg_launch_ms"] * 1e-3) / 1e9
            rows_entry["frac_of_gather_ceiling"] = rows_entry["G_gathers_per_s"] / gather["rows_G_gathers_per_s"]

    out = {
        "metric": "ADMM iterations/sec (all layers+communities)",
        "value": args.steps / dt,
        "unit": "iterations/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": DTYPE,
        "data": "synthetic",
        "config": {"workload": workload_key, "N": w.N, "communities": w.M,
                   "edges": w.E, "nnz": nnz, "layers": w.L, "widths": w.dims, "scale": args.scale,
                   "schedule": args.schedule, "step_policy": args.step_policy, "fista_mode": args.fista_mode,
                   "partition": args.partition},
        "roofline": None if dominant is None else {k: dominant[k] for k in
                                                   ("bound", "achieved", "peak", "unit", "frac", "traffic")},
        "dominant_kernel": None if dominant is None else dominant["kernel"],
        "traffic_source": traffic_source,
        "kernels": entries,
        # all aggregation launches of the timed steps together.  achieved_GBs uses the algorithmic minimum (every
        # row of the gathered matrix read once); gather_volume_GBs counts what the kernel actually requests from
        # the memory system, nnz gathers of 4*width bytes (2 flops per gathered float) plus the entries
        "spmm": {"achieved_GBs": spmm_bytes / (spmm_ms * 1e-3) / 1e9 if spmm_ms > 0 else None,
                 "frac_of_hbm_peak": spmm_bytes / (spmm_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if spmm_ms > 0 else None,
                 "edges_features_per_s": 0.5 * spmm_flops / (spmm_ms * 1e-3) if spmm_ms > 0 else None,
                 "gather_volume_GBs": (2.0 * spmm_flops + 8.0 * nnz * sum(prof[k]["records"] for k in spmm_keys))
                 / (spmm_ms * 1e-3) / 1e9 if spmm_ms > 0 else None,
                 "rows_kernel": None if rows_entry is None else {k: rows_entry[k] for k in rows_entry
                                                                 if k in ("bound", "achieved", "peak", "unit", "frac", "traffic",
                                                                          "avg_launch_ms", "launches", "share_of_step",
                                                                          "G_gathers_per_s", "frac_of_gather_ceiling")},
                 "gather_calibration": gather},
        "ms_per_step_with_event_timing": 1e3 * dt_prof / args.steps,
        "objective": stats["objective"], "primal_res": stats["primal_res"], "status": stats["status"],
    }
    if not args.no_mfma_leg and args.scale == 1.0:
        # the same workload with the wide products on the fp32 matrix cores
        solver.tune("gemm_split", 0)
        dt0, prof0, _ = timed_run(solver, args.steps, 1)
        solver.tune("gemm_split", 1)
        out["fp32_mfma_path"] = dict(gemm_split=0, value=args.steps / dt0, unit="iterations/s", ms_per_step=1e3 * dt0 / args.steps,
                                     kernels=[{k: e[k] for k in ("kernel", "bound", "achieved", "peak", "unit", "frac",
                                                                 "avg_launch_ms", "share_of_step")}
                                              for e in class_entries(prof0) if e["kernel"].startswith("gemm")])
    full_forms = None
    if not args.no_cpu_baseline and not args.no_full_size_oracle and args.scale == 1.0 and args.workload == 4:
        full_forms = full_size_oracle_forms(w, solver, solver.eval())
    solver.close()
    del solver
    torch.cuda.empty_cache()
    if not args.no_mfma_leg and args.scale == 1.0:
        out["mfma"] = mfma_leg(args.mfma_steps, 1)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, w.N, nnz, args.communities, args.schedule, args.step_policy)
        if full_forms is not None:
            out["cpu_baseline"]["full_size_full_graph_forms"] = full_forms
    print(json.dumps(out))


if __name__ == "__main__":
    main()
