#!/usr/bin/env python3
"""Benchmark of the ADMM sweep on one MI355X.

A "step" is one full ADMM iteration (W-update, Z-update for every layer and community, last-layer
solve, dual step) on a synthetic SBM workload already resident in HBM.  Prints ONE JSON line:
ADMM iterations/s for the whole job, the roofline of the dominant kernel class measured live with
HIP events on the library's stream, and the CPU oracle timed on a bounded sample of the same recipe.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..5] [--scale S]
"""
import argparse
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

# Bytes per launch group that crossed the L2 -> fabric boundary (FETCH_SIZE + WRITE_SIZE, each scaled by what a plain
# copy of known size reads), measured with rocprofv3 --pmc on this program at the default workload (steady-state
# sweeps); the summary with the commands is profiles/sweep_memory_traffic_powerlaw_dcsbm_2M.txt.
MEASURED_TRAFFIC = {
    (4, "gemm_nn_split_kernel<2>+finish"): 5.15e9 + 2.05e9,   # H_1 gradW_1, first candidate, step on T_1 ahead of the decision
    (4, "spmm_rows_kernel[rows]"): 2.927e9 + 0.131e9,         # width 16
    (4, "spmm_rows_kernel[segments]"): 1.684e9 + 0.184e9 + 0.601e9 + 0.510e9,   # width 16: several entries + single entry
    (4, "gemm_tn_split_kernel+reduce"): 5.16e9 + 0.038e9 + 0.067e9,
    (4, "z_trial_kernel"): 6.126e9 + 0.006e9,
    (4, "z_step_kernel"): 4.297e9 + 2.048e9,
    (4, "gemm_nn_gradz_kernel"): 4.226e9 + 0.128e9,
    (4, "t_carry_kernel"): 1.280e9 + 0.114e9,
    (4, "gemm_nn_kernel<32>"): 2.049e9 + 0.128e9,             # out[N x 16] = A[N x 256] B
    (4, "gemm_tn_kernel<32>+reduce"): 2.188e9 + 0.008e9,
    (4, "last_layer_kernel"): 0.392e9 + 0.256e9,
    (4, "gemm_nn_split_kernel<0>"): 1.114e9 + 2.048e9,        # out[N x 256] = A[N x 128] B
}

# CPU-oracle sample: (scale of N, iterations) per workload, sized for about 10-30 s of host time
ORACLE_SAMPLE = {1: (1.0, 10), 2: (0.25, 4), 3: (0.02, 3), 4: (0.004, 8), 5: (0.004, 2), 6: (0.1, 3), 7: (0.2, 3)}


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
                    launches=p["records"], share_of_step=None, fp32_product_TFLOPs=p["flops"] / sec / 1e12)
    if name.startswith("gemm") and p["bytes"] > 0 and p["flops"] / p["bytes"] > MACHINE_BALANCE:
        ach = p["flops"] / sec / 1e12
        return dict(kernel=name, bound="mfma", achieved=ach, peak=MFMA_FP32_PEAK_TFLOPS, unit="TFLOP/s",
                    frac=ach / MFMA_FP32_PEAK_TFLOPS, traffic=None, avg_launch_ms=per_launch_ms,
                    launches=p["records"], share_of_step=None)
    ach = p["bytes"] / sec / 1e9
    return dict(kernel=name, bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS,
                traffic=None, avg_launch_ms=per_launch_ms, launches=p["records"], share_of_step=None)


def cpu_baseline(index, full_N, full_nnz, communities=None, schedule=0, step_policy=0):
    """The oracle as it stands, on a smaller instance of the same recipe, extrapolated linearly in nnz."""
    from threadpoolctl import threadpool_info
    from oracle.admm import make_oracle
    from paper_2112_09335_amd import synth
    scale, iters = ORACLE_SAMPLE[index]
    w = synth.config(index, scale, communities)
    w.hyper["schedule"] = schedule
    w.hyper["step_policy"] = step_policy
    orc = make_oracle(w)
    orc.iterate(1)                       # first iteration is atypical (zero gradients at the forward-pass start)
    t0 = time.perf_counter()
    orc.iterate(iters)
    dt = time.perf_counter() - t0
    its = iters / dt
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    est_full = its * (orc.g.nnz / float(full_nnz))
    return dict(value=est_full, unit="iterations/s", cores=int(threads), kind="oracle",
                sample=(f"{w.name} recipe at N={w.N} (scale {scale}), M={w.M}, nnz={orc.g.nnz}: {iters} oracle "
                        f"iterations in {dt:.1f} s = {its:.3f} it/s on the sample; value = that rate x "
                        f"nnz_sample/nnz_full (linear extrapolation to N={full_N})"),
                sample_iterations_per_s=its)


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
    ap.add_argument("--partition", choices=["planted", "builtin"], default="planted",
                    help="communities: the generator's planted blocks, or the library's own partitioner")
    ap.add_argument("--scale", type=float, default=1.0, help="shrink N (debugging only)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
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

    solver.run(args.warmup)
    torch.cuda.synchronize()
    # timed region 1: the plain run, nothing but the sweep on the stream
    t0 = time.perf_counter()
    solver.run(args.steps)
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    # timed region 2: the same number of steps with every launch group bracketed by HIP events
    solver.profile(True)
    t0 = time.perf_counter()
    solver.run(args.steps)
    prof = solver.get_profile()          # synchronises
    dt_prof = time.perf_counter() - t0
    solver.profile(False)
    stats = solver.eval()

    total_ms = sum(p["ms"] for p in prof.values())
    entries = []
    for name, p in prof.items():
        e = roofline_entry(name, p)
        if e is not None:
            e["share_of_step"] = p["ms"] / total_ms if total_ms > 0 else None
            entries.append(e)
    if args.scale == 1.0:
        for e in entries:
            e["traffic"] = MEASURED_TRAFFIC.get((args.workload, e["kernel"]))
    entries.sort(key=lambda e: -e["share_of_step"])
    dominant = dict(entries[0]) if entries else None
    spmm_keys = [k for k in prof if k.startswith("spmm")]
    spmm_ms = sum(prof[k]["ms"] for k in spmm_keys)
    spmm_bytes = sum(prof[k]["bytes"] for k in spmm_keys)
    spmm_flops = sum(prof[k]["flops"] for k in spmm_keys)

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
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": f"configs[{args.workload - 1}] {w.name}", "N": w.N, "communities": w.M,
                   "edges": w.E, "nnz": nnz, "layers": w.L, "widths": w.dims, "scale": args.scale,
                   "schedule": args.schedule, "step_policy": args.step_policy, "partition": args.partition},
        "roofline": None if dominant is None else {k: dominant[k] for k in
                                                   ("bound", "achieved", "peak", "unit", "frac", "traffic")},
        "dominant_kernel": None if dominant is None else dominant["kernel"],
        "kernels": entries,
        # all aggregation launches of the timed steps together.  achieved_GBs uses the algorithmic minimum (every
        # row of the gathered matrix read once); gather_volume_GBs counts what the kernel actually requests from
        # the memory system, nnz gathers of 4*width bytes (2 flops per gathered float) plus the entries
        "spmm": {"achieved_GBs": spmm_bytes / (spmm_ms * 1e-3) / 1e9 if spmm_ms > 0 else None,
                 "frac_of_hbm_peak": spmm_bytes / (spmm_ms * 1e-3) / 1e9 / HBM_PEAK_GBS if spmm_ms > 0 else None,
                 "edges_features_per_s": 0.5 * spmm_flops / (spmm_ms * 1e-3) if spmm_ms > 0 else None,
                 "gather_volume_GBs": (2.0 * spmm_flops + 8.0 * nnz * sum(prof[k]["records"] for k in spmm_keys))
                 / (spmm_ms * 1e-3) / 1e9 if spmm_ms > 0 else None},
        "ms_per_step_with_event_timing": 1e3 * dt_prof / args.steps,
        "objective": stats["objective"], "primal_res": stats["primal_res"], "status": stats["status"],
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(args.workload, w.N, nnz, args.communities, args.schedule, args.step_policy)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
