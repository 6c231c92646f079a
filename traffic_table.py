#!/usr/bin/env python3
"""Memory traffic per kernel class of the ADMM sweep, from two rocprofv3 counter runs of bench.py.

    rocprofv3 --pmc FETCH_SIZE --kernel-trace --output-format csv -d DIR -o pmc_FETCH_SIZE -- python3 bench.py --steps 4 --warmup 1 --no-cpu-baseline --no-mfma-leg
    rocprofv3 --pmc WRITE_SIZE --kernel-trace --output-format csv -d DIR -o pmc_WRITE_SIZE -- python3 bench.py --steps 4 --warmup 1 --no-cpu-baseline --no-mfma-leg
    python traffic_table.py --dir DIR --workload "configs[3] powerlaw_dcsbm" --out profiles/sweep_memory_traffic_powerlaw_dcsbm_2M

Writes OUT.txt (one row per kernel symbol and grid) and OUT.json (bytes per launch group of bench.py's kernel classes,
the commit and a hash of the kernel sources they were measured at), which bench.py reports as `traffic`.
The counters are KiB per dispatch between the L2 and the fabric.  Each is scaled by what the same counter reads for the
library's plain copy of 1 GiB, which the same bench.py run launches (cadmm_op_calibrate kind 0, stream_copy_kernel).
A row is the mean over the typical dispatches of that kernel and grid: those within a factor of two of its median duration.
"""
import argparse
import collections
import csv
import json
import os
import re
import subprocess
import time

ROOT = os.path.dirname(os.path.abspath(__file__))

# bench.py class -> kernel symbols (regular expressions on the demangled name) whose steady-state dispatches make up one
# launch group of the class.  "rows" / "segments" select the aggregation launches by how often their grid occurs.
CLASSES = {
    "spmm_rows_kernel[rows]": [("spmm_rows_kernel", "rows"), ("spmm_combine_kernel", "rows")],
    "spmm_rows_kernel[segments]": [("spmm_rows_kernel", "segments"), ("spmm_combine_kernel", "segments"), ("spmm_single_kernel", None)],
    "gemm_nn_split_kernel<2>+finish": [(r"gemm_nn_split_kernel<2>", None)],
    "gemm_nn_split_kernel<0>": [(r"gemm_nn_split_kernel<0>", None)],
    "gemm_tn_split_kernel+reduce": [(r"gemm_tn_split_kernel", None)],
    "gemm_nn_kernel<32>": [(r"gemm_nn_kernel<32, 0>", None)],
    "gemm_tn_kernel<32>+reduce": [(r"gemm_tn_kernel<32", None)],
    "gemm_nn_gradz_kernel": [(r"gemm_nn_gradz_kernel", None)],
    "z_trial_kernel": [(r"z_trial_kernel<1,", None)],
    "z_step_kernel": [(r"z_step(_lowrank)?_kernel", None)],
    "t_carry_kernel": [(r"t_carry_kernel", None)],
    "last_layer_kernel": [(r"last_layer_kernel", None)],
    "phi_G_kernel": [(r"phi_G_kernel<1,", None)],
    "G_only_kernel": [(r"G_only_kernel", None)],
    "w_trial_kernel": [(r"w_trial_kernel<1, 1,", None)],
    "w_step_kernel": [(r"w_step_kernel", None)],
}


def short(name):
    return name.replace("cadmm::(anonymous namespace)::", "").replace("void ", "").split("(")[0]


def load(path):
    d = collections.defaultdict(list)
    for r in csv.DictReader(open(path)):
        d[(short(r["Kernel_Name"]), int(r["Grid_Size"]))].append(
            (float(r["Counter_Value"]), (int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3))
    return d


def steady(v):
    """Mean counter value, mean duration and count of the typical dispatches: those within a factor of two of the median
    duration (the first iterations and the periodic exact re-evaluations run longer forms of some kernels)."""
    med = sorted(x[1] for x in v)[len(v) // 2]
    sel = [x for x in v if 0.5 * med <= x[1] <= 2.0 * med] or v
    return sum(x[0] for x in sel) / len(sel), sum(x[1] for x in sel) / len(sel), len(sel)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dir", required=True)
    ap.add_argument("--workload", required=True)
    ap.add_argument("--out", required=True)
    ap.add_argument("--command", default="")
    args = ap.parse_args()
    f = load(os.path.join(args.dir, "pmc_FETCH_SIZE_counter_collection.csv"))
    w = load(os.path.join(args.dir, "pmc_WRITE_SIZE_counter_collection.csv"))
    copy = [k for k in f if k[0] == "stream_copy_kernel"]
    if not copy:
        raise SystemExit("no stream_copy_kernel dispatch in the counter run: cannot calibrate")
    gib = float(1 << 30)
    fetch_scale = gib / (steady(f[copy[0]])[0] * 1024.0)
    write_scale = gib / (steady(w[copy[0]])[0] * 1024.0)
    rows = {}
    for k in f:
        fv, us, n = steady(f[k])
        wv = steady(w[k])[0] if k in w else 0.0
        rows[k] = dict(fetch=fetch_scale * fv * 1024.0, write=write_scale * wv * 1024.0, us=us, n=n, total_us=us * n)
    # the aggregation over the rows runs several times per iteration, the one over the segments once: of the two most
    # frequent grids of the narrow aggregation kernel the one with more dispatches is the rows
    agg = sorted((k for k in rows if k[0].startswith("spmm_rows_kernel") and rows[k]["n"] >= 3), key=lambda k: -rows[k]["n"])
    role = {}
    if len(agg) >= 2:
        role[agg[0]] = "rows"
        role[agg[1]] = "segments"
    comb = sorted((k for k in rows if k[0].startswith("spmm_combine_kernel") and rows[k]["n"] >= 3), key=lambda k: -rows[k]["n"])
    if len(comb) >= 2:
        role[comb[0]] = "rows"
        role[comb[1]] = "segments"
    classes = {}
    for cls, members in CLASSES.items():
        tot = 0.0
        found = False
        for pat, sel in members:
            ks = [k for k in rows if re.match(pat, k[0]) and (sel is None or role.get(k) == sel)]
            if not ks:
                continue
            k = max(ks, key=lambda q: rows[q]["total_us"])
            tot += rows[k]["fetch"] + rows[k]["write"]
            found = True
        if found:
            classes[cls] = tot
    try:
        commit = subprocess.run(["git", "rev-parse", "--short", "HEAD"], cwd=ROOT, capture_output=True, text=True).stdout.strip()
    except OSError:
        commit = ""
    import bench
    meta = dict(workload=args.workload, commit=commit, date=time.strftime("%Y-%m-%d"),
                kernel_source_hash=bench.kernel_source_hash(), fetch_scale=fetch_scale, write_scale=write_scale,
                unit="bytes per launch group (FETCH_SIZE + WRITE_SIZE, scaled)", classes=classes)
    with open(args.out + ".json", "w") as fo:
        json.dump(meta, fo, indent=1)
    with open(args.out + ".txt", "w") as fo:
        fo.write(f"HBM-side traffic of every kernel inside the ADMM sweep, workload {args.workload}, MI355X\n")
        fo.write("commands (two runs, one counter each; then this table):\n")
        for ctr in ("FETCH_SIZE", "WRITE_SIZE"):
            fo.write(f"  rocprofv3 --pmc {ctr} --kernel-trace --output-format csv -d {args.dir} -o pmc_{ctr} -- "
                     f"python3 bench.py --steps 4 --warmup 1 --no-cpu-baseline --no-mfma-leg\n")
        fo.write(f"  python3 traffic_table.py --dir {args.dir} --workload \"{args.workload}\" --out {args.out}\n")
        fo.write(f"measured at commit {commit} (kernel sources {meta['kernel_source_hash']}), {meta['date']}\n")
        fo.write("Counter values are KiB per dispatch between the L2 and the fabric; a row is the mean over the dispatches of that\n"
                 "kernel and grid within a factor of two of its median duration.  GB = 1e9 bytes.  Calibration: the library's\n"
                 f"plain copy of 1 GiB in the same run shows 1/{fetch_scale:.3f} of its size in FETCH_SIZE and 1/{write_scale:.3f} in WRITE_SIZE,\n"
                 "so the counters are multiplied by these factors.\n\n")
        fo.write(f"{'kernel':46s} {'grid':>11s} {'n':>4s} {'fetch GB':>9s} {'write GB':>9s} {'avg us':>9s}\n")
        for k in sorted(rows, key=lambda q: -rows[q]["total_us"]):
            r = rows[k]
            fo.write(f"{k[0][:46]:46s} {k[1]:11d} {r['n']:4d} {r['fetch'] / 1e9:9.3f} {r['write'] / 1e9:9.3f} {r['us']:9.1f}\n")
        fo.write("\nper bench.py kernel class (fetch + write per launch group, GB):\n")
        for cls, v in classes.items():
            fo.write(f"  {cls:34s} {v / 1e9:8.3f}\n")
    print(open(args.out + ".txt").read())


if __name__ == "__main__":
    main()
