#!/usr/bin/env python3
"""Time single kernels of the library on a synthetic workload (for profiling under rocprofv3).

    python kernel_bench.py --workload 4 --ops copy aggregate:256 segments:16 \
           transform:256:256 wgrad:128:256 --reps 5

ops:  copy            a plain device copy of 1 GiB (torch), the calibration point for memory counters
      stream          the library's own copy kernel on 1 GiB (cadmm_op_calibrate): what a streaming kernel can reach
      update          dst = 0.999 dst + src in place (the memory mix of the step kernels)
      mfma            register-only chains of fp32 MFMAs (cadmm_op_calibrate): what the matrix cores can reach
      mfma_bf16       the same with bf16 MFMAs; mfma_bf16_valu4 / 6 / 8: with that many vector instructions after each
      gather:W        only the gathers of the row aggregation at width W, no row structure (cadmm_op_calibrate):
                      what the memory system serves to the graph's column stream; gatherseg:W the same for the segments
      aggregate:W     Y = A~ X, X of width W                    (cadmm_op_aggregate)
      segments:W      per-(row, community) aggregation          (cadmm_op_aggregate_segments)
      transform:K:C   out[N x C] = A[N x K] B[K x C]            (cadmm_op_transform)
      wgrad:K:C       out[K x C] = A[N x K]^T G[N x C]          (cadmm_op_wgrad)
Prints one line per op: mean milliseconds, algorithmic bytes and flops, and the resulting rates.
"""
import argparse
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", type=int, default=4)
    ap.add_argument("--scale", type=float, default=1.0)
    ap.add_argument("--ops", nargs="+", default=["copy", "aggregate:256"])
    ap.add_argument("--reps", type=int, default=5)
    ap.add_argument("--tune", nargs="*", default=[], help="key=value tuning knobs")
    args = ap.parse_args()

    import torch
    from paper_2112_09335_amd import binding, synth

    w = synth.config(args.workload, args.scale)
    s = binding.Solver.from_workload(w, 0)
    for kv in args.tune:
        k, v = kv.split("=")
        s.tune(k, int(v))
    nnz, nseg, _ = s.graph_sizes()
    N = w.N
    print(f"# {w.name}: N={N} nnz={nnz} segments={nseg}", flush=True)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / args.reps

    for op in args.ops:
        parts = op.split(":")
        kind = parts[0]
        if kind in ("gather", "gatherseg"):
            W = int(parts[1])
            rate = s.op_calibrate("gather" if kind == "gather" else "gather_segments", W, args.reps)
            print(f"{op:20s} gathers of {4 * W}-byte rows along the real column stream: {rate:8.1f} GB/s requested "
                  f"(pairs + rows) = {rate / (8.0 + 4.0 * W):7.2f} G gathers/s", flush=True)
            continue
        if kind.startswith("mfma_bf16"):
            rate = s.op_calibrate(kind, 20000, args.reps)
            print(f"{op:20s} bf16 MFMA chains on registers"
                  + (f" with {kind[-1]} vector instructions after each" if kind != "mfma_bf16" else "")
                  + f": {rate:7.1f} TFLOP/s ({rate / 2500.0:.3f} of the published 2500)", flush=True)
            continue
        if kind == "update":
            rate = s.op_calibrate("update", 1 << 28, args.reps)
            print(f"{op:20s} library in-place update kernel, 2 GiB read + 1 GiB written back: {rate:8.1f} GB/s", flush=True)
            continue
        if kind in ("stream", "mfma"):
            if kind == "stream":
                rate = s.op_calibrate("copy", 1 << 28, args.reps)
                print(f"{op:20s} library copy kernel, 1 GiB read + 1 GiB written: {rate:8.1f} GB/s", flush=True)
            else:
                rate = s.op_calibrate("mfma", 20000, args.reps)
                print(f"{op:20s} fp32 MFMA chains on registers: {rate:7.2f} TFLOP/s "
                      f"({rate / 157.3:.3f} of the published 157.3)", flush=True)
            continue
        if kind == "copy":
            n = 1 << 28                                           # 1 GiB of fp32
            src = torch.randn(n, device="cuda")
            dst = torch.empty_like(src)
            ms = timed(lambda: dst.copy_(src))
            byt, flop = 8.0 * n, 0.0
        elif kind == "aggregate":
            W = int(parts[1])
            X = torch.randn(N, W, device="cuda")
            ms = timed(lambda: s.op_aggregate(X))
            byt = 8.0 * nnz + 16.0 * N + 8.0 * N * W
            flop = 2.0 * nnz * W
        elif kind == "segments":
            W = int(parts[1])
            X = torch.randn(N, W, device="cuda")
            ms = timed(lambda: s.op_aggregate_segments(X))
            byt = 8.0 * nnz + 16.0 * nseg + 4.0 * N * W + 4.0 * nseg * W
            flop = 2.0 * nnz * W
        elif kind == "transform":
            K, C = int(parts[1]), int(parts[2])
            A = torch.randn(N, K, device="cuda")
            B = torch.randn(K, C, device="cuda")
            ms = timed(lambda: s.op_transform(A, B))
            byt = 4.0 * (N * K + K * C + N * C)
            flop = 2.0 * N * K * C
        elif kind == "wgrad":
            K, C = int(parts[1]), int(parts[2])
            A = torch.randn(N, K, device="cuda")
            G = torch.randn(N, C, device="cuda")
            ms = timed(lambda: s.op_wgrad(A, G))
            byt = 4.0 * (N * K + N * C + K * C)
            flop = 2.0 * N * K * C
        else:
            raise SystemExit(f"unknown op {op}")
        print(f"{op:20s} {ms:9.3f} ms   algorithmic {byt / 1e9:8.3f} GB -> {byt / ms / 1e6:8.1f} GB/s   "
              f"{flop / 1e9:9.2f} GFLOP -> {flop / ms / 1e9:7.2f} TFLOP/s", flush=True)


if __name__ == "__main__":
    main()
