#!/usr/bin/env python3
"""Benchmark of the tiled GEMM hot path on one MI355X.

Default workload: fp32 GEMM M=N=K=8000, tile T=1024 (ragged 832-wide edge tiles), operands
uniform[-1,1) from a seed, resident in HBM before the timed region -- one step = one tgemm_run,
i.e. one pass of the whole in-core path (plan, launch, every tile product).  Prints one JSON line.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

METRIC = "tiled GEMM TFLOP/s (in-core, out-of-core) + MLP train samples/s, 1 GPU"
PEAK_F32_MFMA_TFLOPS = 157.3   # MI355X dense fp32 matrix peak
# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (summaries under
# profiles/); keyed by (size, tile).  None where no counter run exists.
MEASURED_TRAFFIC_BYTES = {(8000, 1024): 1.920e9}


def cpu_baseline_gemm(A_host, B_host, budget_s=12.0):
    """Times the oracle (as it stands) on a row slab of the same product, sized to ~budget_s."""
    import oracle
    K, N = B_host.shape
    rows = 64
    t0 = time.perf_counter()
    oracle.gemm(A_host[:rows], B_host)
    t = time.perf_counter() - t0
    rows = int(max(rows, min(A_host.shape[0], rows * budget_s / max(t, 1e-3))))
    t0 = time.perf_counter()
    oracle.gemm(A_host[:rows], B_host)
    t = time.perf_counter() - t0
    return {"value": 2.0 * rows * N * K / t / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(),
            "kind": "oracle", "sample": "first %d rows of C (of %d) at full N=%d, K=%d, %.1f s" % (rows, A_host.shape[0], N, K, t)}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--size", type=int, default=8000)
    ap.add_argument("--tile", type=int, default=1024)
    ap.add_argument("--kernel-config", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run 5 plain device copies of 256 MiB (a known-size reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    from paper_1511_04348_amd import binding as tg
    from paper_1511_04348_amd import inputs

    torch.cuda.set_device(0)
    n, T = args.size, args.tile
    A = inputs.uniform_matrix(1, n, n, device="cuda")
    B = inputs.uniform_matrix(2, n, n, device="cuda")
    C = torch.zeros(n, n, device="cuda")
    ctx = tg.tgemm_create(0, kernel_config=args.kernel_config)
    flops = 2.0 * n * n * n
    torch.cuda.synchronize()      # inputs complete before the library's own streams read them

    for _ in range(args.warmup):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T)
    torch.cuda.synchronize()
    tg.tgemm_sync(ctx)
    kernel_ms = 0.0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T)            # synchronous: returns when C is complete
        kernel_ms += tg.tgemm_last_stats(ctx)["kernel_ms"]  # HIP events on the launch stream
    tg.tgemm_sync(ctx)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    tg.tgemm_destroy(ctx)

    if args.copy_probe:
        src = torch.ones(64 * 1024 * 1024, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()

    ms_per_step = wall * 1e3 / args.steps
    avg_kernel_ms = kernel_ms / args.steps
    achieved = flops / (avg_kernel_ms * 1e-3) / 1e12
    out = {
        "metric": METRIC, "value": flops / (ms_per_step * 1e-3) / 1e12, "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "fp32 tiled GEMM M=N=K=%d, T=%d, in-core (A, B, C resident in HBM), C += A B" % (n, T),
                   "tile": T, "tasks": ((n + T - 1) // T) ** 2},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_F32_MFMA_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_F32_MFMA_TFLOPS,
                     "traffic": MEASURED_TRAFFIC_BYTES.get((n, T)) if args.kernel_config == 0 else None,
                     "kernel": "tile_gemm_f32", "avg_kernel_ms": avg_kernel_ms,
                     "flops_per_launch": flops},
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_gemm(A.cpu().numpy(), B.cpu().numpy())
    print(json.dumps(out))


if __name__ == "__main__":
    main()
