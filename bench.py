#!/usr/bin/env python3
"""Benchmark of the tiled GEMM / MLP hot path on one MI355X.

Default workload (`--workload c2`): fp32 GEMM M=N=K=8000, tile T=1024 (ragged 832-wide edge tiles),
operands uniform[-1,1) from a seed, resident in HBM before the timed region -- one step = one
tgemm_run, i.e. one pass of the whole in-core path (plan, launch, every tile product).  Prints one
JSON line.  The other workloads (`c1`, `c3`, `c4`, `c5`, `bf16`) time the remaining benchmark
configurations with the same protocol and print the same kind of line.
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
PEAK_F32_MFMA_TFLOPS = 157.3    # MI355X dense fp32 matrix peak
PEAK_BF16_MFMA_TFLOPS = 2500.0  # MI355X dense bf16 matrix peak
HOST_LINK_GBS = 57.0            # measured hipMemcpy peak of the box, either direction
# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (summaries under
# profiles/); keyed by (workload, size, tile).  None where no counter run exists.
MEASURED_TRAFFIC_BYTES = {("c2", 8000, 1024): 1.920e9}


def cpu_baseline_gemm(A_host, B_host, budget_s=15.0):
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


def base_line(args, value, unit, ms_per_step, dtype, workload, extra_cfg=None):
    cfg = {"workload": workload}
    cfg.update(extra_cfg or {})
    return {"metric": METRIC, "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": dtype, "data": "synthetic", "config": cfg}


def run_gemm_incore(args, tg, inputs, torch, n, T, bf16):
    A = inputs.uniform_matrix(1, n, n, device="cuda")
    B = inputs.uniform_matrix(2, n, n, device="cuda")
    if bf16:
        A, B = A.to(torch.bfloat16), B.to(torch.bfloat16)
    C = torch.zeros(n, n, device="cuda")
    ctx = tg.tgemm_create(0, kernel_config=args.kernel_config)
    dt = tg.TGEMM_BF16 if bf16 else tg.TGEMM_F32
    flops = 2.0 * n * n * n
    torch.cuda.synchronize()      # inputs complete before the library's own streams read them
    for _ in range(args.warmup):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, dt)
    torch.cuda.synchronize()
    tg.tgemm_sync(ctx)
    kernel_ms = 0.0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, dt)          # synchronous: returns when C is complete
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
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_F32_MFMA_TFLOPS
    out = base_line(args, flops / (ms_per_step * 1e-3) / 1e12, "TFLOP/s", ms_per_step, "bf16" if bf16 else "f32",
                    "%s tiled GEMM M=N=K=%d, T=%d, in-core (A, B, C resident in HBM), C += A B"
                    % ("bf16-input fp32-accumulate" if bf16 else "fp32", n, T),
                    {"tile": T, "tasks": ((n + T - 1) // T) ** 2})
    out["roofline"] = {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                       "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, n, T)) if args.kernel_config == 0 else None,
                       "kernel": "tile_gemm_bf16" if bf16 else "tile_gemm_f32", "avg_kernel_ms": avg_kernel_ms,
                       "flops_per_launch": flops}
    if not args.no_cpu_baseline:
        Ah = A.float().cpu().numpy() if bf16 else A.cpu().numpy()
        Bh = B.float().cpu().numpy() if bf16 else B.cpu().numpy()
        out["cpu_baseline"] = cpu_baseline_gemm(Ah, Bh)
    return out


def run_gemm_ooc(args, tg, inputs, torch, n, T, budget):
    A = torch.empty(n, n, pin_memory=True)
    B = torch.empty(n, n, pin_memory=True)
    C = torch.zeros(n, n, pin_memory=True)
    inputs.fill(A, 1, "uniform", gen_device="cuda")
    inputs.fill(B, 2, "uniform", gen_device="cuda")
    torch.cuda.synchronize()
    ctx = tg.tgemm_create(0, order=args.order, strip_width=args.strip, rs_depth=args.rs_depth)
    flops = 2.0 * n * n * n
    for _ in range(args.warmup):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, budget)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, budget)
    wall = time.perf_counter() - t0
    st = tg.tgemm_last_stats(ctx)
    tg.tgemm_destroy(ctx)
    ms_per_step = wall * 1e3 / args.steps
    tfl = flops / (ms_per_step * 1e-3) / 1e12
    out = base_line(args, tfl, "TFLOP/s", ms_per_step, "f32",
                    "fp32 out-of-core tiled GEMM M=N=K=%d, T=%d, A, B, C in pinned host memory, HBM tile-cache budget %d bytes"
                    % (n, T, budget), {"tile": T, "slots": st["n_slots"], "order": ("serpentine", "row_major", "strips")[args.order], "rs_depth": args.rs_depth})
    link = (st["h2d_bytes"] / 1e9) / (ms_per_step * 1e-3)
    out["roofline"] = {"bound": "mfma", "achieved": tfl, "peak": PEAK_F32_MFMA_TFLOPS, "unit": "TFLOP/s",
                       "frac": tfl / PEAK_F32_MFMA_TFLOPS, "traffic": None, "kernel": "tile_gemm_f32 (whole run, transfers included)"}
    out["host_link"] = {"h2d_GBps": link, "d2h_GBps": (st["d2h_bytes"] / 1e9) / (ms_per_step * 1e-3),
                        "peak_GBps": HOST_LINK_GBS, "h2d_frac": link / HOST_LINK_GBS, "h2d_bytes": st["h2d_bytes"],
                        "d2h_bytes": st["d2h_bytes"], "hits": st["hits"], "misses": st["misses"]}
    return out


def run_mlp(args, tg, inputs, torch, dims, batch, T, bf16, budget):
    dt = torch.bfloat16 if bf16 else torch.float32
    X = inputs.normal_matrix(1, batch, dims[0], device="cuda").to(dt)
    y = inputs.labels(5, batch, dims[-1], device="cuda")
    W = []
    for l in range(len(dims) - 1):
        if budget:     # out-of-core: weights in pinned host memory
            w = torch.empty(dims[l], dims[l + 1], dtype=dt, pin_memory=True)
            inputs.fill(w, 10 + l, "normal", gen_device="cuda", std=0.01)
        else:
            w = inputs.normal_matrix(10 + l, dims[l], dims[l + 1], std=0.01, device="cuda").to(dt)
        W.append(w)
    torch.cuda.synchronize()
    # out-of-core: the write-back of a step's updated tiles may overlap the next step's forward pass;
    # tgemm_sync inside the timed region waits for the last of them
    ctx = tg.tgemm_create(0, kernel_config=args.kernel_config, deferred_writeback=0 if args.sync_writeback else 1)
    mlp = tg.mlp_create(ctx, dims, W, tg.TGEMM_BF16 if bf16 else tg.TGEMM_F32, T, hbm_budget=budget)
    if bf16 and args.stochastic_rounding:
        tg.mlp_set_rounding(mlp, tg.TGEMM_ROUND_STOCHASTIC, 1)
    if args.bias:
        bias = [torch.zeros(dims[l + 1], device="cuda") for l in range(len(dims) - 1)]
        tg.mlp_set_bias(mlp, bias)
    # velocities and master copies live where the weights live (out-of-core: pinned host memory)
    if args.momentum is not None:
        vel = [torch.zeros(dims[l], dims[l + 1], pin_memory=True) if budget else torch.zeros(dims[l], dims[l + 1], device="cuda")
               for l in range(len(dims) - 1)]
        tg.mlp_set_momentum(mlp, args.momentum, vel)
    if args.master_weights and bf16:
        master = []
        for w in W:
            if budget:
                mw = torch.empty(w.shape, dtype=torch.float32, pin_memory=True)
                mw.copy_(w)
            else:
                mw = w.float()
            master.append(mw)
        tg.mlp_set_master_weights(mlp, master)
    for _ in range(args.warmup):
        tg.mlp_step(mlp, X, y, batch, 0.01)
    tg.tgemm_sync(ctx)
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loss = tg.mlp_step(mlp, X, y, batch, 0.01)
    tg.tgemm_sync(ctx)
    wall = time.perf_counter() - t0
    st = tg.tgemm_last_stats(ctx)
    tg.mlp_destroy(mlp)
    tg.tgemm_destroy(ctx)
    ms_per_step = wall * 1e3 / args.steps
    flops = sum(2.0 * batch * dims[l] * dims[l + 1] * (3 if l > 0 else 2) for l in range(len(dims) - 1))
    tfl = flops / (ms_per_step * 1e-3) / 1e12
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_F32_MFMA_TFLOPS
    out = base_line(args, batch / (ms_per_step * 1e-3), "samples/s", ms_per_step, "bf16" if bf16 else "f32",
                    "MLP train step %s, layers %s, batch %d, sigmoid hidden, softmax + cross-entropy, SGD lr 0.01, T=%d%s"
                    % ("bf16 storage / fp32 accumulate" if bf16 else "fp32", "->".join(str(d) for d in dims), batch, T,
                       ", weights in pinned host memory, HBM budget %d bytes" % budget if budget else ", in-core"),
                    {"tile": T, "loss": loss, "rounding": "stochastic" if bf16 and args.stochastic_rounding else "nearest", "bias": bool(args.bias), "momentum": args.momentum,
                     "master_weights": bool(args.master_weights and bf16)})
    out["roofline"] = {"bound": "mfma", "achieved": tfl, "peak": peak, "unit": "TFLOP/s", "frac": tfl / peak,
                       "traffic": None, "kernel": "tile_gemm_%s (whole step)" % ("bf16" if bf16 else "f32"),
                       "flops_per_step": flops}
    if budget:
        out["host_link"] = {"h2d_GBps": st["h2d_bytes"] / 1e9 / (ms_per_step * 1e-3),
                            "d2h_GBps": st["d2h_bytes"] / 1e9 / (ms_per_step * 1e-3), "peak_GBps": HOST_LINK_GBS,
                            "h2d_bytes": st["h2d_bytes"], "d2h_bytes": st["d2h_bytes"], "slots": st["n_slots"],
                            "hits": st["hits"], "misses": st["misses"]}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5", "bf16"])
    ap.add_argument("--size", type=int, default=None, help="override the matrix size of a GEMM workload")
    ap.add_argument("--tile", type=int, default=None)
    ap.add_argument("--kernel-config", type=int, default=0)
    ap.add_argument("--order", type=int, default=2, choices=[0, 1, 2],
                    help="out-of-core task order: 0 serpentine, 1 row-major, 2 strips (default)")
    ap.add_argument("--strip", type=int, default=0, help="strip width for --order 2; 0 = from the slot count")
    ap.add_argument("--rs-depth", type=int, default=0,
                    help="out-of-core GEMM: reservation station of this many tasks, the one with the most cached tiles first (0: queue order)")
    ap.add_argument("--sync-writeback", action="store_true",
                    help="out-of-core MLP: every step waits for its weight write-back (default: deferred)")
    ap.add_argument("--stochastic-rounding", action="store_true",
                    help="c5: round the updated bf16 weights stochastically (mlp_set_rounding) instead of to nearest")
    ap.add_argument("--bias", action="store_true", help="c4 / c5: train bias rows too (mlp_set_bias)")
    ap.add_argument("--momentum", type=float, default=None, help="c4 / c5: SGD with this momentum coefficient (mlp_set_momentum)")
    ap.add_argument("--master-weights", action="store_true",
                    help="c4 --bf16 / c5: keep fp32 master copies of the bf16 weights (mlp_set_master_weights)")
    ap.add_argument("--bf16", action="store_true", help="c4: bf16 storage with fp32 accumulation instead of fp32 (extra data point)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run 5 plain device copies of 256 MiB (a known-size reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")
    defaults = {"c1": (200, 20), "c2": (50, 5), "c3": (3, 1), "c4": (10, 3), "c5": (10, 2), "bf16": (50, 5)}
    if args.steps is None:
        args.steps = defaults[args.workload][0]
    if args.warmup is None:
        args.warmup = defaults[args.workload][1]

    import torch
    from paper_1511_04348_amd import binding as tg
    from paper_1511_04348_amd import inputs

    torch.cuda.set_device(0)
    w = args.workload
    if w == "c1":
        out = run_gemm_incore(args, tg, inputs, torch, args.size or 1000, args.tile or 256, False)
    elif w == "c2":
        out = run_gemm_incore(args, tg, inputs, torch, args.size or 8000, args.tile or 1024, False)
    elif w == "bf16":
        out = run_gemm_incore(args, tg, inputs, torch, args.size or 8192, args.tile or 2048, True)
    elif w == "c3":
        out = run_gemm_ooc(args, tg, inputs, torch, args.size or 65536, args.tile or 4096, 8 * 10 ** 9)
    elif w == "c4":
        out = run_mlp(args, tg, inputs, torch, [4096, 16384, 16384, 16384, 10000], 4096, args.tile or 1024, args.bf16, 0)
    else:
        out = run_mlp(args, tg, inputs, torch, [8192, 32768, 32768, 262144], 8192, args.tile or 2048, True, 32 * 10 ** 9)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
