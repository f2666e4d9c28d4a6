#!/usr/bin/env python3
"""Benchmark of the tiled GEMM / MLP hot path on one MI355X.  Prints ONE JSON line.

Headline (`value`, `ms_per_step`, `roofline`, `cpu_baseline` at the top level): config 2, fp32 GEMM
M=N=K=8000, tile T=1024 (ragged 832-wide edge tiles), operands uniform[-1,1) from a seed, resident in
HBM before the timed region; one step = one tgemm_run, i.e. one pass of the whole in-core path (plan,
launch, every tile product).  `--steps` / `--warmup` apply to it.

Without `--workload` the same line also carries, under "configs", one sub-record per remaining
benchmark configuration (c1, c3, c4, c5, and the supplementary in-core bf16 product), each timed with
the same protocol (warm-up, then a timed loop bracketed by full synchronisation, inputs already
resident where the configuration says so) with its own `roofline`, `cpu_baseline` and, for the
out-of-core ones, `host_link` against the hipMemcpy peak probed in this run.  `--workload X` times
that one configuration alone and prints its record as the line (used for profiling).

cpu_baseline: the oracle (oracle/, as it stands) timed on the host cores on a bounded slab of the
same workload -- rows of C for the products, a batch-64 slab for the MLP steps -- and scaled
linearly in the row count (exact for independent rows); the `sample` field says what was run.
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
# HBM bytes per launch measured with rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE in separate counter runs
# (a counter run perturbs timing, so it cannot be this run); keyed by (workload, size, tile), with the
# summary under profiles/ that holds the figure.  None where no counter run exists.
MEASURED_TRAFFIC_BYTES = {("c2", 8000, 1024): (7.007e9, "profiles/tile_gemm_f32_incore_8000_T1024.md"),
                          ("c1", 1000, 256): (3.32e7, "profiles/tile_gemm_f32_incore_1000_T256.md"),
                          ("bf16", 8192, 2048): (2.148e9, "profiles/tile_gemm_bf16_incore_8192_T2048.md"),
                          # per training step, every kernel of the step summed
                          ("c4",): (6.88e10, "profiles/mlp_steps_config4_config5.md"),
                          ("c5",): (7.99e11, "profiles/mlp_steps_config4_config5.md")}
DEFAULT_STEPS = {"c1": (200, 20), "c2": (50, 5), "c3": (3, 1), "c4": (10, 3), "c5": (20, 2), "bf16": (50, 5)}
C4_DIMS, C4_BATCH = [4096, 16384, 16384, 16384, 10000], 4096
C5_DIMS, C5_BATCH = [8192, 32768, 32768, 262144], 8192


def note(*a):
    print("[bench]", *a, file=sys.stderr, flush=True)


def blas_threads():
    try:
        from threadpoolctl import threadpool_info
        n = [p.get("num_threads", 1) for p in threadpool_info() if p.get("user_api") == "blas"]
        return max(n) if n else (os.cpu_count() or 1)
    except Exception:
        return os.cpu_count() or 1


def probe_host_link(torch, nbytes=1 << 30, reps=3):
    """hipMemcpy peak of this machine, each direction: one pinned <-> device copy of `nbytes`, best of `reps`."""
    h = torch.empty(nbytes, dtype=torch.uint8, pin_memory=True)
    d = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    h.zero_()
    out = {}
    for name, dst, src in (("h2d_GBps", d, h), ("d2h_GBps", h, d)):
        dst.copy_(src, non_blocking=True)
        torch.cuda.synchronize()
        best = 0.0
        for _ in range(reps):
            t0 = time.perf_counter()
            dst.copy_(src, non_blocking=True)
            torch.cuda.synchronize()
            best = max(best, nbytes / (time.perf_counter() - t0) / 1e9)
        out[name] = best
    out["probe"] = "pinned <-> device copy of %d bytes, best of %d" % (nbytes, reps)
    del h, d
    return out


def cpu_baseline_gemm(A_rows, B_host, total_rows, budget_s):
    """The oracle on the first rows of the same product, sized to about budget_s seconds."""
    import oracle
    K, N = B_host.shape
    rows = min(64, A_rows.shape[0])
    t0 = time.perf_counter()
    oracle.gemm(A_rows[:rows], B_host)
    t = time.perf_counter() - t0
    more = int(min(A_rows.shape[0], rows * budget_s / max(t, 1e-3)))
    if more > rows:
        rows = more
        t0 = time.perf_counter()
        oracle.gemm(A_rows[:rows], B_host)
        t = time.perf_counter() - t0
    return {"value": 2.0 * rows * N * K / t / 1e12, "unit": "TFLOP/s", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "first %d rows of C (of %d) at full N=%d, K=%d, %.1f s%s"
                      % (rows, total_rows, N, K, t, "" if rows == total_rows else "; extrapolated from slab (rows are independent)")}


def cpu_baseline_mlp(torch, inputs, dims, batch, bf16, shrink):
    """oracle.mlp_step on a batch-64 slab.  shrink > 1: every width divided by it (the fp64 images the
    oracle forms of config 5's 9.9e9 weights, their gradients and the new weights would take 240 GB of
    host memory); the multiply-adds of every product, and with them the triple-loop cost, fall by
    shrink^2 exactly, and the reported rate is scaled back by that factor."""
    import numpy as np
    import oracle
    sdims = [d // shrink for d in dims]
    slab = 64
    X = inputs.normal_matrix(1, slab, sdims[0])
    y = inputs.labels(5, slab, sdims[-1]).numpy()
    Ws = []
    for l in range(len(sdims) - 1):
        w = inputs.normal_matrix(10 + l, sdims[l], sdims[l + 1], std=0.01, device="cuda")
        Ws.append(inputs.bf16_bits(w.to(torch.bfloat16)) if bf16 else w.cpu().numpy())
        del w
    Xn = inputs.bf16_bits(X.to(torch.bfloat16)) if bf16 else X.numpy()
    t0 = time.perf_counter()
    loss, _, _ = oracle.mlp_step(Xn, Ws, y, 0.01)
    t = time.perf_counter() - t0
    assert np.isfinite(loss)
    what = "oracle.mlp_step on a batch-%d slab (of %d)" % (slab, batch)
    if shrink > 1:
        what += " of the same network with every width divided by %d (%s), %.1f s; rate divided by %d (multiply-adds per sample)" \
                % (shrink, "->".join(str(d) for d in sdims), t, shrink * shrink)
    else:
        what += " at full widths, %.1f s" % t
    return {"value": slab / t / (shrink * shrink), "unit": "samples/s", "cores": blas_threads(), "kind": "oracle",
            "sample": what + "; extrapolated from slab (samples are independent; numpy fp64 matmul is the oracle's product)"}


def record(steps, warmup, value, unit, ms_per_step, dtype, workload, extra_cfg=None):
    cfg = {"workload": workload}
    cfg.update(extra_cfg or {})
    return {"metric": METRIC, "value": value, "unit": unit, "n_gpus": 1, "steps": steps, "warmup": warmup,
            "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": dtype, "data": "synthetic", "config": cfg}


def run_gemm_incore(args, env, name, steps, warmup, n, T, bf16):
    tg, inputs, torch = env["tg"], env["inputs"], env["torch"]
    A = inputs.uniform_matrix(1, n, n, device="cuda")
    B = inputs.uniform_matrix(2, n, n, device="cuda")
    if bf16:
        A, B = A.to(torch.bfloat16), B.to(torch.bfloat16)
    C = torch.zeros(n, n, device="cuda")
    ctx = tg.tgemm_create(0, kernel_config=args.kernel_config, incore_schedule=args.incore_schedule)
    dt = tg.TGEMM_BF16 if bf16 else tg.TGEMM_F32
    flops = 2.0 * n * n * n
    torch.cuda.synchronize()      # inputs complete before the library's own streams read them
    for _ in range(warmup):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, dt)
    torch.cuda.synchronize()
    tg.tgemm_sync(ctx)
    t0 = time.perf_counter()
    for _ in range(steps):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, dt)          # synchronous: returns when C is complete
    tg.tgemm_sync(ctx)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    # The kernel time of the same call from the library's HIP events on its launch stream, over `steps`
    # further calls: reading the statistics back after every call costs a 1000^3 product a tenth of its
    # wall time, so it stays out of the loop above.
    kernel_ms = 0.0
    for _ in range(steps):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, dt)
        kernel_ms += tg.tgemm_last_stats(ctx)["kernel_ms"]
    launches = tg.tgemm_last_stats(ctx)["kernel_launches"]
    tg.tgemm_destroy(ctx)
    pipelined = None
    if name == "c1":
        # the same calls enqueued back to back (tgemm_opts.async_incore), one synchronisation at the end: what
        # a caller that does not wait for every product sees; every call still accumulates into the same C
        actx = tg.tgemm_create(0, kernel_config=args.kernel_config, incore_schedule=args.incore_schedule, async_incore=1)
        for _ in range(warmup):
            tg.tgemm_run(actx, A, B, C, n, n, n, T, dt)
        tg.tgemm_sync(actx)
        t1 = time.perf_counter()
        for _ in range(steps):
            tg.tgemm_run(actx, A, B, C, n, n, n, T, dt)
        tg.tgemm_sync(actx)
        awall = time.perf_counter() - t1
        tg.tgemm_destroy(actx)
        pipelined = {"ms_per_step": awall * 1e3 / steps, "value": flops / (awall / steps) / 1e12, "unit": "TFLOP/s",
                     "what": "%d asynchronous calls (tgemm_opts.async_incore), one tgemm_sync at the end" % steps}
    if args.copy_probe:
        src = torch.ones(64 * 1024 * 1024, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
    ms_per_step = wall * 1e3 / steps
    avg_kernel_ms = kernel_ms / steps
    achieved = flops / (avg_kernel_ms * 1e-3) / 1e12
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_F32_MFMA_TFLOPS
    out = record(steps, warmup, flops / (ms_per_step * 1e-3) / 1e12, "TFLOP/s", ms_per_step, "bf16" if bf16 else "f32",
                 "%s tiled GEMM M=N=K=%d, T=%d, in-core (A, B, C resident in HBM), C += A B"
                 % ("bf16-input fp32-accumulate" if bf16 else "fp32", n, T),
                 {"tile": T, "tasks": ((n + T - 1) // T) ** 2})
    traffic = MEASURED_TRAFFIC_BYTES.get((name, n, T)) if args.kernel_config == 0 and args.incore_schedule == 0 else None
    kernel = "tile_gemm_bf16" if bf16 else "tile_gemm_f32"
    if launches > 1:     # the balanced schedule: whole rounds, k segments of the partial round, strips, fix-up
        kernel += " (balanced schedule: the %d launches of a step, first to last on the launch stream)" % launches
    out["roofline"] = {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                       "traffic": traffic[0] if traffic else None, "traffic_source": traffic[1] if traffic else None,
                       "kernel": kernel, "avg_kernel_ms": avg_kernel_ms, "launches_per_step": launches,
                       "flops_per_launch": flops}
    if pipelined:
        out["pipelined"] = pipelined
    if not args.no_cpu_baseline:
        Ah = A.float().cpu().numpy() if bf16 else A.cpu().numpy()
        Bh = B.float().cpu().numpy() if bf16 else B.cpu().numpy()
        out["cpu_baseline"] = cpu_baseline_gemm(Ah, Bh, n, args.cpu_seconds)
    return out


def run_gemm_ooc(args, env, name, steps, warmup, n, T, budget):
    tg, inputs, torch = env["tg"], env["inputs"], env["torch"]
    A = torch.empty(n, n, pin_memory=True)
    B = torch.empty(n, n, pin_memory=True)
    C = torch.zeros(n, n, pin_memory=True)
    inputs.fill(A, 1, "uniform", gen_device="cuda")
    inputs.fill(B, 2, "uniform", gen_device="cuda")
    torch.cuda.synchronize()
    note(name, "inputs in pinned host memory")
    ctx = tg.tgemm_create(0, order=args.order, strip_width=args.strip, rs_depth=args.rs_depth)
    flops = 2.0 * n * n * n
    for _ in range(warmup):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, budget)
    t0 = time.perf_counter()
    for _ in range(steps):
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, budget)     # synchronous: C is complete in host memory
    wall = time.perf_counter() - t0
    st = tg.tgemm_last_stats(ctx)
    tg.tgemm_destroy(ctx)
    ms_per_step = wall * 1e3 / steps
    tfl = flops / (ms_per_step * 1e-3) / 1e12
    out = record(steps, warmup, tfl, "TFLOP/s", ms_per_step, "f32",
                 "fp32 out-of-core tiled GEMM M=N=K=%d, T=%d, A, B, C in pinned host memory, HBM tile-cache budget %d bytes"
                 % (n, T, budget), {"tile": T, "slots": st["n_slots"], "order": ("serpentine", "row_major", "strips")[args.order],
                                   "rs_depth": args.rs_depth})
    link = env["link"]
    h2d = (st["h2d_bytes"] / 1e9) / (ms_per_step * 1e-3)
    d2h = (st["d2h_bytes"] / 1e9) / (ms_per_step * 1e-3)
    # 4096 tile products on two compute streams, overlapping the transfers: the rate of the whole run
    # (every transfer included) is what is reported, a lower bound of the kernel's own
    out["roofline"] = {"bound": "mfma", "achieved": tfl, "peak": PEAK_F32_MFMA_TFLOPS, "unit": "TFLOP/s",
                       "frac": tfl / PEAK_F32_MFMA_TFLOPS, "traffic": None,
                       "kernel": "tile_gemm_f32 (whole run, transfers included; MFMA-bound under the strips order)",
                       "flops_per_run": flops}
    out["host_link"] = {"h2d_GBps": h2d, "d2h_GBps": d2h, "peak_h2d_GBps": link["h2d_GBps"], "peak_d2h_GBps": link["d2h_GBps"],
                        "peak_probe": link["probe"], "h2d_frac": h2d / link["h2d_GBps"], "d2h_frac": d2h / link["d2h_GBps"],
                        "h2d_bytes": st["h2d_bytes"], "d2h_bytes": st["d2h_bytes"], "hits": st["hits"], "misses": st["misses"]}
    if not args.no_cpu_baseline:
        note(name, "oracle slab")
        out["cpu_baseline"] = cpu_baseline_gemm(A[:64].numpy(), B.numpy(), n, 0.0)
    return out


def run_mlp(args, env, name, steps, warmup, dims, batch, T, bf16, budget):
    tg, inputs, torch = env["tg"], env["inputs"], env["torch"]
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
    note(name, "inputs ready")
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
    for _ in range(warmup):
        tg.mlp_step(mlp, X, y, batch, 0.01)
    tg.tgemm_sync(ctx)
    kernel_ms = 0.0
    t0 = time.perf_counter()
    per_step = []
    for _ in range(steps):
        loss = tg.mlp_step(mlp, X, y, batch, 0.01)
        s1 = tg.tgemm_last_stats(ctx)
        kernel_ms += s1["kernel_ms"]   # first to last launch of the step, HIP events on the compute stream
        per_step.append((round(s1["wall_ms"], 1), round(s1["kernel_ms"], 1)))
    tg.tgemm_sync(ctx)
    wall = time.perf_counter() - t0
    st = tg.tgemm_last_stats(ctx)
    note(name, "per step (host wall ms, compute stream ms):", per_step)
    tg.mlp_destroy(mlp)
    tg.tgemm_destroy(ctx)
    ms_per_step = wall * 1e3 / steps
    avg_kernel_ms = kernel_ms / steps
    flops = sum(2.0 * batch * dims[l] * dims[l + 1] * (3 if l > 0 else 2) for l in range(len(dims) - 1))
    achieved = flops / (avg_kernel_ms * 1e-3) / 1e12
    peak = PEAK_BF16_MFMA_TFLOPS if bf16 else PEAK_F32_MFMA_TFLOPS
    out = record(steps, warmup, batch / (ms_per_step * 1e-3), "samples/s", ms_per_step, "bf16" if bf16 else "f32",
                 "MLP train step %s, layers %s, batch %d, sigmoid hidden, softmax + cross-entropy, SGD lr 0.01, T=%d%s"
                 % ("bf16 storage / fp32 accumulate" if bf16 else "fp32", "->".join(str(d) for d in dims), batch, T,
                    ", weights in pinned host memory, HBM budget %d bytes" % budget if budget else ", in-core"),
                 {"tile": T, "loss": loss, "rounding": "stochastic" if bf16 and args.stochastic_rounding else "nearest",
                  "bias": bool(args.bias), "momentum": args.momentum, "master_weights": bool(args.master_weights and bf16),
                  "step_TFLOPs": flops / (ms_per_step * 1e-3) / 1e12})
    plain = not (args.bias or args.momentum is not None or args.master_weights or args.stochastic_rounding or args.sync_writeback
                 or args.kernel_config or (name == "c4" and bf16))
    traffic = MEASURED_TRAFFIC_BYTES.get((name,)) if plain else None
    out["roofline"] = {"bound": "mfma", "achieved": achieved, "peak": peak, "unit": "TFLOP/s", "frac": achieved / peak,
                       "traffic": traffic[0] if traffic else None, "traffic_source": traffic[1] if traffic else None,
                       "kernel": "tile_gemm_%s (all %d launches of a step, first to last on the compute stream; "
                       "the softmax launch included)" % ("bf16" if bf16 else "f32", st["kernel_launches"]),
                       "avg_kernel_ms": avg_kernel_ms, "flops_per_step": flops}
    if budget:
        link = env["link"]
        h2d = st["h2d_bytes"] / 1e9 / (ms_per_step * 1e-3)
        d2h = st["d2h_bytes"] / 1e9 / (ms_per_step * 1e-3)
        out["host_link"] = {"h2d_GBps": h2d, "d2h_GBps": d2h, "peak_h2d_GBps": link["h2d_GBps"], "peak_d2h_GBps": link["d2h_GBps"],
                            "peak_probe": link["probe"], "h2d_frac": h2d / link["h2d_GBps"], "d2h_frac": d2h / link["d2h_GBps"],
                            "h2d_bytes": st["h2d_bytes"], "d2h_bytes": st["d2h_bytes"], "slots": st["n_slots"],
                            "hits": st["hits"], "misses": st["misses"]}
    del W, X, y
    if not args.no_cpu_baseline:
        note(name, "oracle slab")
        out["cpu_baseline"] = cpu_baseline_mlp(torch, inputs, dims, batch, bf16, 4 if budget else 1)
    return out


def run_one(args, env, name, steps, warmup):
    if name == "c1":
        return run_gemm_incore(args, env, name, steps, warmup, args.size or 1000, args.tile or 256, False)
    if name == "c2":
        return run_gemm_incore(args, env, name, steps, warmup, args.size or 8000, args.tile or 1024, False)
    if name == "bf16":
        return run_gemm_incore(args, env, name, steps, warmup, args.size or 8192, args.tile or 2048, True)
    if name == "c3":
        return run_gemm_ooc(args, env, name, steps, warmup, args.size or 65536, args.tile or 4096, 8 * 10 ** 9)
    if name == "c4":
        return run_mlp(args, env, name, steps, warmup, C4_DIMS, C4_BATCH, args.tile or 1024, args.bf16, 0)
    return run_mlp(args, env, name, steps, warmup, C5_DIMS, C5_BATCH, args.tile or 2048, True, 32 * 10 ** 9)


def release(torch):
    import gc
    gc.collect()
    torch.cuda.empty_cache()
    if hasattr(torch._C, "_host_emptyCache"):
        torch._C._host_emptyCache()      # pinned host blocks back to the system (config 3 needs 52 GB of them)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default=None, choices=["c1", "c2", "c3", "c4", "c5", "bf16"],
                    help="time this configuration alone (default: config 2 as the headline plus every other one under \"configs\")")
    ap.add_argument("--size", type=int, default=None, help="override the matrix size of a GEMM workload (with --workload)")
    ap.add_argument("--tile", type=int, default=None)
    ap.add_argument("--kernel-config", type=int, default=0)
    ap.add_argument("--incore-schedule", type=int, default=0, choices=[0, 1, 2],
                    help="fp32 in-core products: 0 automatic, 1 always one launch, 2 balanced wherever it applies (tgemm_opts.incore_schedule)")
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
    ap.add_argument("--cpu-seconds", type=float, default=12.0, help="size of the oracle's slab for the in-core products, in seconds")
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run 5 plain device copies of 256 MiB (a known-size reference for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import torch
    from paper_1511_04348_amd import binding as tg
    from paper_1511_04348_amd import inputs

    torch.cuda.set_device(0)
    env = {"tg": tg, "inputs": inputs, "torch": torch, "link": None}

    def steps_for(name, headline):
        s, w = DEFAULT_STEPS[name]
        if headline:
            s = args.steps if args.steps is not None else s
            w = args.warmup if args.warmup is not None else w
        return s, w

    if args.workload is not None:
        if args.workload in ("c3", "c5"):
            env["link"] = probe_host_link(torch)
        out = run_one(args, env, args.workload, *steps_for(args.workload, True))
        print(json.dumps(out))
        return

    t_start = time.perf_counter()
    note("config 2 (headline)")
    out = run_one(args, env, "c2", *steps_for("c2", True))
    release(torch)
    env["link"] = probe_host_link(torch)
    note("host link", env["link"])
    configs = {}
    for name in ("c1", "bf16", "c4", "c5", "c3"):
        note("config", name, "at %.0f s" % (time.perf_counter() - t_start))
        try:
            sub = run_one(args, env, name, *steps_for(name, False))
            for k in ("metric", "n_gpus", "higher_is_better", "scaling", "vs_baseline", "data"):
                sub.pop(k, None)
            configs[name] = sub
        except Exception as e:      # the headline still gets printed
            configs[name] = {"error": "%s: %s" % (type(e).__name__, e)}
            note("config", name, "failed:", configs[name]["error"])
        release(torch)
    out["configs"] = configs
    out["host_link_probe"] = env["link"]
    out["bench_wall_s"] = time.perf_counter() - t_start
    print(json.dumps(out))


if __name__ == "__main__":
    main()
