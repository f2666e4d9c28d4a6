"""Throughput of the in-core product C += A B against the matrix size (the analogue of the paper's
section 4.1 sweep of square single-precision products), through the C ABI's tgemm_run:

    python examples/size_sweep.py [--dtype f32|bf16] [--tile 512] [--sizes 2048,3072,...] [--reps 6]

Per size: the schedule the library chose (one launch, or the balanced schedule's launches: whole rounds
of macro tiles, k segments of the partial round, fix-up, strips) with its kernel time and rate, the same
product forced into one launch, and what tgemm_balance_plan says about the product."""
import argparse
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_1511_04348_amd import binding as tg  # noqa: E402


def time_product(ctx, A, B, C, n, tile, dtype, reps):
    ms = []
    for _ in range(reps + 2):
        tg.tgemm_run(ctx, A, B, C, n, n, n, tile, dtype, 0)
        ms.append(tg.tgemm_last_stats(ctx)["kernel_ms"])
    ms = ms[2:]
    return sum(ms) / len(ms), tg.tgemm_last_stats(ctx)["kernel_launches"]


def run(sizes, dtype="f32", tile=512, reps=6, quiet=False):
    code = tg.TGEMM_BF16 if dtype == "bf16" else tg.TGEMM_F32
    auto = tg.tgemm_create(0)
    one = tg.tgemm_create(0, incore_schedule=tg.TGEMM_SCHEDULE_ONE_LAUNCH)
    gen = torch.Generator(device="cuda").manual_seed(0)
    out = []
    try:
        for n in sizes:
            A = torch.empty(n, n, device="cuda").uniform_(-1, 1, generator=gen)
            B = torch.empty(n, n, device="cuda").uniform_(-1, 1, generator=gen)
            if dtype == "bf16":
                A, B = A.to(torch.bfloat16), B.to(torch.bfloat16)
            C = torch.zeros(n, n, device="cuda")
            torch.cuda.synchronize()
            t_auto, launches = time_product(auto, A, B, C, n, tile, code, reps)
            t_one, _ = time_product(one, A, B, C, n, tile, code, reps)
            plan, _ = tg.tgemm_balance_plan(n, n, n, tile, code)
            flops = 2.0 * n ** 3
            out.append((n, launches, flops / t_auto / 1e9, flops / t_one / 1e9, plan))
            if not quiet:
                what = ("%d whole-round tiles + %d tiles in %d segments" % (plan["whole_round_tiles"], plan["tail_tiles"], plan["n_segments"])
                        if plan["applies"] else "one launch")
                print("n %6d  %d launch%s %8.3f ms %7.1f TFLOP/s | as one launch %8.3f ms %7.1f TFLOP/s | %s"
                      % (n, launches, " " if launches == 1 else "es", t_auto, flops / t_auto / 1e9, t_one, flops / t_one / 1e9, what), flush=True)
            del A, B, C
    finally:
        tg.tgemm_destroy(auto)
        tg.tgemm_destroy(one)
    return out


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="f32", choices=["f32", "bf16"])
    ap.add_argument("--tile", type=int, default=512)
    ap.add_argument("--reps", type=int, default=6)
    ap.add_argument("--sizes", default="1024,2048,3072,4096,5120,6144,7168,8000,8192,9216,10240")
    a = ap.parse_args()
    run([int(s) for s in a.sizes.split(",")], a.dtype, a.tile, a.reps)
