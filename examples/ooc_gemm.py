"""An out-of-core product C += A B through the C ABI's tgemm_run (ctypes binding): the matrices stay in
pinned host memory, tiles pass through a bounded HBM tile cache, and the run's statistics show what
the cache did under each task order, and with the reservation station's locality priority.

    python examples/ooc_gemm.py [--n 16384] [--tile 2048] [--budget-mb 768]

Prints, per task order, the wall time, the rate, the tile-cache hits / misses and the host-link bytes,
and checks 64 sampled entries of C against a float64 dot product computed by torch on the CPU."""
import argparse
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_1511_04348_amd import binding as tg  # noqa: E402

# (name, task order, depth of the reservation station: > 1 lets the task with the most cached tiles go first)
ORDERS = [("strips", tg.TGEMM_ORDER_STRIPS, 0), ("serpentine", tg.TGEMM_ORDER_SERPENTINE, 0), ("row-major", tg.TGEMM_ORDER_ROW_MAJOR, 0),
          ("row-major + station", tg.TGEMM_ORDER_ROW_MAJOR, 16)]


def run(n=16384, tile=2048, budget_mb=768, quiet=False):
    gen = torch.Generator().manual_seed(0)
    A = torch.empty(n, n, pin_memory=True).uniform_(-1, 1, generator=gen)
    B = torch.empty(n, n, pin_memory=True).uniform_(-1, 1, generator=gen)
    rows = torch.randint(0, n, (64,), generator=gen)
    cols = torch.randint(0, n, (64,), generator=gen)
    want = (A[rows].double() * B[:, cols].double().t()).sum(dim=1)
    results = []
    for name, order, depth in ORDERS:
        C = torch.zeros(n, n, pin_memory=True)
        ctx = tg.tgemm_create(0, order=order, rs_depth=depth)
        tg.tgemm_run(ctx, A, B, C, n, n, n, tile, tg.TGEMM_F32, budget_mb << 20)
        st = tg.tgemm_last_stats(ctx)
        tg.tgemm_destroy(ctx)
        err = float((C[rows, cols].double() - want).abs().max() / want.abs().max())
        results.append((name, st, err))
        if not quiet:
            print("%-19s %7.1f ms  %6.1f TFLOP/s  slots %3d  hits %5d  misses %5d  H2D %6.2f GB  D2H %5.2f GB  max rel. error %.1e"
                  % (name, st["wall_ms"], 2.0 * n ** 3 / st["wall_ms"] / 1e9, st["n_slots"], st["hits"], st["misses"],
                     st["h2d_bytes"] / 1e9, st["d2h_bytes"] / 1e9, err))
    return results


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--n", type=int, default=16384)
    ap.add_argument("--tile", type=int, default=2048)
    ap.add_argument("--budget-mb", type=int, default=768)
    a = ap.parse_args()
    run(a.n, a.tile, a.budget_mb)
