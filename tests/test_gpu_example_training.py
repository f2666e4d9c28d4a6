"""End to end: the example trainer (bias rows, momentum, tanh, mini-batches through mlp_step) must
actually learn -- the loss falls from about ln 16 to a small value and held-out accuracy is high -- in
fp32, with bf16 weights rounded stochastically, and with bf16 weights that follow fp32 master copies;
the out-of-core GEMM example must be right under every task order and show the cache's effect."""
import math
import os
import sys

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, os.path.join(ROOT, "examples"))

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("bf16,master", [(False, False), (True, False), (True, True)])
def test_example_trainer_learns(bf16, master):
    import train_mlp
    print("[case] example trainer", "bf16" if bf16 else "f32", "master copies" if master else "", flush=True)
    losses, acc = train_mlp.run(bf16=bf16, epochs=5, quiet=True, master_weights=master)
    assert losses[0] < math.log(16) + 0.5
    assert all(b <= a + 1e-3 for a, b in zip(losses, losses[1:])), losses
    assert losses[-1] < 0.1 * losses[0], losses
    assert acc > 0.97, acc


def test_example_out_of_core_gemm():
    import ooc_gemm
    print("[case] example out-of-core GEMM", flush=True)
    res = {name: (st, err) for name, st, err in ooc_gemm.run(n=4096, tile=512, budget_mb=48, quiet=True)}
    for name, (st, err) in res.items():
        assert err < 1e-5, (name, err)
        assert st["in_core"] == 0 and st["n_tasks"] == 64 and st["n_tile_gemms"] == 512
        assert st["d2h_bytes"] == 4096 * 4096 * 4                       # every C tile harvested once
        assert st["hits"] + st["misses"] == 2 * 512                     # one A and one B lookup per tile product
    # the strip order reuses what the cache holds; row-major order re-fetches B for every task row
    assert res["strips"][0]["misses"] < res["serpentine"][0]["misses"] <= res["row-major"][0]["misses"]
    assert res["row-major + station"][0]["misses"] < res["row-major"][0]["misses"]


def test_example_size_sweep():
    import size_sweep
    print("[case] example size sweep", flush=True)
    res = size_sweep.run([2048, 4608, 4096], "f32", 512, reps=3, quiet=True)
    by_n = {n: (launches, rate, rate_one, plan) for n, launches, rate, rate_one, plan in res}
    assert by_n[2048][0] == 1 and by_n[4096][0] == 1            # too small to gain; whole rounds only
    launches, rate, rate_one, plan = by_n[4608]                 # 324 macro tiles: one whole round and 68 tiles cut up
    assert launches == 3 and plan["applies"] == 1 and plan["whole_round_tiles"] == 256 and plan["tail_tiles"] == 68
    assert rate > rate_one                                      # measured: 137 against 127 TFLOP/s
