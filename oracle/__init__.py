"""CPU oracle -- TEST INFRASTRUCTURE ONLY.

Plain, slow, obviously-correct definitions of everything the GPU library
computes: the GEMM (section 3.1 of the paper: tile products accumulated over
k), the tile plan (section 3.1, Algorithm 1 "decode"), the L1 tile cache
behaviour under LRU (section 3.4, Algorithm 1 lookups) and the MLP passes
(section 2, equations 1, 3, 4), with the optional stochastic rounding of
updated bf16 weights and fp32 master copies.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It never imports the GPU package and
shares no code or table with it (the random bits of the stochastic rounding
are an interface written out in the library's header, which each side
implements on its own).

Parity pins: every function here is pinned by ``tests/test_oracle_*.py``
against closed forms, brute force, numpy's fp64 matmul, finite differences
and the tile counts the paper prints; nothing is "parity unpinned".
"""
from .build import build_oracle, lib_path  # noqa: F401
from .gemm import gemm, gemm_tiled, gemm_samples, num_threads, bf16_to_f64  # noqa: F401
from .plan import plan_tiles, tile_counts, decode_task, kstep_ranges  # noqa: F401
from .lru import Invalidate, lru_simulate, tgemm_access_sequence, task_order, auto_strip, station_simulate, next_use_simulate, mlp_sweep_groups  # noqa: F401
from .mlp import mlp_forward, mlp_backward, mlp_step, mlp_step_stochastic, mlp_step_momentum, mlp_step_master, mlp_loss, mlp_rows  # noqa: F401
from .rounding import mix32, step_key, rounding_bits, stochastic_round_bf16, stochastic_round_matrix, round_bf16_nearest  # noqa: F401
