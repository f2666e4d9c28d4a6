"""The pins must be able to fail: every planted mistake in a copy of the oracle's source (a
dropped term, a wrong sign, a wrong index or axis, a transposed operand) has to be caught by at
least one pin test, and the untouched source has to pass all of them.

Each mutant is built on the CPU from the oracle's own source text with one substitution; the
oracle package on disk and the GPU library are never touched.  The pin tests are the functions
of the test_oracle_* modules, called directly with a stand-in for the `oracle` fixture."""
import os
import subprocess
import types

import pytest

import test_oracle_gemm as pins_gemm
import test_oracle_mlp as pins_mlp
import test_oracle_plan_lru as pins_plan
import test_oracle_rounding as pins_round

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _mutated_module(oracle, fname, old, new, extra_globals=None):
    """oracle/<fname> with the single occurrence of `old` replaced by `new`, as a module object."""
    src = open(os.path.join(ROOT, "oracle", fname)).read()
    assert src.count(old) == 1, "mutation target must occur exactly once: %r" % old
    src = src.replace(old, new)
    mod = types.ModuleType("oracle._mutant_" + fname[:-3])
    mod.__package__ = "oracle"
    mod.__file__ = os.path.join(ROOT, "oracle", fname)
    if extra_globals:
        mod.__dict__.update(extra_globals)
    exec(compile(src, mod.__file__ + "<mutant>", "exec"), mod.__dict__)
    return mod


def _stand_in(oracle, mod):
    """A namespace like the oracle package in which the mutant's public functions win."""
    ns = types.SimpleNamespace(**{k: v for k, v in vars(oracle).items() if not k.startswith("__")})
    for k, v in vars(mod).items():
        if callable(v) and not k.startswith("_") and hasattr(oracle, k):
            setattr(ns, k, v)
    return ns


def _killed_by(ns, pins):
    """Names of the pin tests that fail on the stand-in."""
    killers = []
    for fn, args in pins:
        try:
            fn(ns, *args)
        except Exception as e:                    # an assertion, or a crash from a broken shape
            killers.append("%s: %s" % (fn.__name__, type(e).__name__))
    return killers


MLP_PINS = [(pins_mlp.test_finite_differences_every_weight, ()), (pins_mlp.test_zero_weights_closed_form, ()),
            (pins_mlp.test_single_layer_is_softmax_regression, ()), (pins_mlp.test_invariants_and_orientation, ()),
            (pins_mlp.test_step_descends_first_order, ()), (pins_mlp.test_bf16_inputs_widen_exactly, ()),
            (pins_mlp.test_finite_differences_tanh_and_relu, ()), (pins_mlp.test_activation_values_written_out, ()),
            (pins_mlp.test_activation_symmetries, ()), (pins_mlp.test_step_descends_for_every_activation, ()),
            (pins_mlp.test_bias_finite_differences, ()), (pins_mlp.test_bias_is_a_constant_one_input_column, ()),
            (pins_mlp.test_bias_closed_forms, ()), (pins_mlp.test_bias_step, ()),
            (pins_mlp.test_momentum_reduces_to_sgd_and_heavy_ball_identity, ()), (pins_mlp.test_momentum_with_bias_rows, ()),
            (pins_round.test_master_step_written_out, ()), (pins_round.test_master_copies_keep_the_steps_that_bf16_storage_loses, ()),
            (pins_mlp.test_rows_equal_the_whole_batch_pass, ()), (pins_mlp.test_rows_closed_forms_and_input_gradient, ())]

MLP_MUTANTS = [
    ("sigmoid sign", "        return 1.0 / (1.0 + np.exp(-z))", "        return 1.0 / (1.0 + np.exp(z))"),
    ("tanh of 2z", "        return np.tanh(z)", "        return np.tanh(2.0 * z)"),
    ("tanh replaced by the sigmoid", "        return np.tanh(z)", "        return 1.0 / (1.0 + np.exp(-z))"),
    ("relu replaced by abs", "        return np.where(z > 0.0, z, 0.0)", "        return np.abs(z)"),
    ("relu passes negatives scaled", "        return np.where(z > 0.0, z, 0.0)", "        return np.where(z > 0.0, z, 0.1 * z)"),
    ("softmax axis", "probs = e / e.sum(axis=1, keepdims=True)", "probs = e / e.sum(axis=0, keepdims=True)"),
    ("loss sum instead of mean", "return float(np.mean(lse - z[np.arange(z.shape[0]), y]))",
     "return float(np.sum(lse - z[np.arange(z.shape[0]), y]))"),
    ("one-hot sign", "d[np.arange(B), y] -= 1.0", "d[np.arange(B), y] += 1.0"),
    ("dropped 1/batch", "    d /= B\n", "    d = d\n"),
    ("sigmoid slope: dropped (1 - a) factor", "        return a * (1.0 - a)", "        return a"),
    ("sigmoid slope: dropped a factor", "        return a * (1.0 - a)", "        return 1.0 - a"),
    ("tanh slope: a instead of a squared", "        return 1.0 - a * a", "        return 1.0 - a"),
    ("relu slope: always on", "        return (z > 0.0).astype(np.float64)", "        return np.ones_like(z)"),
    ("relu slope: sign flipped", "        return (z > 0.0).astype(np.float64)", "        return (z < 0.0).astype(np.float64)"),
    ("slope dropped from the error", "d = dA * _act_slope(pre[l], acts[l], act)", "d = dA"),
    ("slope of the wrong layer", "d = dA * _act_slope(pre[l], acts[l], act)", "d = dA * _act_slope(pre[l], acts[l], 'sigmoid')"),
    ("dW from the wrong activation", "dWs[l] = acts[l].T @ d", "dWs[l] = acts[max(l - 1, 0)].T @ d"),
    ("delta not propagated", "dA = d @ _f64(Ws[l]).T", "dA = d @ np.abs(_f64(Ws[l])).T"),
    ("update sign", "new = [_f64(W) - lr * g for W, g in zip(Ws, dWs)]", "new = [_f64(W) + lr * g for W, g in zip(Ws, dWs)]"),
    ("update without lr", "new = [_f64(W) - lr * g for W, g in zip(Ws, dWs)]", "new = [_f64(W) - g for W, g in zip(Ws, dWs)]"),
    ("loss ignores the activation", "    _, z, _ = mlp_forward(X, Ws, act, bs=bs)", "    _, z, _ = mlp_forward(X, Ws, bs=bs)"),
    ("loss ignores the bias rows", "    _, z, _ = mlp_forward(X, Ws, act, bs=bs)", "    _, z, _ = mlp_forward(X, Ws, act)"),
    ("bias added along the batch", "            z = z + np.asarray(bs[l], dtype=np.float64)[None, :]",
     "            z = z + np.asarray(bs[l], dtype=np.float64)[None, :].mean()"),
    ("bias subtracted", "            z = z + np.asarray(bs[l], dtype=np.float64)[None, :]",
     "            z = z - np.asarray(bs[l], dtype=np.float64)[None, :]"),
    ("bias of the wrong layer", "            z = z + np.asarray(bs[l], dtype=np.float64)[None, :]",
     "            z = z + np.asarray(bs[l if l == 0 or bs[l - 1].shape != bs[l].shape else l - 1], dtype=np.float64)[None, :]"),
    ("backward pass forgets the bias in its forward", "    acts, z, probs, pre = mlp_forward(X, Ws, act, return_pre=True, bs=bs)",
     "    acts, z, probs, pre = mlp_forward(X, Ws, act, return_pre=True)"),
    ("db summed over the wrong axis", "[dl.sum(axis=0) for dl in deltas]", "[dl.sum(axis=1) for dl in deltas]"),
    ("db averaged instead of summed", "[dl.sum(axis=0) for dl in deltas]", "[dl.mean(axis=0) for dl in deltas]"),
    ("bias update sign", "new_bs = [np.asarray(b, dtype=np.float64) - lr * g for b, g in zip(bs, dbs)]",
     "new_bs = [np.asarray(b, dtype=np.float64) + lr * g for b, g in zip(bs, dbs)]"),
    ("momentum: mu on the gradient instead of the velocity", "new_V = [mu * np.asarray(V, dtype=np.float64) + g for V, g in zip(Vs, dWs)]",
     "new_V = [np.asarray(V, dtype=np.float64) + mu * g for V, g in zip(Vs, dWs)]"),
    ("momentum: gradient subtracted", "new_V = [mu * np.asarray(V, dtype=np.float64) + g for V, g in zip(Vs, dWs)]",
     "new_V = [mu * np.asarray(V, dtype=np.float64) - g for V, g in zip(Vs, dWs)]"),
    ("momentum: weights move by the gradient, not the velocity", "new_W = [_f64(W) - lr * V for W, V in zip(Ws, new_V)]",
     "new_W = [_f64(W) - lr * V for W, V in zip(Ws, dWs)]"),
    ("momentum: weights move by the old velocity", "new_W = [_f64(W) - lr * V for W, V in zip(Ws, new_V)]",
     "new_W = [_f64(W) - lr * np.asarray(V) for W, V in zip(Ws, Vs)]"),
    ("momentum: lr applied twice over", "new_W = [_f64(W) - lr * V for W, V in zip(Ws, new_V)]",
     "new_W = [_f64(W) - lr * lr * V for W, V in zip(Ws, new_V)]"),
    ("momentum: bias velocity ignores mu", "new_Vb = [mu * np.asarray(v, dtype=np.float64) + g for v, g in zip(Vbs, dbs)]",
     "new_Vb = [np.asarray(v, dtype=np.float64) + g for v, g in zip(Vbs, dbs)]"),
    ("momentum: bias rows move by the gradient", "new_b = [np.asarray(b, dtype=np.float64) - lr * v for b, v in zip(bs, new_Vb)]",
     "new_b = [np.asarray(b, dtype=np.float64) - lr * v for b, v in zip(bs, dbs)]"),
    ("master copies: gradient taken at the master copies", "    loss, dWs, _ = mlp_backward(X, Ws, y, act)\n    vel = None",
     "    loss, dWs, _ = mlp_backward(X, [np.asarray(M, dtype=np.float64) for M in masters], y, act)\n    vel = None"),
    ("master copies: step applied to the bf16 weights", "exact = [np.asarray(M, dtype=np.float32).astype(np.float64) - lr * d for M, d in zip(masters, moves)]",
     "exact = [_f64(M) - lr * d for M, d in zip(Ws, moves)]"),
    ("master copies: step added", "exact = [np.asarray(M, dtype=np.float32).astype(np.float64) - lr * d for M, d in zip(masters, moves)]",
     "exact = [np.asarray(M, dtype=np.float32).astype(np.float64) + lr * d for M, d in zip(masters, moves)]"),
    ("master copies: kept in fp64", "    new_M = [e.astype(np.float32) for e in exact]", "    new_M = [e for e in exact]"),
    ("master copies: bf16 weights not refreshed", "    bits = [round_bf16_nearest(m) for m in new_M]", "    bits = [np.asarray(w) for w in Ws]"),
    ("master copies: bf16 weights truncated", "    bits = [round_bf16_nearest(m) for m in new_M]",
     "    bits = [(m.view(np.uint32) >> 16).astype(np.uint16) for m in new_M]"),
    ("master copies: momentum step moves by the gradient", "    moves = dWs if Vs is None else vel", "    moves = dWs"),
    ("master copies: velocity ignores mu", "[g + mu * np.asarray(V, dtype=np.float64) for g, V in zip(dWs, Vs)]",
     "[g + np.asarray(V, dtype=np.float64) for g, V in zip(dWs, Vs)]"),
    ("bias update without lr", "new_bs = [np.asarray(b, dtype=np.float64) - lr * g for b, g in zip(bs, dbs)]",
     "new_bs = [np.asarray(b, dtype=np.float64) - g for b, g in zip(bs, dbs)]"),
    ("rows: block product drops the transposition", "            out[:, o0:o1] = R @ _f64(W[o0:o1, :]).T\n", "            out[:, o0:o1] = R @ _f64(W[:, o0:o1])\n"),
    ("rows: blocks land one block late", "            out[:, o0:o1] = R @ _f64(np.ascontiguousarray(W[:, o0:o1]))",
     "            out[:, o0:o1] = R @ _f64(np.ascontiguousarray(W[:, max(0, o0 - (o1 - o0)):max(0, o0 - (o1 - o0)) + o1 - o0]))"),
    ("rows: last block dropped", "    starts = range(0, n_out, block)\n", "    starts = range(0, n_out - block + 1, block)\n"),
    ("rows: softmax without the row sum", "    probs = e / e.sum(axis=1)[:, None]", "    probs = e / e.sum()"),
    ("rows: one-hot sign", "    d[r, y] -= 1.0", "    d[r, y] += 1.0"),
    ("rows: divided by the number of rows given", "    d /= batch\n", "    d /= z.shape[0]\n"),
    ("rows: loss without the label's logit", "    loss_rows = zmax[:, 0] + np.log(e.sum(axis=1)) - z[r, y]", "    loss_rows = zmax[:, 0] + np.log(e.sum(axis=1))"),
    ("rows: slope dropped", "            d = _rows_times(d, Ws[l], transpose=True, block=block, workers=workers) * _act_slope(pre[l], acts[l], act)",
     "            d = _rows_times(d, Ws[l], transpose=True, block=block, workers=workers)"),
    ("rows: error through the wrong layer's weights", "            d = _rows_times(d, Ws[l], transpose=True, block=block, workers=workers) * _act_slope(pre[l], acts[l], act)",
     "            d = _rows_times(d, Ws[l], transpose=True, block=block, workers=workers) * _act_slope(pre[l - 1] if l > 1 else pre[l], acts[l - 1] if l > 1 else acts[l], act)"),
]


@pytest.mark.parametrize("name,old,new", MLP_MUTANTS, ids=[m[0] for m in MLP_MUTANTS])
def test_mlp_mutant_is_caught(oracle, name, old, new):
    mod = _mutated_module(oracle, "mlp.py", old, new)
    killers = _killed_by(_stand_in(oracle, mod), MLP_PINS)
    print(name, "->", killers)
    assert killers, "no pin notices: " + name


PLAN_LRU_PINS = ([(pins_plan.test_paper_tile_counts, ()), (pins_plan.test_edge_extents_config1, ()),
                  (pins_plan.test_lru_closed_forms, ()), (pins_plan.test_lru_vs_brute_force, ()), (pins_plan.test_lru_invalidate, ()),
                  (pins_plan.test_access_sequence_structure, ()), (pins_plan.test_row_major_reuse_closed_form, ()),
                  (pins_plan.test_strips_order_written_out, ()), (pins_plan.test_strips_traffic_closed_form, ()),
                  (pins_plan.test_station_of_depth_one_is_queue_order, ()), (pins_plan.test_station_worked_example, ()),
                  (pins_plan.test_station_leaves_by_priority, ()),
                  (pins_plan.test_next_use_is_optimal_on_every_small_sweep, ()), (pins_plan.test_next_use_worked_example_and_closed_forms, ()),
                  (pins_plan.test_next_use_against_explicit_scan_with_groups, ()), (pins_plan.test_mlp_sweep_written_out, ())]
                 + [(pins_plan.test_plan_partitions_output, a) for a in [(1000, 1000, 1000, 256), (7, 13, 5, 3), (5, 5, 5, 8)]])

LRU_MUTANTS = [
    ("hit does not refresh (FIFO)", "            cache.move_to_end(key)\n", "            pass\n"),
    ("station: ties go to the later entry", "            if score > best_score:", "            if score >= best_score:"),
    ("station: the least cached task leaves", "        best, best_score = 0, -1\n", "        best, best_score = 0, 10 ** 9\n"),
    ("station: only A tiles count", 'score = sum((("A", ti, k) in lru) + (("B", k, tj) in lru) for k in range(n_k))',
     'score = sum((("A", ti, k) in lru) for k in range(n_k))'),
    ("station: B tile index transposed in the score", 'score = sum((("A", ti, k) in lru) + (("B", k, tj) in lru) for k in range(n_k))',
     'score = sum((("A", ti, k) in lru) + (("B", tj, k) in lru) for k in range(n_k))'),
    ("station: depth ignored", "        while queue and len(station) < depth:", "        while queue and len(station) < 1:"),
    ("station: one task too many", "        while queue and len(station) < depth:", "        while queue and len(station) < depth + 1:"),
    ("station: B looked up before A", '            events.append(lru.lookup(("A", ti, k)))\n            events.append(lru.lookup(("B", k, tj)))',
     '            events.append(lru.lookup(("B", k, tj)))\n            events.append(lru.lookup(("A", ti, k)))'),
    ("station: the score refreshes the tiles it finds", "    def __contains__(self, key):\n        return key in self.cache",
     "    def __contains__(self, key):\n        if key in self.cache:\n            self.cache.move_to_end(key)\n        return key in self.cache"),
    ("evicts the most recent", "victim, _ = cache.popitem(last=False)", "victim, _ = cache.popitem(last=True)"),
    ("one slot too many", "if len(cache) >= n_slots:", "if len(cache) > n_slots:"),
    ("serpentine parity", 'if order == "serpentine" and i % 2 == 1:', 'if order == "serpentine" and i % 2 == 0:'),
    ("strips parity", "rows = range(n_i) if s % 2 == 0 else range(n_i - 1, -1, -1)",
     "rows = range(n_i) if s % 2 == 1 else range(n_i - 1, -1, -1)"),
    ("strips never turn round", "rows = range(n_i) if s % 2 == 0 else range(n_i - 1, -1, -1)", "rows = range(n_i)"),
    ("B tile index transposed", 'seq.append(("B", k, j, tid, k))', 'seq.append(("B", j, k, tid, k))'),
    ("B looked up before A", 'seq.append(("A", i, k, tid, k))\n            seq.append(("B", k, j, tid, k))',
     'seq.append(("B", k, j, tid, k))\n            seq.append(("A", i, k, tid, k))'),
    ("task id decoded column-major", "i, j = tid // n_j, tid % n_j", "i, j = tid % n_i, tid // n_i"),
    ("automatic strip one too wide", "widest = min(max(1, n_j), max(1, n_slots // n_k - 2))", "widest = min(max(1, n_j), max(1, n_slots // n_k - 1))"),
    ("automatic strip: widest, not evened out", "return max(1, -(-n_j // n_strips)) if n_strips > 0 else 1", "return widest"),
    ("automatic strip: one strip too many", "n_strips = -(-n_j // widest)", "n_strips = -(-n_j // widest) + 1"),
    ("invalidate: drops the other matrices", "        for key in [k for k in self.cache if k[0] == name]:", "        for key in [k for k in self.cache if k[0] != name]:"),
    ("invalidate: drops everything", "        for key in [k for k in self.cache if k[0] == name]:", "        for key in list(self.cache):"),
    ("invalidate: ignored", "            lru.drop(key.name)\n", "            pass\n"),
    ("invalidate: counted as a lookup", "            lru.drop(key.name)\n", "            lru.drop(key.name)\n            events.append((False, None))\n"),
    ("next use: the nearest leaves", "                    if ahead > best:", "                    if ahead < best or best < 0:"),
    ("next use: distance counted backwards", "ahead = min((u - t - 1) % period for u in where[cand])", "ahead = min((t - u - 1) % period for u in where[cand])"),
    ("next use: the later of a key's lookups counts", "ahead = min((u - t - 1) % period for u in where[cand])", "ahead = max((u - t - 1) % period for u in where[cand])"),
    ("next use: no wrap-around into the next sweep", "ahead = min((u - t - 1) % period for u in where[cand])",
     "ahead = min(((u - t - 1) if u > t else 10 ** 9) for u in where[cand])"),
    ("next use: the current group may be evicted", "                    if cand in current:\n                        continue\n", ""),
    ("next use: one slot too many", "            if len(resident) >= n_slots:", "            if len(resident) > n_slots:"),
    ("next use: victim stays resident", "                resident.discard(victim)\n", ""),
    ("sweep: forward by tile rows", "        for c in range(n_c):\n            groups.append([(l, r, c) for r in range(n_r)])",
     "        for r in range(n_r):\n            groups.append([(l, r, c) for c in range(n_c)])"),
    ("sweep: backward layers ascending", "    for l in range(L, 0, -1):", "    for l in range(1, L + 1):"),
    ("sweep: backward by tile columns", "        for r in range(n_r):\n            groups.append([(l, r, c) for c in range(n_c)])",
     "        for c in range(n_c):\n            groups.append([(l, r, c) for r in range(n_r)])"),
    ("sweep: tile counts rounded down", "        n_r, n_c = _ceil_div(dims[l - 1], T), _ceil_div(dims[l], T)\n        for c in range(n_c):",
     "        n_r, n_c = dims[l - 1] // T, dims[l] // T\n        for c in range(n_c):"),
]

PLAN_MUTANTS = [
    ("floor instead of ceil", "    return -(-a // b)", "    return a // b"),
    ("edge tiles counted as full", "    full = (n // t) ** 2", "    full = _ceil_div(n, t) ** 2"),
    ("edge not clamped", "r0=i * T, r1=min(M, (i + 1) * T)", "r0=i * T, r1=(i + 1) * T"),
    ("columns clamped to M", "c0=j * T, c1=min(N, (j + 1) * T)", "c0=j * T, c1=min(M, (j + 1) * T)"),
    ("id column-major", "id=i * n_j + j", "id=j * n_i + i"),
    ("k-steps from N", "n_i, n_j, n_k = _ceil_div(M, T), _ceil_div(N, T), _ceil_div(K, T)\n    tasks",
     "n_i, n_j, n_k = _ceil_div(M, T), _ceil_div(N, T), _ceil_div(N, T)\n    tasks"),
]


@pytest.mark.parametrize("name,old,new", LRU_MUTANTS, ids=[m[0] for m in LRU_MUTANTS])
def test_lru_mutant_is_caught(oracle, name, old, new):
    mod = _mutated_module(oracle, "lru.py", old, new)
    killers = _killed_by(_stand_in(oracle, mod), PLAN_LRU_PINS)
    print(name, "->", killers)
    assert killers, "no pin notices: " + name


@pytest.mark.parametrize("name,old,new", PLAN_MUTANTS, ids=[m[0] for m in PLAN_MUTANTS])
def test_plan_mutant_is_caught(oracle, name, old, new):
    mod = _mutated_module(oracle, "plan.py", old, new)
    killers = _killed_by(_stand_in(oracle, mod), PLAN_LRU_PINS)
    print(name, "->", killers)
    assert killers, "no pin notices: " + name


GEMM_PINS = ([(pins_gemm.test_identity_zero_ones, ()), (pins_gemm.test_rank1_closed_form, ()),
              (pins_gemm.test_brute_force_vs_numpy_all_small_shapes, ("f32",)),
              (pins_gemm.test_brute_force_vs_numpy_all_small_shapes, ("bf16",)),
              (pins_gemm.test_bf16_widening_is_exact, ()), (pins_gemm.test_pure_python_triple_loop, ()),
              (pins_gemm.test_integer_inputs_exact, ()), (pins_gemm.test_tiled_equals_untiled_any_T, ()),
              (pins_gemm.test_samples_match_full, ()), (pins_gemm.test_empty_dims, ())])

GEMM_C_MUTANTS = [
    ("A read transposed", "const double a = load_elem(A, m * sam + k * sak, dtype);",
     "const double a = load_elem(A, m * sak + k * sam, dtype);"),
    ("B read transposed", "row[n] += a * load_elem(B, k * sbk + n * sbn, dtype);",
     "row[n] += a * load_elem(B, k * sbn + n * sbk, dtype);"),
    ("C input dropped", "row[n] = c_in ? (double)c_in[m * ldc_in + n] : 0.0;", "row[n] = 0.0;"),
    ("last k dropped", "        for (int64_t k = 0; k < K; ++k) {\n            const double a",
     "        for (int64_t k = 0; k < K - 1; ++k) {\n            const double a"),
    ("difference instead of sum", "row[n] += a * load_elem(B, k * sbk + n * sbn, dtype);",
     "row[n] -= a * load_elem(B, k * sbk + n * sbn, dtype);"),
    ("bf16 widened from the low half", "uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]) << 16;",
     "uint32_t bits = ((uint32_t)((const uint16_t *)base)[idx]);"),
    ("tiled: edge tile not clamped in k", "const int64_t k0 = tk * T, k1 = min64(K, k0 + T);",
     "const int64_t k0 = tk * T, k1 = (tk + 1 < nK) ? k0 + T : k0 + (K - k0) / 2 * 2;"),
    ("tiled: k-steps overwrite instead of accumulate", "                    c_out[m * N + n] += s;",
     "                    c_out[m * N + n] = s;"),
    ("samples: row and column swapped", "const int64_t m = rows[s], n = cols[s];", "const int64_t m = cols[s], n = rows[s];"),
    ("samples: C input dropped", "double acc = c_in ? (double)c_in[m * ldc_in + n] : 0.0;", "double acc = 0.0;"),
]


ROUNDING_PINS = [(pins_round.test_mix32_known_answers, ()), (pins_round.test_mix32_is_inverted_by_the_closed_form_inverse, ()),
                 (pins_round.test_step_key_depends_on_every_argument, ()),
                 (pins_round.test_rounding_over_all_random_values_is_exactly_unbiased, ()),
                 (pins_round.test_rounding_special_values, ()), (pins_round.test_rounding_bits_layout_and_statistics, ()),
                 (pins_round.test_rounding_a_matrix_is_unbiased_where_nearest_loses_the_update, ()),
                 (pins_round.test_mlp_step_stochastic_brackets_the_exact_update, ()),
                 (pins_round.test_nearest_even_against_torch_and_by_brute_force, ())]

ROUNDING_MUTANTS = [
    ("finalizer: wrong middle shift", "    x = x ^ (x >> np.uint64(13))", "    x = x ^ (x >> np.uint64(15))"),
    ("finalizer: last xor-shift dropped", "    x = (x * np.uint64(0xC2B2AE35)) & _M32\n    x = x ^ (x >> np.uint64(16))",
     "    x = (x * np.uint64(0xC2B2AE35)) & _M32"),
    ("finalizer: multipliers swapped", "    x = (x * np.uint64(0x85EBCA6B)) & _M32", "    x = (x * np.uint64(0xC2B2AE35)) & _M32 if False else (x * np.uint64(0xC2B2AE37)) & _M32"),
    ("key ignores the step", "    k = mix32(k ^ np.uint64(int(step) & 0xFFFFFFFF))", "    k = mix32(k)"),
    ("key ignores the layer", "    k = mix32(k ^ np.uint64(int(layer) & 0xFFFFFFFF))", "    k = mix32(k)"),
    ("key ignores the high half of the seed", "    k = mix32(k ^ np.uint64((seed >> 32) & 0xFFFFFFFF))", "    k = mix32(k)"),
    ("bits ignore the row", "    hrow = mix32((rows + np.uint64(key)) & _M32)", "    hrow = mix32((rows * np.uint64(0) + np.uint64(key)) & _M32)"),
    ("bits: one word per column instead of per pair", "(((cols >> np.uint64(1)) * np.uint64(0x9E3779B9)) & _M32)",
     "((cols * np.uint64(0x9E3779B9)) & _M32)"),
    ("bits: halves swapped", "np.where(odd, bits >> np.uint64(16), bits & np.uint64(0xFFFF))",
     "np.where(odd, bits & np.uint64(0xFFFF), bits >> np.uint64(16))"),
    ("bits: only 15 random bits", "np.where(odd, bits >> np.uint64(16), bits & np.uint64(0xFFFF))",
     "np.where(odd, bits >> np.uint64(17), bits & np.uint64(0x7FFF))"),
    ("rounding: random bits not added (truncation)", "    out = ((u + r) >> np.uint64(16)) & np.uint64(0xFFFF)",
     "    out = (u >> np.uint64(16)) & np.uint64(0xFFFF)"),
    ("rounding: nearest instead of stochastic", "    out = ((u + r) >> np.uint64(16)) & np.uint64(0xFFFF)",
     "    out = ((u + np.uint64(0x8000)) >> np.uint64(16)) & np.uint64(0xFFFF)"),
    ("rounding: one added to the random bits (rounds exact values up)", "    out = ((u + r) >> np.uint64(16)) & np.uint64(0xFFFF)",
     "    out = ((u + r + np.uint64(1)) >> np.uint64(16)) & np.uint64(0xFFFF)"),
    ("rounding: NaN not kept quiet", "np.where(is_nan, np.uint64(0x40), np.uint64(0))", "np.where(is_nan, np.uint64(0), np.uint64(0))"),
    ("nearest: ties go up", "    take_up = (low > half) | ((low == half) & ((down & np.uint64(1)) == np.uint64(1)))", "    take_up = low >= half"),
    ("nearest: ties go to the odd pattern", "((low == half) & ((down & np.uint64(1)) == np.uint64(1)))", "((low == half) & ((down & np.uint64(1)) == np.uint64(0)))"),
    ("nearest: ties go down", "    take_up = (low > half) | ((low == half) & ((down & np.uint64(1)) == np.uint64(1)))", "    take_up = low > half"),
    ("nearest: NaN loses its payload", "    keep = np.where(is_nan, down | np.uint64(0x40), down)", "    keep = np.where(is_nan, down & np.uint64(0xFF80), down)"),
    ("nearest: infinities rounded like numbers", "    return np.where(special, keep, out).astype(np.uint16)\n\n\ndef stochastic_round_matrix",
     "    return np.where(is_nan, keep, np.where(special, up, out)).astype(np.uint16)\n\n\ndef stochastic_round_matrix"),
    ("matrix: rows and columns swapped", "np.arange(n_r, dtype=np.uint64)[:, None], np.arange(n_c, dtype=np.uint64)[None, :]",
     "np.arange(n_c, dtype=np.uint64)[None, :], np.arange(n_r, dtype=np.uint64)[:, None]"),
]


@pytest.mark.parametrize("name,old,new", ROUNDING_MUTANTS, ids=[m[0] for m in ROUNDING_MUTANTS])
def test_rounding_mutant_is_caught(oracle, name, old, new):
    mod = _mutated_module(oracle, "rounding.py", old, new)
    killers = _killed_by(_stand_in(oracle, mod), ROUNDING_PINS)
    print(name, "->", killers)
    assert killers, "no pin notices: " + name


@pytest.fixture(scope="module")
def mutant_dir(tmp_path_factory):
    return tmp_path_factory.mktemp("oracle_mutants")


@pytest.mark.parametrize("name,old,new", GEMM_C_MUTANTS, ids=[m[0] for m in GEMM_C_MUTANTS])
def test_gemm_c_mutant_is_caught(oracle, mutant_dir, name, old, new):
    src = open(os.path.join(ROOT, "oracle", "oracle_gemm.c")).read()
    assert src.count(old) == 1, "mutation target must occur exactly once: %r" % old
    tag = "m%d" % [m[0] for m in GEMM_C_MUTANTS].index(name)
    c_path, so_path = str(mutant_dir / (tag + ".c")), str(mutant_dir / (tag + ".so"))
    open(c_path, "w").write(src.replace(old, new))
    subprocess.run(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", so_path, c_path], check=True)
    # the ctypes front end, unchanged, on top of the mutated library
    mod = _mutated_module(oracle, "gemm.py", "from .build import build_oracle\n",
                          "build_oracle = lambda: %r\n" % so_path)
    killers = _killed_by(_stand_in(oracle, mod), GEMM_PINS)
    print(name, "->", killers)
    assert killers, "no pin notices: " + name


def test_the_untouched_oracle_passes_every_pin(oracle):
    """The harness itself: with no substitution nothing is reported."""
    ident = _mutated_module(oracle, "mlp.py", "import numpy as np\n", "import numpy as np\n")
    assert _killed_by(_stand_in(oracle, ident), MLP_PINS) == []
    ident = _mutated_module(oracle, "lru.py", "from collections import OrderedDict\n", "from collections import OrderedDict\n")
    assert _killed_by(_stand_in(oracle, ident), PLAN_LRU_PINS) == []
    ident = _mutated_module(oracle, "plan.py", "def _ceil_div(a, b):", "def _ceil_div(a, b):")
    assert _killed_by(_stand_in(oracle, ident), PLAN_LRU_PINS) == []
    ident = _mutated_module(oracle, "rounding.py", "import numpy as np\n", "import numpy as np\n")
    assert _killed_by(_stand_in(oracle, ident), ROUNDING_PINS) == []
    ident = _mutated_module(oracle, "gemm.py", "from .build import build_oracle\n", "from .build import build_oracle\n")
    assert _killed_by(_stand_in(oracle, ident), GEMM_PINS) == []
