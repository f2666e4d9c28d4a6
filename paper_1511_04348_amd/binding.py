"""ctypes binding of libtgemm.so: argument marshalling only, same names as include/tgemm.h.

Pointers are passed as integers (``tensor.data_ptr()``) or anything with a ``data_ptr()`` method.
Every error code raises ``TgemmError`` carrying the code and the library's message.  The library
must have been built (``python -m paper_1511_04348_amd.build``); there is no fallback.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libtgemm.so")

TGEMM_F32, TGEMM_BF16 = 0, 1
TGEMM_OK, TGEMM_EARG, TGEMM_ENOMEM, TGEMM_EUNPINNED, TGEMM_EBUDGET, TGEMM_EHIP, TGEMM_ESTATE = 0, -1, -2, -3, -4, -5, -6
TGEMM_ORDER_SERPENTINE, TGEMM_ORDER_ROW_MAJOR, TGEMM_ORDER_STRIPS = 0, 1, 2
TGEMM_SCHEDULE_AUTO, TGEMM_SCHEDULE_ONE_LAUNCH, TGEMM_SCHEDULE_BALANCED = 0, 1, 2
TGEMM_ACT_SIGMOID, TGEMM_ACT_TANH, TGEMM_ACT_RELU = 0, 1, 2
TGEMM_ROUND_NEAREST, TGEMM_ROUND_STOCHASTIC = 0, 1

EXPORTS = [
    "tgemm_strerror", "tgemm_last_error", "tgemm_create", "tgemm_destroy", "tgemm_run", "tgemm_sync", "tgemm_invalidate",
    "tgemm_plan", "tgemm_task_order", "tgemm_last_stats", "tgemm_trace", "tgemm_queue_selftest", "tgemm_balance_plan",
    "mlp_create", "mlp_destroy", "mlp_set_activation", "mlp_set_rounding", "mlp_set_bias", "mlp_set_momentum", "mlp_set_master_weights", "mlp_forward", "mlp_forward_static", "mlp_backward", "mlp_step", "mlp_read", "mlp_trace",
]


class tgemm_opts(ctypes.Structure):
    _fields_ = [("trace", ctypes.c_int32), ("order", ctypes.c_int32), ("affinity_core", ctypes.c_int32),
                ("async_incore", ctypes.c_int32), ("kernel_config", ctypes.c_int32),
                ("strip_width", ctypes.c_int32), ("deferred_writeback", ctypes.c_int32),
                ("rs_depth", ctypes.c_int32), ("exact_replacement", ctypes.c_int32), ("keep_tiles", ctypes.c_int32),
                ("incore_schedule", ctypes.c_int32)]


class tgemm_segment(ctypes.Structure):
    _fields_ = [("tile", ctypes.c_int32), ("first_chunk", ctypes.c_int32), ("n_chunks", ctypes.c_int32), ("slot", ctypes.c_int32)]


class tgemm_balance(ctypes.Structure):
    _fields_ = [("applies", ctypes.c_int32), ("whole_round_tiles", ctypes.c_int32), ("tail_tiles", ctypes.c_int32),
                ("n_segments", ctypes.c_int32), ("chunks_per_tile", ctypes.c_int32), ("even_parts", ctypes.c_int32),
                ("interior_rows", ctypes.c_int64), ("interior_cols", ctypes.c_int64)]


class tgemm_task(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int64) for n in ("id", "i", "j", "r0", "r1", "c0", "c1", "n_k")]


class tgemm_stats(ctypes.Structure):
    _fields_ = [("wall_ms", ctypes.c_double), ("kernel_ms", ctypes.c_double)] + \
               [(n, ctypes.c_int64) for n in ("in_core", "n_tasks", "n_tile_gemms", "n_slots", "hits", "misses",
                                              "evictions", "h2d_bytes", "d2h_bytes", "kernel_launches")]

    def as_dict(self):
        return {n: getattr(self, n) for n, _ in self._fields_}


class tgemm_trace_rec(ctypes.Structure):
    _fields_ = [("task_id", ctypes.c_int64)] + \
               [(n, ctypes.c_int32) for n in ("i", "j", "k", "stream", "a_hit", "b_hit", "a_slot", "b_slot",
                                              "a_evicted", "b_evicted")]


class tgemm_mlp_trace_rec(ctypes.Structure):
    _fields_ = [("group", ctypes.c_int64)] + \
               [(n, ctypes.c_int32) for n in ("layer", "r", "c", "backward", "hit", "slot", "ev_layer", "ev_r", "ev_c")]


class TgemmError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__("tgemm error %d: %s" % (code, msg))
        self.code = code


_lib = None


def load():
    """Loads libtgemm.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libtgemm.so is missing at %s: run `python -m paper_1511_04348_amd.build` "
                           "(there is no CPU fallback)" % LIB_PATH)
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    P = ctypes.POINTER
    lib.tgemm_strerror.argtypes, lib.tgemm_strerror.restype = [ctypes.c_int], ctypes.c_char_p
    lib.tgemm_last_error.argtypes, lib.tgemm_last_error.restype = [], ctypes.c_char_p
    lib.tgemm_create.argtypes = [P(vp), ctypes.c_int, P(vp), P(tgemm_opts)]
    lib.tgemm_destroy.argtypes = [vp]
    lib.tgemm_run.argtypes = [vp, vp, vp, vp, i64, i64, i64, i32, i32, sz]
    lib.tgemm_sync.argtypes = [vp]
    lib.tgemm_invalidate.argtypes = [vp, vp]
    lib.tgemm_plan.argtypes = [i64, i64, i64, i32, P(tgemm_task), i64, P(i64)]
    lib.tgemm_task_order.argtypes = [i64, i64, i32, i64, P(i64)]
    lib.tgemm_last_stats.argtypes = [vp, P(tgemm_stats)]
    lib.tgemm_trace.argtypes = [vp, P(tgemm_trace_rec), i64, P(i64)]
    lib.tgemm_queue_selftest.argtypes = [i64, i32, i32, P(i32)]
    lib.tgemm_balance_plan.argtypes = [i64, i64, i64, i32, i32, i32, i32, P(tgemm_balance), P(tgemm_segment), i64]
    lib.mlp_create.argtypes = [vp, P(vp), i32, P(i64), P(vp), i32, i32, sz]
    lib.mlp_destroy.argtypes = [vp]
    lib.mlp_set_activation.argtypes = [vp, i32]
    lib.mlp_set_rounding.argtypes = [vp, i32, ctypes.c_uint64]
    lib.mlp_set_bias.argtypes = [vp, P(vp), P(vp)]
    lib.mlp_set_momentum.argtypes = [vp, ctypes.c_float, P(vp), P(vp)]
    lib.mlp_set_master_weights.argtypes = [vp, P(vp)]
    lib.mlp_forward.argtypes = [vp, vp, i64, vp]
    lib.mlp_forward_static.argtypes = [vp, vp, i64, vp]
    lib.mlp_backward.argtypes = [vp, vp, P(vp), P(ctypes.c_float)]
    lib.mlp_step.argtypes = [vp, vp, vp, i64, ctypes.c_float, P(ctypes.c_float)]
    lib.mlp_read.argtypes = [vp, i32, i32, vp, sz, sz]
    lib.mlp_trace.argtypes = [vp, P(tgemm_mlp_trace_rec), i64, P(i64)]
    for name in EXPORTS:
        if name not in ("tgemm_strerror", "tgemm_last_error"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def _check(rc):
    if rc != 0:
        raise TgemmError(rc, load().tgemm_last_error().decode("utf-8", "replace"))


def _p(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    if hasattr(x, "cuda_stream"):
        return x.cuda_stream
    return int(x)


def tgemm_strerror(code):
    return load().tgemm_strerror(code).decode()


def tgemm_last_error():
    return load().tgemm_last_error().decode("utf-8", "replace")


def tgemm_create(device=0, streams=None, trace=0, order=TGEMM_ORDER_STRIPS, affinity_core=-1,
                 async_incore=0, kernel_config=0, strip_width=0, deferred_writeback=0, rs_depth=0,
                 exact_replacement=0, keep_tiles=0, incore_schedule=0):
    lib = load()
    o = tgemm_opts(trace=trace, order=order, affinity_core=affinity_core, async_incore=async_incore,
                   kernel_config=kernel_config, strip_width=strip_width,
                   deferred_writeback=deferred_writeback, rs_depth=rs_depth, exact_replacement=exact_replacement, keep_tiles=keep_tiles,
                   incore_schedule=incore_schedule)
    arr = None
    if streams is not None:
        if len(streams) != 4:
            raise ValueError("streams must have 4 entries")
        arr = (ctypes.c_void_p * 4)(*[_p(s) for s in streams])
    out = ctypes.c_void_p()
    _check(lib.tgemm_create(ctypes.byref(out), device, arr, ctypes.byref(o)))
    return out


def tgemm_destroy(ctx):
    _check(load().tgemm_destroy(ctx))


def tgemm_run(ctx, A, B, C, M, N, K, T, dtype=TGEMM_F32, hbm_budget=0):
    _check(load().tgemm_run(ctx, _p(A), _p(B), _p(C), M, N, K, T, dtype, hbm_budget))


def tgemm_sync(ctx):
    _check(load().tgemm_sync(ctx))


def tgemm_invalidate(ctx, host_matrix):
    _check(load().tgemm_invalidate(ctx, _p(host_matrix)))


def tgemm_plan(M, N, K, T):
    lib = load()
    n = ctypes.c_int64()
    _check(lib.tgemm_plan(M, N, K, T, None, 0, ctypes.byref(n)))
    buf = (tgemm_task * max(1, n.value))()
    _check(lib.tgemm_plan(M, N, K, T, buf, n.value, ctypes.byref(n)))
    return [{f: getattr(buf[t], f) for f, _ in tgemm_task._fields_} for t in range(n.value)]


def tgemm_task_order(n_i, n_j, order, strip=1):
    buf = (ctypes.c_int64 * max(1, n_i * n_j))()
    _check(load().tgemm_task_order(n_i, n_j, order, strip, buf))
    return list(buf[: n_i * n_j])


def tgemm_last_stats(ctx):
    s = tgemm_stats()
    _check(load().tgemm_last_stats(ctx, ctypes.byref(s)))
    return s.as_dict()


def tgemm_trace(ctx):
    lib = load()
    n = ctypes.c_int64()
    _check(lib.tgemm_trace(ctx, None, 0, ctypes.byref(n)))
    buf = (tgemm_trace_rec * max(1, n.value))()
    _check(lib.tgemm_trace(ctx, buf, n.value, ctypes.byref(n)))
    return [{f: getattr(buf[t], f) for f, _ in tgemm_trace_rec._fields_} for t in range(n.value)]


def tgemm_balance_plan(M, N, K, T, dtype=0, n_cus=256, whatever_the_estimate=0):
    """(plan as a dict, segments in launch order as a list of dicts); plan["applies"] == 0: one launch."""
    lib = load()
    b = tgemm_balance()
    _check(lib.tgemm_balance_plan(M, N, K, T, dtype, n_cus, whatever_the_estimate, ctypes.byref(b), None, 0))
    segs = (tgemm_segment * max(1, b.n_segments))()
    _check(lib.tgemm_balance_plan(M, N, K, T, dtype, n_cus, whatever_the_estimate, ctypes.byref(b), segs, b.n_segments))
    plan = {f: getattr(b, f) for f, _ in tgemm_balance._fields_}
    return plan, [{f: getattr(segs[i], f) for f, _ in tgemm_segment._fields_} for i in range(b.n_segments)]


def tgemm_queue_selftest(n, producers, consumers):
    buf = (ctypes.c_int32 * max(1, n))()
    _check(load().tgemm_queue_selftest(n, producers, consumers, buf))
    return list(buf[:n])


def mlp_create(ctx, dims, weights, dtype=TGEMM_F32, T=1024, hbm_budget=0):
    n_layers = len(weights)
    if len(dims) != n_layers + 1:
        raise ValueError("dims must have n_layers + 1 entries")
    d = (ctypes.c_int64 * len(dims))(*dims)
    w = (ctypes.c_void_p * n_layers)(*[_p(x) for x in weights])
    out = ctypes.c_void_p()
    _check(load().mlp_create(ctx, ctypes.byref(out), n_layers, d, w, dtype, T, hbm_budget))
    return out


def mlp_destroy(mlp):
    _check(load().mlp_destroy(mlp))


def mlp_set_activation(mlp, act):
    _check(load().mlp_set_activation(mlp, act))


def mlp_set_rounding(mlp, mode, seed=0):
    _check(load().mlp_set_rounding(mlp, mode, seed))


def mlp_set_bias(mlp, b, db=None):
    """b: list of float device tensors (one row per layer) or None; db: optional list (entries may be None)."""
    arr_b = (ctypes.c_void_p * len(b))(*[_p(x) for x in b]) if b is not None else None
    arr_db = (ctypes.c_void_p * len(db))(*[_p(x) for x in db]) if db is not None else None
    _check(load().mlp_set_bias(mlp, arr_b, arr_db))


def mlp_set_momentum(mlp, mu, V, Vb=None):
    """V: list of float device tensors shaped like the weights, or None; Vb: optional list of float rows."""
    arr_v = (ctypes.c_void_p * len(V))(*[_p(x) for x in V]) if V is not None else None
    arr_vb = (ctypes.c_void_p * len(Vb))(*[_p(x) for x in Vb]) if Vb is not None else None
    _check(load().mlp_set_momentum(mlp, mu, arr_v, arr_vb))


def mlp_set_master_weights(mlp, Wm):
    """Wm: list of float device tensors shaped like the (bf16) weights, or None."""
    arr = (ctypes.c_void_p * len(Wm))(*[_p(x) for x in Wm]) if Wm is not None else None
    _check(load().mlp_set_master_weights(mlp, arr))


def mlp_forward(mlp, X, batch, probs=None):
    _check(load().mlp_forward(mlp, _p(X), batch, _p(probs)))


def mlp_forward_static(mlp, X, batch, probs):
    _check(load().mlp_forward_static(mlp, _p(X), batch, _p(probs)))


def mlp_backward(mlp, labels, dW=None):
    loss = ctypes.c_float()
    arr = None
    if dW is not None:
        arr = (ctypes.c_void_p * len(dW))(*[_p(x) for x in dW])
    _check(load().mlp_backward(mlp, _p(labels), arr, ctypes.byref(loss)))
    return loss.value


def mlp_step(mlp, X, labels, batch, lr):
    loss = ctypes.c_float()
    _check(load().mlp_step(mlp, _p(X), _p(labels), batch, lr, ctypes.byref(loss)))
    return loss.value


def mlp_read(mlp, what, layer, dst, nbytes, offset=0):
    _check(load().mlp_read(mlp, what, layer, _p(dst), offset, nbytes))


def mlp_trace(mlp):
    lib = load()
    n = ctypes.c_int64()
    _check(lib.mlp_trace(mlp, None, 0, ctypes.byref(n)))
    buf = (tgemm_mlp_trace_rec * max(1, n.value))()
    _check(lib.mlp_trace(mlp, buf, n.value, ctypes.byref(n)))
    return [{f: getattr(buf[t], f) for f, _ in tgemm_mlp_trace_rec._fields_} for t in range(n.value)]
