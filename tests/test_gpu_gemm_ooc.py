"""GPU parity of the out-of-core tiled GEMM (matrices in pinned host memory, tiles staged through
the bounded HBM tile cache on 4 streams) against the CPU oracle, through the C ABI.

Checked: values (bit-exact for integer inputs, rel. Frobenius <= 1e-5 for uniform fp32), the
per-step trace against the oracle's independent task enumeration and LRU simulation (bit-exact),
the transfer statistics, error paths, and config 3 at full size by sampled entries plus a
Freivalds-style identity C x = A (B x) that touches every tile."""
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import pytest
import torch

from gpu_util import announce, rel_fro
from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs

pytestmark = pytest.mark.gpu
TOL_F32 = 1e-5


def _pinned(t):
    return t.contiguous().pin_memory()


def _budget(T, n_ab, M, N, K):
    tm, tn, tk = min(T, M), min(T, N), min(T, K)
    up = lambda v: (v + 255) // 256 * 256
    return 4 * up(tm * tn * 4) + n_ab * up(max(tm * tk, tk * tn) * 4)


def _check_trace(oracle, ctx, M, N, K, T, order_name, n_slots, strip=None):
    trace = tg.tgemm_trace(ctx)
    seq = oracle.tgemm_access_sequence(M, N, K, T, order=order_name, strip=strip)
    events, st = oracle.lru_simulate([s[:3] for s in seq], n_slots)
    assert len(trace) * 2 == len(seq)
    n_j = -(-N // T)
    per_task_stream = {}
    for t, rec in enumerate(trace):
        (ma, ai, ak, tid, k), (mb, bk, bj, _, _) = seq[2 * t], seq[2 * t + 1]
        assert (rec["task_id"], rec["i"], rec["j"], rec["k"]) == (tid, tid // n_j, tid % n_j, k)
        assert (rec["i"], rec["k"]) == (ai, ak) and (rec["k"], rec["j"]) == (bk, bj)
        assert bool(rec["a_hit"]) == events[2 * t][0] and bool(rec["b_hit"]) == events[2 * t + 1][0]
        assert bool(rec["a_evicted"]) == (events[2 * t][1] is not None)
        assert bool(rec["b_evicted"]) == (events[2 * t + 1][1] is not None)
        assert 0 <= rec["stream"] < 4 and rec["a_slot"] != rec["b_slot"]
        assert per_task_stream.setdefault(tid, rec["stream"]) == rec["stream"]   # one task, one stream
    stats = tg.tgemm_last_stats(ctx)
    assert (stats["hits"], stats["misses"], stats["evictions"]) == (st["hits"], st["misses"], st["evictions"])
    return seq, events, stats


def _tile_bytes(key, M, N, K, T):
    mat, r, c = key
    rows = min(T, (M if mat == "A" else K) - r * T)
    cols = min(T, (K if mat == "A" else N) - c * T)
    return rows * cols * 4


@pytest.mark.parametrize("order,order_name,strip", [(tg.TGEMM_ORDER_SERPENTINE, "serpentine", 0),
                                                    (tg.TGEMM_ORDER_ROW_MAJOR, "row_major", 0),
                                                    (tg.TGEMM_ORDER_STRIPS, "strips", 0),     # automatic width
                                                    (tg.TGEMM_ORDER_STRIPS, "strips", 3)])
@pytest.mark.parametrize("M,N,K,T,n_ab", [(1500, 1400, 1300, 256, 20), (640, 640, 640, 128, 8),
                                          (300, 2000, 700, 256, 11), (1024, 1024, 1024, 256, 64),
                                          (1280, 2304, 768, 256, 15)])
def test_scaled_down_parity_trace_and_stats(oracle, M, N, K, T, n_ab, order, order_name, strip):
    announce("ooc", M, N, K, T, n_ab, order_name, strip)
    A = inputs.uniform_matrix(1, M, K)
    B = inputs.uniform_matrix(2, K, N)
    C0 = inputs.uniform_matrix(3, M, N)
    ref = oracle.gemm(A.numpy(), B.numpy(), c_in=C0.numpy())
    ctx = tg.tgemm_create(0, trace=1, order=order, strip_width=strip)
    try:
        Ap, Bp, Cp = _pinned(A), _pinned(B), _pinned(C0)
        tg.tgemm_run(ctx, Ap, Bp, Cp, M, N, K, T, tg.TGEMM_F32, _budget(T, n_ab, M, N, K))
        err = rel_fro(Cp.numpy(), ref)
        print("rel fro", err)
        assert err <= TOL_F32
        assert torch.equal(Ap, A) and torch.equal(Bp, B)           # inputs untouched
        stats = tg.tgemm_last_stats(ctx)
        n_i, n_j, n_k = -(-M // T), -(-N // T), -(-K // T)
        distinct = n_i * n_k + n_k * n_j
        assert stats["n_slots"] == min(n_ab, distinct) and stats["in_core"] == 0
        assert stats["n_tasks"] == n_i * n_j and stats["n_tile_gemms"] == n_i * n_j * n_k == stats["kernel_launches"]
        if order_name == "strips" and strip == 0:
            strip = oracle.auto_strip(stats["n_slots"], n_k, n_j)
        seq, events, _ = _check_trace(oracle, ctx, M, N, K, T, order_name, stats["n_slots"], strip or None)
        miss_bytes = sum(_tile_bytes(s[:3], M, N, K, T) for s, e in zip(seq, events) if not e[0])
        assert stats["h2d_bytes"] == miss_bytes + M * N * 4          # every miss fetched once + C in
        assert stats["d2h_bytes"] == M * N * 4                       # every C tile harvested once
        assert stats["misses"] >= distinct                         # at least the compulsory ones
    finally:
        tg.tgemm_destroy(ctx)


def test_integer_inputs_bit_exact_and_repeatable(oracle):
    M, N, K, T = 1100, 900, 1300, 256
    A = inputs.int_matrix(11, M, K)
    B = inputs.int_matrix(12, K, N)
    C0 = inputs.int_matrix(13, M, N, lo=-7, hi=7)
    ref = oracle.gemm(A.numpy(), B.numpy(), c_in=C0.numpy())
    ctx = tg.tgemm_create(0)
    try:
        Ap, Bp = _pinned(A), _pinned(B)
        for rep in range(3):          # the pool and its events are reused across runs
            announce("ooc int rep", rep)
            Cp = _pinned(C0)
            tg.tgemm_run(ctx, Ap, Bp, Cp, M, N, K, T, tg.TGEMM_F32, _budget(T, 9 + rep, M, N, K))
            assert np.array_equal(Cp.numpy().astype(np.float64), ref)
    finally:
        tg.tgemm_destroy(ctx)


def test_uniform_run_is_bitwise_reproducible_across_orders(oracle):
    """Each C element belongs to one task and its k-steps ascend, so the task order and the
    stream a task lands on must not change a single bit."""
    M, N, K, T = 900, 1000, 1100, 256
    A = _pinned(inputs.uniform_matrix(1, M, K))
    B = _pinned(inputs.uniform_matrix(2, K, N))
    outs = []
    for order in (tg.TGEMM_ORDER_SERPENTINE, tg.TGEMM_ORDER_ROW_MAJOR, tg.TGEMM_ORDER_STRIPS):
        ctx = tg.tgemm_create(0, order=order, strip_width=2)
        try:
            C = torch.zeros(M, N).pin_memory()
            tg.tgemm_run(ctx, A, B, C, M, N, K, T, tg.TGEMM_F32, _budget(T, 8, M, N, K))
            outs.append(C.clone())
        finally:
            tg.tgemm_destroy(ctx)
    assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2])


@pytest.mark.parametrize("dtype,M,N,K,T", [("f32", 1024, 768, 512, 256),      # 16-byte units
                                          ("f32", 1101, 903, 1303, 256),     # odd pitch: 4-byte units
                                          ("bf16", 1024, 1024, 512, 256),    # 16-byte units
                                          ("bf16", 1101, 903, 1303, 256)])   # odd pitch: 2-byte units
def test_copy_kernel_transfers_match_dma(oracle, monkeypatch, dtype, M, N, K, T):
    """The optional transfer path (a strided copy kernel that reads and writes the pinned host
    matrices directly) must give the bits the DMA path gives, and both the oracle's values:
    integer inputs, so the comparison is exact.  The unit width of the copy follows the
    alignment of pointers, pitches and row bytes, hence the odd shapes."""
    announce("ooc copy kernel", dtype, M, N, K, T)
    A = inputs.int_matrix(21, M, K)
    B = inputs.int_matrix(22, K, N)
    C0 = inputs.int_matrix(23, M, N, lo=-7, hi=7)
    if dtype == "bf16":
        A, B = A.to(torch.bfloat16), B.to(torch.bfloat16)      # small integers: exact
        code, esz = tg.TGEMM_BF16, 2
    else:
        code, esz = tg.TGEMM_F32, 4
    ref = oracle.gemm(A.float().numpy(), B.float().numpy(), c_in=C0.numpy())
    Ap, Bp = _pinned(A), _pinned(B)
    budget = 4 * T * T * 4 + 9 * T * T * esz
    outs = {}
    for mode in ("kernel", "dma"):
        monkeypatch.setenv("TGEMM_COPY", mode)
        ctx = tg.tgemm_create(0, order=tg.TGEMM_ORDER_SERPENTINE)
        try:
            Cp = _pinned(C0)
            tg.tgemm_run(ctx, Ap, Bp, Cp, M, N, K, T, code, budget)
            st = tg.tgemm_last_stats(ctx)
            assert st["in_core"] == 0 and st["n_slots"] == 9 and st["evictions"] > 0
            outs[mode] = Cp.clone()
        finally:
            tg.tgemm_destroy(ctx)
    assert np.array_equal(outs["kernel"].numpy().astype(np.float64), ref)
    assert torch.equal(outs["kernel"], outs["dma"])
    assert torch.equal(Ap, A) and torch.equal(Bp, B)


def test_changed_host_matrix_is_seen_by_the_next_call(oracle):
    """No tile outlives a call: after the caller changes A in place the next product uses the new
    values, with or without tgemm_invalidate (which has nothing to drop and says so by succeeding)."""
    M = N = K = 192
    T = 64
    A = inputs.int_matrix(1, M, K).pin_memory()
    B = inputs.int_matrix(2, K, N).pin_memory()
    ctx = tg.tgemm_create(0)
    try:
        for k in range(3):
            C = torch.zeros(M, N).pin_memory()
            tg.tgemm_run(ctx, A, B, C, M, N, K, T, tg.TGEMM_F32, 40 * T * T * 4)
            assert np.array_equal(C.numpy().astype(np.float64), oracle.gemm(A.numpy(), B.numpy()))
            A.mul_(-2.0)                       # the caller rewrites its matrix between calls
            if k == 1:
                tg.tgemm_invalidate(ctx, A)
    finally:
        tg.tgemm_destroy(ctx)


def _names_sequence(oracle, M, N, K, T, order_name, name_a, name_b, strip=None):
    seq = oracle.tgemm_access_sequence(M, N, K, T, order=order_name, strip=strip)
    return [((name_a if s[0] == "A" else name_b), s[1], s[2]) for s in seq]


def test_tiles_survive_between_calls_and_invalidate_drops_them(oracle):
    """tgemm_opts.keep_tiles (section 3.4: cached tiles are reused): a later call on the context finds
    the tiles an earlier call left, recency order included; a matrix seen as the left operand is the
    same matrix when it comes back as the right operand; tgemm_invalidate drops one matrix's tiles.
    Hits, misses and evictions of every call equal the oracle's strict LRU run over the calls' lookups
    put end to end (keys = matrix, tile row, tile column), with the invalidation marked; results are
    bit-exact (integer inputs); without the invalidation a changed matrix is seen stale, which is the
    caller's error in this mode and shows that the copy really was reused."""
    n, T, n_ab = 640, 128, 30
    announce("out-of-core GEMM: tiles kept across calls", n, T, n_ab)
    X = inputs.int_matrix(1, n, n).pin_memory()
    Y = inputs.int_matrix(2, n, n).pin_memory()
    Z = inputs.int_matrix(3, n, n).pin_memory()
    budget = _budget(T, n_ab, n, n, n)
    ctx = tg.tgemm_create(0, trace=1, keep_tiles=1, order=tg.TGEMM_ORDER_SERPENTINE)
    keys, calls = [], []

    def run(A, name_a, B, name_b):
        C = torch.zeros(n, n).pin_memory()
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, budget)
        ks = _names_sequence(oracle, n, n, n, T, "serpentine", name_a, name_b)
        keys.extend(ks)
        calls.append((tg.tgemm_trace(ctx), tg.tgemm_last_stats(ctx), len(ks)))
        return C

    try:
        C1 = run(X, "X", Y, "Y")
        assert np.array_equal(C1.numpy().astype(np.float64), oracle.gemm(X.numpy(), Y.numpy()))
        C2 = run(X, "X", Z, "Z")                     # X's tiles are still there
        assert np.array_equal(C2.numpy().astype(np.float64), oracle.gemm(X.numpy(), Z.numpy()))
        C3 = run(Z, "Z", X, "X")                     # the same matrices in the other roles
        assert np.array_equal(C3.numpy().astype(np.float64), oracle.gemm(Z.numpy(), X.numpy()))
        X_old = X.clone()
        X.mul_(-2.0)                                 # the caller changes X ...
        tg.tgemm_invalidate(ctx, X)                  # ... and says so
        keys.append(oracle.Invalidate("X"))
        C4 = run(Z, "Z", X, "X")
        assert np.array_equal(C4.numpy().astype(np.float64), oracle.gemm(Z.numpy(), X.numpy()))
        assert not torch.equal(X, X_old)
    finally:
        tg.tgemm_destroy(ctx)
    events, _ = oracle.lru_simulate(keys, n_ab)
    at = 0
    reused = 0
    for c, (trace, st, n_lookups) in enumerate(calls):
        assert len(trace) * 2 == n_lookups and st["n_slots"] == n_ab
        ev = events[at:at + n_lookups]
        at += n_lookups
        for t, rec in enumerate(trace):
            assert bool(rec["a_hit"]) == ev[2 * t][0] and bool(rec["b_hit"]) == ev[2 * t + 1][0], (c, t)
            assert bool(rec["a_evicted"]) == (ev[2 * t][1] is not None) and bool(rec["b_evicted"]) == (ev[2 * t + 1][1] is not None)
        hits = sum(1 for e in ev if e[0])
        assert (st["hits"], st["misses"], st["evictions"]) == (hits, len(ev) - hits, sum(1 for e in ev if e[1] is not None)), c
        assert st["h2d_bytes"] == (len(ev) - hits) * T * T * 4 + n * n * 4
        if c > 0:
            alone, _ = oracle.lru_simulate(keys_of_call(keys, calls, c), n_ab)
            reused += hits - sum(1 for e in alone if e[0])
    assert at == len(events) and reused > 0            # later calls hit tiles that earlier calls fetched


def keys_of_call(keys, calls, c):
    """The lookups of call c alone (markers left out)."""
    plain = [k for k in keys if not hasattr(k, "name")]
    start = sum(n for _, _, n in calls[:c])
    return plain[start:start + calls[c][2]]


def test_kept_tiles_go_stale_without_invalidate_and_not_at_all_by_default(oracle):
    n, T = 256, 64
    announce("out-of-core GEMM: stale tiles are the caller's error only with keep_tiles")
    budget = _budget(T, 40, n, n, n)                 # room for every tile of A and B: nothing is evicted
    for keep in (1, 0):
        A = inputs.int_matrix(1, n, n).pin_memory()
        B = inputs.int_matrix(2, n, n).pin_memory()
        ctx = tg.tgemm_create(0, keep_tiles=keep)
        try:
            C = torch.zeros(n, n).pin_memory()
            tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, budget)
            old = oracle.gemm(A.numpy(), B.numpy())
            assert np.array_equal(C.numpy().astype(np.float64), old)
            A.mul_(-2.0)
            new = oracle.gemm(A.numpy(), B.numpy())
            C.zero_()
            tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, budget)
            st = tg.tgemm_last_stats(ctx)
            if keep:
                assert st["misses"] == 0 and st["h2d_bytes"] == n * n * 4      # only C travelled
                assert np.array_equal(C.numpy().astype(np.float64), old)       # the cached copy of the old A
                tg.tgemm_invalidate(ctx, A)
                C.zero_()
                tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, budget)
                st = tg.tgemm_last_stats(ctx)
                assert st["misses"] == 16 and st["hits"] == 2 * 64 - 16         # A fetched again, B still cached
            assert np.array_equal(C.numpy().astype(np.float64), new)
        finally:
            tg.tgemm_destroy(ctx)


def test_tile_pool_follows_the_budget_down():
    """A context that has run with a large budget gives the memory back when a later call allows less."""
    n, T = 4096, 512
    announce("out-of-core GEMM: the slot pool shrinks with the budget")
    A = inputs.int_matrix(1, n, n).pin_memory()
    B = inputs.int_matrix(2, n, n).pin_memory()
    ctx = tg.tgemm_create(0)
    try:
        frees = []
        for n_ab in (128, 16, 64):
            C = torch.zeros(n, n).pin_memory()
            tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, _budget(T, n_ab, n, n, n))
            assert tg.tgemm_last_stats(ctx)["n_slots"] == n_ab
            if n_ab == 16:
                assert torch.equal(C, A @ B)
            frees.append(torch.cuda.mem_get_info()[0])
        slot = T * T * 4
        assert frees[1] - frees[0] >= (128 - 16) * slot // 2, frees        # memory came back
        assert frees[1] - frees[2] >= (64 - 16) * slot // 2, frees         # and is taken again when allowed
    finally:
        tg.tgemm_destroy(ctx)


def test_error_paths():
    ctx = tg.tgemm_create(0)
    try:
        A = torch.zeros(512, 512).pin_memory()
        B = torch.zeros(512, 512).pin_memory()
        C = torch.zeros(512, 512).pin_memory()
        with pytest.raises(tg.TgemmError) as e:
            tg.tgemm_run(ctx, A, B, C, 512, 512, 512, 128, tg.TGEMM_F32, _budget(128, 8, 512, 512, 512) - 1)
        assert e.value.code == tg.TGEMM_EBUDGET
        with pytest.raises(tg.TgemmError) as e:
            tg.tgemm_run(ctx, A, B, torch.zeros(512, 512), 512, 512, 512, 128, tg.TGEMM_F32, 1 << 30)
        assert e.value.code == tg.TGEMM_EUNPINNED
        C.fill_(2.0)
        tg.tgemm_run(ctx, A, B, C, 512, 512, 512, 128, tg.TGEMM_F32, _budget(128, 8, 512, 512, 512))
        assert torch.equal(C, torch.full((512, 512), 2.0))           # still usable after the errors
    finally:
        tg.tgemm_destroy(ctx)


def _matvec64(Mat, x, block=2048, workers=8):
    """fp64 Mat @ x for a big fp32 host matrix, in row blocks."""
    n = Mat.shape[0]
    out = np.empty(n)

    def work(r):
        out[r:r + block] = Mat[r:r + block].astype(np.float64) @ x

    with ThreadPoolExecutor(workers) as ex:
        list(ex.map(work, range(0, n, block)))
    return out


def test_config3_full_size(oracle):
    """fp32 65536^3, T = 4096, A, B, C in pinned host memory (17.2 GB each), budget 8e9 bytes."""
    n, T, budget = 65536, 4096, 8 * 10 ** 9
    announce("config3 allocate + fill")
    A = torch.empty(n, n, pin_memory=True)
    B = torch.empty(n, n, pin_memory=True)
    C = torch.zeros(n, n, pin_memory=True)
    inputs.fill(A, 1, "uniform", gen_device="cuda")
    inputs.fill(B, 2, "uniform", gen_device="cuda")
    torch.cuda.synchronize()
    ctx = tg.tgemm_create(0, trace=1)
    try:
        announce("config3 run")
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, budget)
        stats = tg.tgemm_last_stats(ctx)
        print("config3 stats", stats, "TFLOP/s", 2.0 * n ** 3 / stats["wall_ms"] / 1e9, flush=True)
        assert stats["n_slots"] == 115 and stats["n_tasks"] == 256 and stats["n_tile_gemms"] == 4096
        # default order: the cache has room for strips of 115 / 16 - 2 = 5 tile columns, so the 16 columns
        # go into four strips of 4; B comes in once and A once per strip, less what survives in the cache
        # across a strip boundary
        assert oracle.auto_strip(115, 16, 16) == 4
        _check_trace(oracle, ctx, n, n, n, T, "strips", 115, strip=4)
        assert stats["misses"] == 1232
        assert stats["h2d_bytes"] == (stats["misses"] + 256) * T * T * 4 and stats["d2h_bytes"] == n * n * 4
    finally:
        tg.tgemm_destroy(ctx)
    An, Bn, Cn = A.numpy(), B.numpy(), C.numpy()
    announce("config3 sampled entries")
    edges = sorted(set([0, n - 1] + [t * T for t in range(1, 16)] + [t * T - 1 for t in range(1, 16)]))
    rr, cc = np.meshgrid(edges, edges, indexing="ij")
    rnd = np.random.default_rng(0)
    rows = np.concatenate([rr.ravel(), rnd.integers(0, n, 4096)])
    cols = np.concatenate([cc.ravel(), rnd.integers(0, n, 4096)])
    # the generator is counter-based: regenerate a few operands entries from (seed, index) alone
    probe = torch.from_numpy(rows[:64] * n + cols[:64])
    assert torch.equal(inputs.uniform_pm1_at(1, probe), A.view(-1)[probe])
    ref = oracle.gemm_samples(An, Bn, rows, cols)
    err = rel_fro(Cn[rows, cols], ref)
    print("config3 sampled rel fro", err, flush=True)
    assert err <= TOL_F32
    announce("config3 Freivalds")
    x = rnd.integers(-1, 2, n).astype(np.float64)
    lhs = _matvec64(Cn, x)
    rhs = _matvec64(An, _matvec64(Bn, x))
    err = rel_fro(lhs, rhs)
    print("config3 Freivalds rel err", err, flush=True)
    assert err <= TOL_F32
    # The same product with small-integer operands: every partial sum is an integer below 2^24, so
    # the result is exact in any order and must equal the fp64 definition bit for bit -- on the
    # sampled entries (tile corners included) and, through Freivalds' check, on every tile.
    announce("config3 integer operands: fill")
    inputs.fill(A, 11, "int", gen_device="cuda")
    inputs.fill(B, 12, "int", gen_device="cuda")
    C.zero_()
    torch.cuda.synchronize()
    ctx = tg.tgemm_create(0)
    try:
        announce("config3 integer operands: run")
        tg.tgemm_run(ctx, A, B, C, n, n, n, T, tg.TGEMM_F32, budget)
    finally:
        tg.tgemm_destroy(ctx)
    announce("config3 integer operands: sampled entries")
    ref = oracle.gemm_samples(An, Bn, rows, cols)
    assert np.array_equal(Cn[rows, cols].astype(np.float64), ref)
    assert np.abs(ref).max() > 100                                  # not a trivially small result
    announce("config3 integer operands: Freivalds")
    lhs = _matvec64(Cn, x)
    rhs = _matvec64(An, _matvec64(Bn, x))
    assert np.array_equal(lhs, rhs)                                  # integers in fp64: exact on both sides


@pytest.mark.parametrize("order,order_name", [(tg.TGEMM_ORDER_ROW_MAJOR, "row_major"), (tg.TGEMM_ORDER_SERPENTINE, "serpentine")])
@pytest.mark.parametrize("M,N,K,T,n_ab,depth", [(1500, 1400, 1300, 256, 20, 4), (640, 640, 640, 128, 8, 8),
                                                (300, 2000, 700, 256, 11, 3), (1280, 2304, 768, 256, 15, 64)])
def test_reservation_station_priority(oracle, M, N, K, T, n_ab, depth, order, order_name):
    """opts.rs_depth: the order in which tasks leave the reservation station, every hit, miss and
    eviction of the trace, and the statistics equal the oracle's station simulation; the values are
    those of the plain product (integer inputs: bit for bit); the priority saves host-link traffic."""
    announce("ooc reservation station", M, N, K, T, n_ab, depth, order_name)
    A = inputs.int_matrix(11, M, K)
    B = inputs.int_matrix(12, K, N)
    C0 = inputs.int_matrix(13, M, N)
    ref = oracle.gemm(A.numpy(), B.numpy(), c_in=C0.numpy())
    misses = {}
    for d in (depth, 1):
        ctx = tg.tgemm_create(0, trace=1, order=order, rs_depth=d)
        try:
            Ap, Bp, Cp = _pinned(A), _pinned(B), _pinned(C0)
            tg.tgemm_run(ctx, Ap, Bp, Cp, M, N, K, T, tg.TGEMM_F32, _budget(T, n_ab, M, N, K))
            assert np.array_equal(Cp.numpy().astype(np.float64), ref)
            stats = tg.tgemm_last_stats(ctx)
            trace = tg.tgemm_trace(ctx)
            left, events, st = oracle.station_simulate(M, N, K, T, stats["n_slots"], order_name, None, d)
            n_j, n_k = -(-N // T), -(-K // T)
            assert [r["task_id"] for r in trace[::n_k]] == left
            assert len(trace) * 2 == len(events)
            for t, rec in enumerate(trace):
                tid = left[t // n_k]
                assert (rec["task_id"], rec["i"], rec["j"], rec["k"]) == (tid, tid // n_j, tid % n_j, t % n_k)
                assert bool(rec["a_hit"]) == events[2 * t][0] and bool(rec["b_hit"]) == events[2 * t + 1][0]
                assert bool(rec["a_evicted"]) == (events[2 * t][1] is not None)
                assert bool(rec["b_evicted"]) == (events[2 * t + 1][1] is not None)
            assert (stats["hits"], stats["misses"], stats["evictions"]) == (st["hits"], st["misses"], st["evictions"])
            assert stats["d2h_bytes"] == M * N * 4
            misses[d] = stats["misses"]
        finally:
            tg.tgemm_destroy(ctx)
    assert misses[depth] <= misses[1]


def test_reservation_station_depth_is_checked():
    for bad in (-1, 65):
        with pytest.raises(tg.TgemmError) as e:
            tg.tgemm_create(0, rs_depth=bad)
        assert e.value.code == tg.TGEMM_EARG
