"""The weight-tile cache of the out-of-core MLP step (section 3.4 of the paper: a hit uses the cached
tile, a miss fetches it from host memory), lookup by lookup, through the C ABI (mlp_trace).

With tgemm_opts.exact_replacement the victim of every miss is the cached tile whose next use in the
step's fixed sweep lies furthest ahead: a pure function of sizes, tile size and slot count, so the
trace must equal oracle.next_use_simulate on oracle.mlp_sweep_groups record by record (lookup order,
hit / miss, displaced tile) and the statistics and host-link bytes must follow from it.

In the default mode the library may prefer, among the tiles whose next use is at least half as far
away as the furthest, one that has no read or write-back in flight (which one depends on timing).
There the lookup order is still unique and is compared; the rest is checked for validity by
replaying the trace: a hit is reported exactly when the tile is resident, a displaced tile was
resident and does not belong to the launch group being assembled, its next use is at least half the
furthest one's, slots are consistent; and the misses lie between the oracle's (which are minimal) and
those of strict LRU."""
import numpy as np
import pytest
import torch

from gpu_util import announce
from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs

pytestmark = pytest.mark.gpu


def _workspace_bytes(dims, batch, es, T):
    L = len(dims) - 1
    total = batch * 4 + batch * dims[L] * 4
    for l in range(1, L + 1):
        total += batch * dims[l] * es * (2 if l < L else 1)
    return total + 96 * max(-(-d // T) for d in dims) * 8


def _tile_bytes(dims, T, es, key):
    l, r, c = key
    return min(T, dims[l - 1] - r * T) * min(T, dims[l] - c * T) * es


def _run_steps(dims, batch, T, n_slots, dtype, n_steps, **opts):
    tdt = torch.bfloat16 if dtype == tg.TGEMM_BF16 else torch.float32
    es = 2 if dtype == tg.TGEMM_BF16 else 4
    X = inputs.normal_matrix(1, batch, dims[0]).to(tdt).cuda()
    y = inputs.labels(5, batch, dims[-1]).cuda()
    Wp = [inputs.normal_matrix(10 + l, dims[l], dims[l + 1], std=0.05).to(tdt).pin_memory() for l in range(len(dims) - 1)]
    torch.cuda.synchronize()
    budget = _workspace_bytes(dims, batch, es, T) + n_slots * T * T * es
    ctx = tg.tgemm_create(0, trace=1, **opts)
    steps = []
    try:
        mlp = tg.mlp_create(ctx, dims, Wp, dtype, T, hbm_budget=budget)
        for _ in range(n_steps):
            tg.mlp_step(mlp, X, y, batch, 0.01)
            st = tg.tgemm_last_stats(ctx)
            steps.append((tg.mlp_trace(mlp), st))
        tg.tgemm_sync(ctx)
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)
    return steps


CASES = [([512, 1024, 768, 2000], 384, 256, 0.4, tg.TGEMM_F32), ([300, 700, 900, 1250], 200, 128, 0.55, tg.TGEMM_BF16),
         ([640, 640, 640], 128, 64, 0.3, tg.TGEMM_BF16), ([450, 1000], 64, 100, 0.5, tg.TGEMM_F32)]


def _slots_for(dims, T, frac):
    cd = lambda a: -(-a // T)
    n_tiles = sum(cd(dims[l]) * cd(dims[l + 1]) for l in range(len(dims) - 1))
    return n_tiles, max(int(frac * n_tiles), 2 * max(cd(d) for d in dims) + 2)


@pytest.mark.parametrize("deferred", [0, 1])
@pytest.mark.parametrize("dims,batch,T,frac,dtype", CASES)
def test_exact_replacement_equals_the_oracle_record_by_record(oracle, dims, batch, T, frac, dtype, deferred):
    announce("mlp cache trace, exact replacement", dims, batch, T, frac, dtype, "deferred" if deferred else "synchronous")
    n_tiles, n_slots = _slots_for(dims, T, frac)
    es = 2 if dtype == tg.TGEMM_BF16 else 4
    n_steps = 3
    steps = _run_steps(dims, batch, T, n_slots, dtype, n_steps, exact_replacement=1, deferred_writeback=deferred)
    groups = oracle.mlp_sweep_groups(dims, T)
    flat = [k for g in groups for k in g]
    events, total = oracle.next_use_simulate(groups, n_slots, n_steps)
    t = 0
    for s, (trace, st) in enumerate(steps):
        assert st["n_slots"] == n_slots and len(trace) == len(flat) == 2 * n_tiles
        misses = hits = evictions = h2d = 0
        for rec, key in zip(trace, flat):
            assert (rec["layer"], rec["r"], rec["c"]) == key, (s, t)
            hit, victim = events[t]
            assert bool(rec["hit"]) == hit, (s, t, key)
            got_victim = None if rec["ev_layer"] < 0 else (rec["ev_layer"], rec["ev_r"], rec["ev_c"])
            assert got_victim == victim, (s, t, key, got_victim, victim)
            hits += hit
            misses += not hit
            evictions += victim is not None
            h2d += 0 if hit else _tile_bytes(dims, T, es, key)
            t += 1
        assert (st["hits"], st["misses"], st["evictions"]) == (hits, misses, evictions), s
        assert st["h2d_bytes"] == h2d and st["d2h_bytes"] == sum(dims[l] * dims[l + 1] for l in range(len(dims) - 1)) * es
        # launch groups: the backward half has the same group structure as the oracle's sweep
        ids = [rec["group"] for rec in trace]
        bounds = np.cumsum([len(g) for g in groups])[:-1]
        assert all(ids[b - 1] != ids[b] for b in bounds) and len(set(ids)) == len(groups)
    assert t == len(events)
    assert sum(st["misses"] for _, st in steps) == total["misses"]


def replay_trace(oracle, dims, T, n_slots, calls):
    """Replays the lookups of successive mlp_* calls on one object (from its creation on, `calls` = one
    trace per call) against the rules every replacement mode must keep.  Returns the number of misses.
    The launch groups come from the records' own group ids; next uses are counted along the fixed sweep
    of a training step from the sweep position of the lookup itself."""
    groups = oracle.mlp_sweep_groups(dims, T)
    flat = [k for g in groups for k in g]
    period = len(flat)
    where = {}
    for pos, key in enumerate(flat):
        where.setdefault(key, []).append(pos)
    resident = {}           # key -> slot
    n_miss = 0
    for trace in calls:
        members = {}
        for rec in trace:
            members.setdefault(rec["group"], set()).add((rec["layer"], rec["r"], rec["c"]))
        for t, rec in enumerate(trace):
            key = (rec["layer"], rec["r"], rec["c"])
            pos = where[key][1 if rec["backward"] else 0]
            ahead = lambda k: min((u - pos - 1) % period for u in where[k])
            assert bool(rec["hit"]) == (key in resident), (t, key)
            if rec["hit"]:
                assert resident[key] == rec["slot"] and rec["ev_layer"] == -1
                continue
            n_miss += 1
            if rec["ev_layer"] >= 0:
                victim = (rec["ev_layer"], rec["ev_r"], rec["ev_c"])
                assert len(resident) == n_slots, "eviction before the cache is full"
                assert victim in resident and resident[victim] == rec["slot"], (t, victim)
                current = members[rec["group"]]
                assert victim not in current, (t, victim)
                furthest = max(ahead(k) for k in resident if k not in current)
                assert 2 * ahead(victim) >= furthest, (t, victim, ahead(victim), furthest)
                del resident[victim]
            else:
                assert len(resident) < n_slots and rec["slot"] not in resident.values()
            resident[key] = rec["slot"]
            assert 0 <= rec["slot"] < n_slots
    return n_miss


@pytest.mark.parametrize("dims,batch,T,frac,dtype", CASES)
def test_default_replacement_trace_is_valid(oracle, dims, batch, T, frac, dtype):
    announce("mlp cache trace, default replacement", dims, batch, T, frac, dtype)
    n_tiles, n_slots = _slots_for(dims, T, frac)
    n_steps = 3
    steps = _run_steps(dims, batch, T, n_slots, dtype, n_steps, deferred_writeback=1)
    groups = oracle.mlp_sweep_groups(dims, T)
    flat = [k for g in groups for k in g]
    for trace, _ in steps:                                           # the lookup order is unique
        assert [(r["layer"], r["r"], r["c"]) for r in trace] == flat
        assert [r["backward"] for r in trace] == [0] * (len(flat) // 2) + [1] * (len(flat) // 2)
    n_miss = replay_trace(oracle, dims, T, n_slots, [trace for trace, _ in steps])
    assert n_miss == sum(st["misses"] for _, st in steps)
    _, best = oracle.next_use_simulate(groups, n_slots, n_steps)
    _, lru = oracle.lru_simulate([k for g in groups for k in g] * n_steps, n_slots)
    print("misses", n_miss, "furthest-next-use", best["misses"], "strict LRU", lru["misses"], flush=True)
    assert best["misses"] <= n_miss <= lru["misses"]


def test_exact_and_default_replacement_give_the_same_weights():
    """Which tile leaves the cache must not change a bit of the result."""
    dims, batch, T, dtype = [300, 700, 900, 1250], 200, 128, tg.TGEMM_BF16
    announce("mlp cache: results do not depend on the replacement mode")
    _, n_slots = _slots_for(dims, T, 0.45)
    out = []
    for exact in (0, 1):
        X = inputs.normal_matrix(1, batch, dims[0]).to(torch.bfloat16).cuda()
        y = inputs.labels(5, batch, dims[-1]).cuda()
        Wp = [inputs.normal_matrix(10 + l, dims[l], dims[l + 1], std=0.05).to(torch.bfloat16).pin_memory() for l in range(3)]
        torch.cuda.synchronize()
        ctx = tg.tgemm_create(0, exact_replacement=exact)
        try:
            mlp = tg.mlp_create(ctx, dims, Wp, dtype, T, hbm_budget=_workspace_bytes(dims, batch, 2, T) + n_slots * T * T * 2)
            losses = [tg.mlp_step(mlp, X, y, batch, 0.5) for _ in range(3)]
            tg.mlp_destroy(mlp)
        finally:
            tg.tgemm_destroy(ctx)
        out.append((losses, [w.clone() for w in Wp]))
    assert out[0][0] == out[1][0]
    for a, b in zip(out[0][1], out[1][1]):
        assert torch.equal(a, b)
