"""Pins of the plan and tile-cache oracles: the tile counts of section 3.1, partition
invariants, closed forms of LRU behaviour, an independent brute-force LRU."""
import os

import pytest

GOLD = os.path.join(os.path.dirname(__file__), "golden", "tile_counts.txt")


def _golden_rows():
    rows = []
    for line in open(GOLD):
        line = line.strip()
        if line and not line.startswith("#"):
            rows.append(tuple(int(x) for x in line.split()))
    return rows


def test_paper_tile_counts(oracle):
    rows = _golden_rows()
    assert len(rows) == 3
    for n, t, full, edge, ksteps in rows:
        assert oracle.tile_counts(n, t) == (full, edge)
        tasks = oracle.plan_tiles(n, n, n, t)
        assert len(tasks) == full + edge
        n_full = sum(1 for x in tasks if x["r1"] - x["r0"] == t and x["c1"] - x["c0"] == t)
        assert n_full == full
        assert all(x["n_k"] == ksteps for x in tasks)
        assert len(oracle.kstep_ranges(n, t)) == ksteps


@pytest.mark.parametrize("M,N,K,T", [(1000, 1000, 1000, 256), (7, 13, 5, 3), (5, 5, 5, 8), (64, 32, 16, 16),
                                     (1, 1, 1, 1), (10, 3, 7, 1)])
def test_plan_partitions_output(oracle, M, N, K, T):
    tasks = oracle.plan_tiles(M, N, K, T)
    seen = set()
    n_j = -(-N // T)
    for idx, t in enumerate(tasks):
        assert t["id"] == idx == t["i"] * n_j + t["j"]
        assert oracle.decode_task(t["id"], n_j) == (t["i"], t["j"])
        assert 0 < t["r1"] - t["r0"] <= T and 0 < t["c1"] - t["c0"] <= T
        for r in range(t["r0"], t["r1"]):
            for c in range(t["c0"], t["c1"]):
                assert (r, c) not in seen
                seen.add((r, c))
    assert len(seen) == M * N
    ks = oracle.kstep_ranges(K, T)
    assert ks[0][0] == 0 and ks[-1][1] == K
    assert all(a[1] == b[0] for a, b in zip(ks, ks[1:]))
    assert all(0 < b - a <= T for a, b in ks)
    # steps per task (section 3.1): one per tile of the shared dimension, counted without ceil
    assert all(t["n_k"] == len(ks) == sum(1 for k in range(K) if k % T == 0) for t in tasks)


def test_edge_extents_config1(oracle):
    tasks = oracle.plan_tiles(1000, 1000, 1000, 256)
    assert tasks[3]["c1"] - tasks[3]["c0"] == 232 and tasks[15]["r1"] - tasks[15]["r0"] == 232
    assert oracle.kstep_ranges(1000, 256)[-1] == (768, 1000)


def _brute_lru(keys, n):
    order = []  # least recent first
    out = []
    for k in keys:
        if k in order:
            order.remove(k)
            order.append(k)
            out.append((True, None))
        else:
            victim = None
            if len(order) == n:
                victim = order.pop(0)
            order.append(k)
            out.append((False, victim))
    return out


def test_lru_closed_forms(oracle):
    n = 5
    # cyclic sweep over n+1 keys: LRU never hits
    ev, st = oracle.lru_simulate([i % (n + 1) for i in range(60)], n)
    assert st["hits"] == 0 and st["misses"] == 60 and st["evictions"] == 60 - n
    # n keys in n slots: only the compulsory misses
    ev, st = oracle.lru_simulate([i % n for i in range(60)], n)
    assert st == dict(hits=60 - n, misses=n, evictions=0)
    # victim is the least recently *used*, not the first inserted
    ev, _ = oracle.lru_simulate(["a", "b", "c", "a", "d"], 3)
    assert ev[-1] == (False, "b")


def test_lru_vs_brute_force(oracle):
    import random
    rnd = random.Random(11)
    for n in (1, 2, 3, 7):
        keys = [rnd.randrange(10) for _ in range(400)]
        ev, st = oracle.lru_simulate(keys, n)
        assert ev == _brute_lru(keys, n)
        assert st["hits"] + st["misses"] == len(keys)


def test_lru_invalidate(oracle):
    """Dropping a changed matrix's tiles: they miss at their next lookup, into the slots they freed (no
    eviction); the other matrices' tiles stay and keep their recency; the marker itself is no event.
    Then random sequences against an independent list-based LRU that handles the marker itself."""
    keys = [("A", 0), ("B", 0), ("A", 1), ("B", 1), oracle.Invalidate("A"), ("B", 0), ("A", 0), ("A", 1), ("C", 0), ("B", 1)]
    ev, st = oracle.lru_simulate(keys, 4)
    assert ev == [(False, None)] * 4 + [(True, None), (False, None), (False, None), (False, ("B", 1)), (False, ("B", 0))]
    assert st == dict(hits=1, misses=8, evictions=2)
    # nothing cached of that matrix: the marker changes nothing
    assert oracle.lru_simulate([("B", 0), oracle.Invalidate("A"), ("B", 0)], 2)[1] == dict(hits=1, misses=1, evictions=0)
    import random
    rnd = random.Random(3)
    for n in (2, 3, 6):
        keys = []
        for _ in range(500):
            keys.append(oracle.Invalidate(rnd.choice("AB")) if rnd.random() < 0.05 else (rnd.choice("AB"), rnd.randrange(5)))
        order, want = [], []
        for k in keys:
            if isinstance(k, oracle.Invalidate):
                order = [c for c in order if c[0] != k.name]
                continue
            if k in order:
                order.remove(k)
                order.append(k)
                want.append((True, None))
            else:
                victim = order.pop(0) if len(order) == n else None
                order.append(k)
                want.append((False, victim))
        ev, st = oracle.lru_simulate(keys, n)
        assert ev == want and st["hits"] + st["misses"] == len(want)


def test_access_sequence_structure(oracle):
    seq = oracle.tgemm_access_sequence(5, 7, 9, 2, order="row_major")
    n_i, n_j, n_k = 3, 4, 5
    assert len(seq) == 2 * n_i * n_j * n_k
    assert seq[0] == ("A", 0, 0, 0, 0) and seq[1] == ("B", 0, 0, 0, 0)
    assert seq[2 * n_k] == ("A", 0, 0, 1, 0) and seq[2 * n_k + 1] == ("B", 0, 1, 1, 0)
    serp = oracle.tgemm_access_sequence(5, 7, 9, 2, order="serpentine")
    tids = [s[3] for s in serp[::2 * n_k]]
    assert tids == [0, 1, 2, 3, 7, 6, 5, 4, 8, 9, 10, 11]
    assert sorted(s[:3] for s in serp) == sorted(s[:3] for s in seq)


def test_row_major_reuse_closed_form(oracle):
    """Row-major order, cache smaller than one sweep of B: every B lookup misses, A misses
    once per (i, k) -- the redundant-transfer pattern section 3.4 describes."""
    n_i = n_j = n_k = 6
    T = 4
    seq = oracle.tgemm_access_sequence(n_i * T, n_j * T, n_k * T, T, order="row_major")
    slots = 2 * n_k + 3          # holds a row panel of A and a bit more, far less than all of B
    ev, st = oracle.lru_simulate([s[:3] for s in seq], slots)
    a_miss = sum(1 for s, e in zip(seq, ev) if s[0] == "A" and not e[0])
    b_miss = sum(1 for s, e in zip(seq, ev) if s[0] == "B" and not e[0])
    assert a_miss == n_i * n_k
    assert b_miss == n_i * n_j * n_k
    # everything fits: compulsory misses only
    ev, st = oracle.lru_simulate([s[:3] for s in seq], n_i * n_k + n_k * n_j)
    assert st["misses"] == n_i * n_k + n_k * n_j and st["evictions"] == 0


def test_strips_order_written_out(oracle):
    """3 x 5 task grid, strips two tile columns wide: the strips go left to right, the rows
    down, up, down, and the columns of a strip left to right in every row."""
    got = oracle.task_order(3, 5, "strips", strip=2)
    assert got == [0, 1, 5, 6, 10, 11,   12, 13, 7, 8, 2, 3,   4, 9, 14]
    assert oracle.task_order(3, 5, "strips", strip=5) == oracle.task_order(3, 5, "row_major")
    assert oracle.task_order(4, 1, "strips", strip=1) == [0, 1, 2, 3]
    for n_i, n_j, w in [(1, 1, 1), (4, 7, 3), (6, 6, 6), (5, 2, 9)]:
        assert sorted(oracle.task_order(n_i, n_j, "strips", strip=w)) == list(range(n_i * n_j))
    with pytest.raises(ValueError):
        oracle.task_order(3, 5, "strips")


def test_strips_traffic_closed_form(oracle):
    """With (w + 2) * n_k slots a strip's B tiles are fetched once and never evicted while the
    strip runs, and each A row panel once per strip, except the panel shared by two consecutive
    strips (the last row of one is the first of the next).  One slot fewer per k-step than
    (w + 1) * n_k and the strip's B tiles are thrown out at every row change."""
    n_i, n_j, n_k, T, w = 5, 6, 4, 2, 2
    n_strips = n_j // w
    seq = oracle.tgemm_access_sequence(n_i * T, n_j * T, n_k * T, T, order="strips", strip=w)
    assert oracle.auto_strip((w + 2) * n_k, n_k, n_j) == w
    # the automatic width: the fewest strips that the cache allows, the columns shared out evenly
    # (16 columns, room for 5: four strips of 4, not 5 + 5 + 5 + 1; both cost the same 1232 misses)
    assert oracle.auto_strip(115, 16, 16) == 4
    for slots, nk, nj in [(115, 16, 16), (40, 8, 8), (64, 4, 9), (200, 16, 16), (8, 16, 16), (1000, 2, 7), (24, 4, 1)]:
        widest = min(nj, max(1, slots // nk - 2))
        got = oracle.auto_strip(slots, nk, nj)
        assert 1 <= got <= widest
        assert -(-nj // got) == -(-nj // widest)                   # as few strips as the widest would need
        assert got == 1 or -(-nj // (got - 1)) > -(-nj // widest)    # and no narrower width does that
    misses = {}
    for width in (4, 5):
        big = oracle.tgemm_access_sequence(16, 16, 16, 1, order="strips", strip=width)
        misses[width] = oracle.lru_simulate([s[:3] for s in big], 115)[1]["misses"]
    assert misses[4] == misses[5] == 1232
    ev, st = oracle.lru_simulate([s[:3] for s in seq], (w + 2) * n_k)
    a_miss = sum(1 for s, e in zip(seq, ev) if s[0] == "A" and not e[0])
    b_miss = sum(1 for s, e in zip(seq, ev) if s[0] == "B" and not e[0])
    assert b_miss == n_k * n_j
    assert a_miss == n_strips * n_i * n_k - (n_strips - 1) * n_k
    ev, tight = oracle.lru_simulate([s[:3] for s in seq], (w + 1) * n_k - 1)
    assert tight["misses"] > 2 * st["misses"]
    # serpentine on the same cache refetches far more
    serp = oracle.tgemm_access_sequence(n_i * T, n_j * T, n_k * T, T, order="serpentine")
    _, st2 = oracle.lru_simulate([s[:3] for s in serp], (w + 2) * n_k)
    assert st2["misses"] > st["misses"]


# ---- reservation station with locality priority --------------------------------------------------------

def _keys(oracle, M, N, K, T, order, strip=None):
    return [(m, a, b) for (m, a, b, _, _) in oracle.tgemm_access_sequence(M, N, K, T, order, strip)]


def test_station_of_depth_one_is_queue_order(oracle):
    for (M, N, K, T, slots, order, strip) in [(12, 12, 8, 4, 5, "row_major", None), (20, 12, 8, 4, 7, "serpentine", None),
                                              (16, 24, 12, 4, 9, "strips", 2), (7, 13, 5, 3, 4, "row_major", None)]:
        left, ev, st = oracle.station_simulate(M, N, K, T, slots, order, strip, depth=1)
        n_i, n_j = -(-M // T), -(-N // T)
        assert left == oracle.task_order(n_i, n_j, order, strip)
        ev0, st0 = oracle.lru_simulate(_keys(oracle, M, N, K, T, order, strip), slots)
        assert ev == ev0 and st == st0


def test_station_worked_example(oracle):
    # 2 x 2 tasks, one k-step, two cache slots, station of two, row-major queue 0 1 2 3
    # (task t = (i, j) = (t / 2, t % 2) looks up A_i then B_j):
    #   station {0,1}: nothing cached, 0 leaves (first in).  A0 miss, B0 miss.      cache A0 B0
    #   station {1,2}: task 1 has A0, task 2 has B0: a tie, 1 leaves.  A0 hit, B1 miss evicts B0.  cache A0 B1
    #   station {2,3}: task 2 = (1,0) has nothing, task 3 = (1,1) has B1: 3 leaves.  A1 miss evicts A0, B1 hit.  cache B1 A1
    #   station {2}:   A1 hit, B0 miss.
    # 5 misses; plain queue order has 6 (task 2 evicts B1 before task 3 wants it).
    left, ev, st = oracle.station_simulate(8, 8, 4, 4, 2, "row_major", None, depth=2)
    assert left == [0, 1, 3, 2]
    assert [e[0] for e in ev] == [False, False, True, False, False, True, True, False]
    assert [e[1] for e in ev] == [None, None, None, ("B", 0, 0), ("A", 0, 0), None, None, ("B", 0, 1)]
    assert st == dict(hits=3, misses=5, evictions=3)
    assert oracle.lru_simulate(_keys(oracle, 8, 8, 4, 4, "row_major"), 2)[1]["misses"] == 6


def test_station_leaves_by_priority(oracle):
    """The defining property, checked with independent machinery: the station is always the earliest
    `depth` tasks of the queue that have not left; the one that leaves has the most input tiles in the
    cache as lru_simulate leaves it after the lookups so far, and among equals it is the earliest."""
    import random
    rnd = random.Random(5)
    reordered = 0
    for case in range(30):
        n_i, n_j, n_k = rnd.randint(1, 5), rnd.randint(1, 5), rnd.randint(1, 3)
        T, slots, depth = 4, rnd.randint(2, 12), rnd.randint(1, 6)
        order = rnd.choice(["row_major", "serpentine"])
        M, N, K = n_i * T - rnd.randint(0, 3), n_j * T - rnd.randint(0, 3), n_k * T - rnd.randint(0, 3)
        left, ev, st = oracle.station_simulate(M, N, K, T, slots, order, None, depth)
        queue = oracle.task_order(n_i, n_j, order)
        assert sorted(left) == sorted(queue) and len(ev) == 2 * n_k * len(queue)
        reordered += left != queue
        done, keys = [], []
        for tid in left:
            waiting = [t for t in queue if t not in done][:depth]
            # cache content now: replay the lookups so far
            resident = set()
            for key, (hit, victim) in zip(keys, oracle.lru_simulate(keys, slots)[0]):
                resident.add(key)
                resident.discard(victim)
            score = lambda t: sum((("A", t // n_j, k) in resident) + (("B", k, t % n_j) in resident) for k in range(n_k))
            best = max(score(t) for t in waiting)
            assert tid == [t for t in waiting if score(t) == best][0], (case, tid, waiting)
            done.append(tid)
            for k in range(n_k):
                keys += [("A", tid // n_j, k), ("B", k, tid % n_j)]
        assert ev == oracle.lru_simulate(keys, slots)[0]
    assert reordered >= 5      # the priority did change the order in a fair share of the cases


# ---- replacement by next use on the cyclic sweep of an out-of-core training step --------------------

def _min_misses(seq, n_slots):
    """Fewest misses any replacement policy can reach on the finite sequence, by exhaustive search
    over every eviction choice (memoised on position and cache content)."""
    from functools import lru_cache

    @lru_cache(maxsize=None)
    def go(t, cache):
        if t == len(seq):
            return 0
        key = seq[t]
        if key in cache:
            return go(t + 1, cache)
        if len(cache) < n_slots:
            return 1 + go(t + 1, cache | {key})
        return 1 + min(go(t + 1, (cache - {v}) | {key}) for v in cache)

    return go(0, frozenset())


def test_next_use_is_optimal_on_every_small_sweep(oracle):
    """Evicting the key needed furthest ahead is Belady's rule, which reaches the minimum number of
    misses on every prefix of a sequence; so on m repetitions of a sweep the simulation must meet the
    exhaustive-search minimum exactly.  All sweeps of length <= 5 over <= 4 keys, 1..3 slots."""
    import itertools
    checked = 0
    for n_keys in (2, 3, 4):
        for length in range(n_keys, 6):
            for sweep in itertools.product(range(n_keys), repeat=length):
                if len(set(sweep)) != n_keys or sweep[0] != 0:
                    continue
                for n_slots in range(1, n_keys + 1):
                    for m in (1, 2, 3):
                        _, st = oracle.next_use_simulate([[k] for k in sweep], n_slots, n_sweeps=m)
                        assert st["misses"] == _min_misses(sweep * m, n_slots), (sweep, n_slots, m)
                        assert st["hits"] + st["misses"] == m * length
                        checked += 1
    assert checked > 1500


def test_next_use_worked_example_and_closed_forms(oracle):
    # sweep a b c, two slots: c evicts b (needed two lookups ahead, a one); a hits; b evicts a; c hits;
    # a evicts c; b hits: from then on every other lookup misses, the rate (n - s) / (n - 1) of a
    # cyclic sweep of n keys through s slots
    ev, st = oracle.next_use_simulate([["a"], ["b"], ["c"]], 2, n_sweeps=3)
    assert ev == [(False, None), (False, None), (False, "b"), (True, None), (False, "a"), (True, None),
                  (False, "c"), (True, None), (False, "b")]
    assert st == dict(hits=3, misses=6, evictions=4)
    for n, s in ((5, 2), (7, 3), (9, 8), (6, 5)):
        m = 4 * (n - 1)
        _, st = oracle.next_use_simulate([[k] for k in range(n)], s, n_sweeps=m + 1)
        _, st1 = oracle.next_use_simulate([[k] for k in range(n)], s, n_sweeps=1)
        assert st["misses"] - st1["misses"] == m * n * (n - s) // (n - 1), (n, s)      # steady state, whole cycles
    # room for every key: compulsory misses only, like LRU; one slot: every lookup of a changing key misses
    seq = [[0], [1], [2], [1], [0]]
    _, st = oracle.next_use_simulate(seq, 3, n_sweeps=4)
    assert st == dict(hits=17, misses=3, evictions=0)
    _, st = oracle.next_use_simulate(seq, 1, n_sweeps=2)
    assert st["misses"] == 9 and st["hits"] == 1                                       # 0 ... 0 | 0: the wrap-around repeats key 0
    # a sweep that runs forward and then back (the shape of a training step): the tile used last in the
    # forward half is the first of the backward half, and LRU -- which must agree whenever the victim is
    # forced -- never does better
    fb = [[k] for k in range(6)] + [[k] for k in range(5, -1, -1)]
    for s in range(1, 7):
        _, st = oracle.next_use_simulate(fb, s, n_sweeps=3)
        _, lru = oracle.lru_simulate([g[0] for g in fb] * 3, s)
        assert st["misses"] <= lru["misses"], s
        if s in (1, 6):
            assert st == lru


def test_next_use_against_explicit_scan_with_groups(oracle):
    """The same rule with independent machinery: the future is written out as a list, every resident
    key's next occurrence is found by scanning it, the current group's keys are passed over; random
    sweeps with repeated keys and ragged groups.  Also: no victim ever belongs to the group being
    assembled, and every victim was resident."""
    import random
    rnd = random.Random(5)
    for case in range(40):
        n_keys = rnd.randint(3, 9)
        groups = []
        for _ in range(rnd.randint(2, 6)):
            groups.append(rnd.sample(range(n_keys), rnd.randint(1, min(3, n_keys))))
        biggest = max(len(g) for g in groups)
        n_slots = rnd.randint(biggest + 1, n_keys + 1)     # one slot beyond the largest group: a victim always exists
        n_sweeps = 3
        events, st = oracle.next_use_simulate(groups, n_slots, n_sweeps)
        flat = [k for g in groups for k in g]
        owner = [gi for gi, g in enumerate(groups) for _ in g]
        future = flat * (n_sweeps + 2)
        cache, t = [], 0
        for sweep in range(n_sweeps):
            for pos, key in enumerate(flat):
                hit, victim = events[t]
                assert hit == (key in cache), (case, t)
                if not hit:
                    if len(cache) >= n_slots:
                        ahead = {}
                        for cand in cache:
                            if cand in groups[owner[pos]]:
                                continue
                            ahead[cand] = future.index(cand, t + 1) - t
                        want = max(ahead, key=lambda c: ahead[c])
                        assert victim == want and victim in cache and victim not in groups[owner[pos]], (case, t)
                        cache.remove(victim)
                    else:
                        assert victim is None
                    cache.append(key)
                t += 1
        assert t == len(events) and st["misses"] == sum(1 for h, _ in events if not h)


def test_mlp_sweep_written_out(oracle):
    # 4 -> 6 -> 2 with T = 2: W_1 is 2 x 3 tiles, W_2 is 3 x 1
    g = oracle.mlp_sweep_groups([4, 6, 2], 2)
    assert g == [[(1, 0, 0), (1, 1, 0)], [(1, 0, 1), (1, 1, 1)], [(1, 0, 2), (1, 1, 2)],      # forward W_1 by tile columns
                 [(2, 0, 0), (2, 1, 0), (2, 2, 0)],                                           # forward W_2
                 [(2, 0, 0)], [(2, 1, 0)], [(2, 2, 0)],                                       # backward W_2 by tile rows
                 [(1, 0, 0), (1, 0, 1), (1, 0, 2)], [(1, 1, 0), (1, 1, 1), (1, 1, 2)]]        # backward W_1
    # without the update nothing needs W_1 in the backward pass
    assert oracle.mlp_sweep_groups([4, 6, 2], 2, update=False) == g[:7]
    # ragged sizes round up; every tile is looked up exactly twice per training step
    for dims, T in (([5, 7, 3], 2), ([8192, 32768, 32768, 262144], 2048), ([10, 10], 3)):
        g = oracle.mlp_sweep_groups(dims, T)
        flat = [k for grp in g for k in grp]
        tiles = sum(-(-dims[l] // T) * -(-dims[l + 1] // T) for l in range(len(dims) - 1))
        assert len(flat) == 2 * tiles and len(set(flat)) == tiles
        assert all(flat.count(k) == 2 for k in set(flat)) if tiles < 100 else True
