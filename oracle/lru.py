"""L1 tile cache oracle (test infrastructure only).

Section 3.4: a tile already present in the GPU's own memory (the L1 tile
cache) is used directly; a tile absent from it is fetched from host memory.
Algorithm 1 looks up A[i,k] then B[k,j] for every k-step of a task.  The
paper does not name the eviction rule; the reading taken is strict LRU with
a touch on every lookup.  On one GPU there is no second-level (peer) cache.

The weight-tile cache of the out-of-core MLP step sees a lookup sequence that repeats every step
(mlp_sweep_groups), so the next use of every resident tile is known; next_use_simulate is the
replacement rule "evict the resident tile whose next use lies furthest ahead" on such a cyclic
sequence, with the tiles of the launch being assembled protected from eviction.
"""
from collections import OrderedDict

from .plan import _ceil_div


def task_order(n_i, n_j, order, strip=None):
    """Task ids in issue order.  'row_major': i then j ascending.  'serpentine': j ascends on even
    tile rows and descends on odd ones.  'strips': column strips `strip` tile columns wide, left
    to right; the tile rows ascend in even strips and descend in odd ones; the strip's columns
    ascend inside every tile row."""
    if order == "strips":
        if strip is None or strip < 1:
            raise ValueError("strip width")
        ids = []
        for s, j0 in enumerate(range(0, n_j, strip)):
            rows = range(n_i) if s % 2 == 0 else range(n_i - 1, -1, -1)
            for i in rows:
                ids.extend(i * n_j + j for j in range(j0, min(n_j, j0 + strip)))
        return ids
    if order not in ("row_major", "serpentine"):
        raise ValueError(order)
    ids = []
    for i in range(n_i):
        js = range(n_j)
        if order == "serpentine" and i % 2 == 1:
            js = range(n_j - 1, -1, -1)
        ids.extend(i * n_j + j for j in js)
    return ids


def auto_strip(n_slots, n_k, n_j):
    """Strip width for the 'strips' order from the slot count.  The widest strip is the one whose B
    tiles and two row panels of A (n_k tiles per tile column / row) fit in the cache together -- two,
    because under strict LRU the previous row panel outlives the strip's oldest B column.  The tile
    columns are shared out evenly over the fewest strips of at most that width (the paper leaves the
    order of the tasks open, section 3.4; a narrow strip left over at the end would fetch a whole row
    panel of A per task for one column of products)."""
    widest = min(max(1, n_j), max(1, n_slots // n_k - 2))
    n_strips = -(-n_j // widest)
    return max(1, -(-n_j // n_strips)) if n_strips > 0 else 1


def tgemm_access_sequence(M, N, K, T, order="serpentine", strip=None):
    """Tile lookups of one tiled GEMM in issue order: for every task, k ascending,
    the A tile then the B tile.  Each entry is (matrix, tile row, tile col, task id, k)."""
    n_i, n_j, n_k = _ceil_div(M, T), _ceil_div(N, T), _ceil_div(K, T)
    seq = []
    for tid in task_order(n_i, n_j, order, strip):
        i, j = tid // n_j, tid % n_j
        for k in range(n_k):
            seq.append(("A", i, k, tid, k))
            seq.append(("B", k, j, tid, k))
    return seq


class Invalidate:
    """Marker inside a lookup sequence: the caller has changed host matrix `name`, so every cached tile
    of it (every key whose first component equals `name`) is dropped and its slot is free again.
    Section 3.4 keeps tiles cached for reuse; a cached copy of a matrix that has since changed must not
    be used.  The marker is no lookup: it produces no event and counts in no statistic."""

    def __init__(self, name):
        self.name = name


class _Lru:
    """Strict LRU over hashable keys with `n_slots` entries; a lookup touches the key."""

    def __init__(self, n_slots):
        if n_slots < 1:
            raise ValueError("need at least one slot")
        self.n_slots = n_slots
        self.cache = OrderedDict()
        self.hits = self.misses = self.evictions = 0

    def __contains__(self, key):
        return key in self.cache

    def lookup(self, key):
        """Returns (hit, evicted_key_or_None)."""
        cache, n_slots = self.cache, self.n_slots
        if key in cache:
            cache.move_to_end(key)
            self.hits += 1
            return (True, None)
        self.misses += 1
        victim = None
        if len(cache) >= n_slots:
            victim, _ = cache.popitem(last=False)
            self.evictions += 1
        cache[key] = True
        return (False, victim)

    def drop(self, name):
        for key in [k for k in self.cache if k[0] == name]:
            del self.cache[key]

    def stats(self):
        return dict(hits=self.hits, misses=self.misses, evictions=self.evictions)


def lru_simulate(keys, n_slots):
    """Runs strict LRU over hashable keys.  Returns (events, stats); events[t] =
    (hit, evicted_key_or_None) for the t-th lookup.  Invalidate markers among the keys drop a
    matrix's tiles and produce no event."""
    lru = _Lru(n_slots)
    events = []
    for key in keys:
        if isinstance(key, Invalidate):
            lru.drop(key.name)
        else:
            events.append(lru.lookup(key))
    return events, lru.stats()


def station_simulate(M, N, K, T, n_slots, order="row_major", strip=None, depth=1):
    """The tile lookups of one tiled GEMM when tasks pass through a reservation station (section 3.2
    of the paper: the buffer between the task queue and the streams, on which the runtime schedules
    by priority).  The paper does not define the priority; the reading taken is locality: the station
    holds up to `depth` tasks taken from the queue in issue order, and whenever a stream asks for
    work the task with the most input tiles (A_ik and B_kj over all k) in the tile cache at that
    moment leaves first, ties going to the task that entered the station first; the station is then
    topped up from the queue.  depth = 1 is plain queue order.  The cache is strict LRU over the
    lookups of the tasks in the order they leave (k ascending, A tile then B tile).

    Returns (task ids in the order they left the station, events as lru_simulate gives them, stats)."""
    if depth < 1:
        raise ValueError("station depth")
    n_i, n_j, n_k = _ceil_div(M, T), _ceil_div(N, T), _ceil_div(K, T)
    queue = list(task_order(n_i, n_j, order, strip))
    station, left = [], []
    lru = _Lru(n_slots)
    events = []
    while queue or station:
        while queue and len(station) < depth:
            station.append(queue.pop(0))
        best, best_score = 0, -1
        for pos, tid in enumerate(station):
            ti, tj = divmod(tid, n_j)
            score = sum((("A", ti, k) in lru) + (("B", k, tj) in lru) for k in range(n_k))
            if score > best_score:          # strictly greater: the earlier entry keeps a tie
                best, best_score = pos, score
        tid = station.pop(best)
        left.append(tid)
        ti, tj = divmod(tid, n_j)
        for k in range(n_k):
            events.append(lru.lookup(("A", ti, k)))
            events.append(lru.lookup(("B", k, tj)))
    return left, events, lru.stats()


def mlp_sweep_groups(dims, T, update=True):
    """The weight-tile lookups of one out-of-core training step, as a list of launch groups (each a
    list of keys (layer, tile row, tile col), layer = 1..L).  Forward: layers ascending, one group
    per tile COLUMN of W_l holding the column's tiles by ascending tile row (the k-steps of the
    product A_{l-1} W_l).  Backward: layers descending, one group per tile ROW of W_l holding the
    row's tiles by ascending tile column (they serve D_l W_l^T and then take the update).  Without
    update and with a single use for W_1 (no error is propagated below the first layer) the first
    layer has no backward lookups."""
    L = len(dims) - 1
    groups = []
    for l in range(1, L + 1):
        n_r, n_c = _ceil_div(dims[l - 1], T), _ceil_div(dims[l], T)
        for c in range(n_c):
            groups.append([(l, r, c) for r in range(n_r)])
    for l in range(L, 0, -1):
        if l == 1 and not update:
            continue
        n_r, n_c = _ceil_div(dims[l - 1], T), _ceil_div(dims[l], T)
        for r in range(n_r):
            groups.append([(l, r, c) for c in range(n_c)])
    return groups


def next_use_simulate(groups, n_slots, n_sweeps=1):
    """Replacement by next use on a cyclic lookup sequence.

    groups   the lookups of one sweep as a list of groups of hashable keys; the sweep repeats
             forever, and `n_sweeps` of it are simulated starting from an empty cache.
    On a miss with the cache full, the victim is the resident key, outside the current group, whose
    next lookup (counted from the current position along the endlessly repeated sweep) lies
    furthest ahead; a key that never occurs again would be infinitely far, but in a cyclic sweep
    every key does.  Two distinct keys cannot tie: they never share a position.

    Returns (events, stats) like lru_simulate: events[t] = (hit, evicted_key_or_None)."""
    if n_slots < 1:
        raise ValueError("need at least one slot")
    flat = [key for g in groups for key in g]
    group_of = [gi for gi, g in enumerate(groups) for _ in g]
    period = len(flat)
    where = {}
    for t, key in enumerate(flat):
        where.setdefault(key, []).append(t)
    resident = set()
    events = []
    hits = misses = evictions = 0
    for sweep in range(n_sweeps):
        for t, key in enumerate(flat):
            if key in resident:
                hits += 1
                events.append((True, None))
                continue
            misses += 1
            victim = None
            if len(resident) >= n_slots:
                current = set(groups[group_of[t]])
                best = -1
                for cand in resident:
                    if cand in current:
                        continue
                    ahead = min((u - t - 1) % period for u in where[cand])
                    if ahead > best:
                        best, victim = ahead, cand
                if victim is None:
                    raise ValueError("the cache cannot hold one group")
                resident.discard(victim)
                evictions += 1
            resident.add(key)
            events.append((False, victim))
    return events, dict(hits=hits, misses=misses, evictions=evictions)
