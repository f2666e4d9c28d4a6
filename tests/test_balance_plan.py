"""Host logic of the balanced in-core schedule (tgemm_balance_plan; no GPU): the k segments of the
partial round must cover every (tile, chunk) pair of its tiles exactly once, number their workspace
slots so that a tile's slots are consecutive and ascend with k (the order in which the fix-up adds
them), stay within the workspace, and spread evenly over the compute units under the dispatcher's rule
(the next workgroup goes to the first unit that falls free)."""
import heapq

import numpy as np
import pytest

from paper_1511_04348_amd import binding as tg

MAX_SLOTS = 512


def _interior_tiles(plan):
    return (plan["interior_rows"] // 256) * (plan["interior_cols"] // 256)


def _check_invariants(M, N, K, T, dtype, n_cus, plan, segs):
    assert plan["applies"] == 1
    assert plan["interior_rows"] == M // 256 * 256 and plan["interior_cols"] == N // 256 * 256
    n_tiles, n_ch = _interior_tiles(plan), K // 32
    assert plan["chunks_per_tile"] == n_ch
    assert plan["tail_tiles"] == n_tiles % n_cus and plan["tail_tiles"] > 0
    assert plan["whole_round_tiles"] == n_tiles - plan["tail_tiles"] and plan["whole_round_tiles"] % n_cus == 0
    assert plan["n_segments"] == len(segs) and 0 < len(segs) <= MAX_SLOTS - 1
    # every (tile, chunk) of the partial round exactly once
    cover = np.zeros((plan["tail_tiles"], n_ch), dtype=np.int32)
    for s in segs:
        t = s["tile"] - plan["whole_round_tiles"]
        assert 0 <= t < plan["tail_tiles"] and s["n_chunks"] >= 1
        assert 0 <= s["first_chunk"] and s["first_chunk"] + s["n_chunks"] <= n_ch
        cover[t, s["first_chunk"]:s["first_chunk"] + s["n_chunks"]] += 1
    assert (cover == 1).all()
    # slots: a permutation of 0 .. n - 1; per tile consecutive, ascending with k
    assert sorted(s["slot"] for s in segs) == list(range(len(segs)))
    by_tile = {}
    for s in segs:
        by_tile.setdefault(s["tile"], []).append(s)
    for t, lst in by_tile.items():
        lst.sort(key=lambda s: s["first_chunk"])
        assert [s["slot"] for s in lst] == list(range(lst[0]["slot"], lst[0]["slot"] + len(lst))), t


def _makespan(segs, n_cus, start=1.5):
    """Workgroup b goes to XCD b % 8; inside an XCD the next one goes to the first free unit."""
    worst = 0.0
    for x in range(8):
        units = [0.0] * max(1, n_cus // 8)
        for b in range(x, len(segs), 8):
            t = heapq.heappop(units)
            heapq.heappush(units, t + segs[b]["n_chunks"] + start)
        worst = max(worst, max(units))
    return worst


def test_config2_plan():
    plan, segs = tg.tgemm_balance_plan(8000, 8000, 8000, 1024)
    _check_invariants(8000, 8000, 8000, 1024, 0, 256, plan, segs)
    assert plan["whole_round_tiles"] == 768 and plan["tail_tiles"] == 193 and plan["even_parts"] == 0
    # 193 x 250 chunks over 256 units: 188.5 each; a range crosses at most one tile boundary
    assert plan["n_segments"] == 447 and max(s["n_chunks"] for s in segs) == 189
    # a unit's share is 188.5 chunks, in one piece or two: with 1.5 chunks to start a piece no unit is busy
    # longer than 189 + 3 (a whole tile takes 250 + 1.5; the same segments simply longest first: 196)
    assert _makespan(segs, 256) <= 192
    assert _makespan(sorted(segs, key=lambda s: -s["n_chunks"]), 256) >= 195


SHAPES = [(8000, 8000, 8000, 1024), (7168, 7168, 4096, 1024), (4376, 4352, 512, 256), (4352, 4452, 544, 256),
          (1600, 1576, 512, 256), (800, 800, 1024, 1024), (2600, 2100, 768, 512), (3328, 3328, 640, 256),
          (5888, 5888, 5888, 256), (9216, 9216, 2048, 512), (256 * 25, 256 * 3, 1024, 256), (256, 256, 512, 256)]


@pytest.mark.parametrize("M,N,K,T", SHAPES)
@pytest.mark.parametrize("n_cus", [256, 64, 8])
def test_fp32_segments_partition_and_balance(M, N, K, T, n_cus):
    plan, segs = tg.tgemm_balance_plan(M, N, K, T, tg.TGEMM_F32, n_cus, 1)
    if (M // 256) * (N // 256) % n_cus == 0:
        assert plan["applies"] == 0       # whole rounds only: nothing to balance
        return
    _check_invariants(M, N, K, T, 0, n_cus, plan, segs)
    assert plan["even_parts"] == 0
    lens = [s["n_chunks"] for s in segs]
    # equal ranges of the (tile, chunk) pairs laid end to end, each cut at most once (where it crosses
    # into the next tile): no piece is longer than a share, and there are at most units + tiles of them
    n_ch = K // 32
    share = plan["tail_tiles"] * n_ch / n_cus
    assert max(lens) <= int(np.ceil(share)) and len(segs) <= n_cus + plan["tail_tiles"]
    # under the dispatcher's rule every unit ends up with one range's worth of chunks: its long piece and
    # a short piece that is its own range's other half, or one no longer
    if share >= 1:
        assert _makespan(segs, n_cus, start=0.0) <= int(np.ceil(share)) + 1


@pytest.mark.parametrize("M,N,K,T", [(6144, 6144, 6144, 2048), (1536, 1536, 1024, 512), (4352, 4352, 512, 256),
                                     (2560, 2048, 768, 512), (7168, 7168, 7168, 1024), (3328, 3328, 640, 256)])
def test_bf16_even_pieces(M, N, K, T):
    plan, segs = tg.tgemm_balance_plan(M, N, K, T, tg.TGEMM_BF16, 256, 1)
    _check_invariants(M, N, K, T, 1, 256, plan, segs)
    t, n_ch = plan["tail_tiles"], K // 32
    if t > 128:
        assert plan["even_parts"] == 0    # no even cut possible: the ranges of the fp32 schedule
        return
    parts = plan["even_parts"]
    assert parts == min(256 // t, n_ch // 4) and len(segs) == t * parts
    lens = [s["n_chunks"] for s in segs]
    assert max(lens) - min(lens) <= 1
    # one wave of workgroups; on every XCD (blocks b % 8) consecutive workgroups walk the same piece of
    # neighbouring tiles: ascending (piece, tile)
    assert len(segs) <= 256
    for x in range(8):
        seq = [(s["first_chunk"], s["tile"]) for s in segs[x::8]]
        assert seq == sorted(seq)


@pytest.mark.parametrize("args", [
    (8192, 8192, 8192, 1024, 0),      # whole rounds only
    (8000, 8000, 8000, 1000, 0),      # tasks are not whole macro tiles
    (8000, 8000, 8008, 1024, 0),      # K no multiple of 32
    (8000, 8000, 256, 1024, 0),       # too shallow
    (200, 8000, 8000, 1024, 0),       # fewer than 256 rows
    (8000, 8000, 8000, 1024, 1),      # bf16 with remainder strips
    (8001, 8000, 8000, 1024, 0),      # rows of A and C are fine, but B / C rows of 8000 floats with M odd still apply?
])
def test_declined(args):
    plan, segs = tg.tgemm_balance_plan(*args, 256, 1)
    if args[0] == 8001:
        assert plan["applies"] == 1 and plan["interior_rows"] == 7936      # an odd M only lengthens the bottom strip
    else:
        assert plan["applies"] == 0 and segs == []


def test_automatic_choice_follows_the_estimate():
    takes = lambda n, K, dt=0, T=1024: tg.tgemm_balance_plan(n, n, K, T, dt)[0]["applies"]
    assert takes(8000, 8000) == 1 and takes(7680, 7680) == 1 and takes(9216, 9216) == 1
    assert takes(8192, 8192) == 0 and takes(2048, 2048) == 0 and takes(2816, 2816, T=256) == 0
    assert takes(6144, 6144, 1, 2048) == 1 and takes(5120, 5120, 1, 2048) == 0 and takes(7680, 7680, 1, 2048) == 0


def test_argument_errors():
    lib = tg.load()
    assert lib.tgemm_balance_plan(8, 8, 8, 8, 0, 256, 0, None, None, 0) == tg.TGEMM_EARG
    b = tg.tgemm_balance()
    import ctypes
    assert lib.tgemm_balance_plan(8, 8, 8, 0, 0, 256, 0, ctypes.byref(b), None, 0) == tg.TGEMM_EARG
    assert lib.tgemm_balance_plan(8, 8, 8, 8, 7, 256, 0, ctypes.byref(b), None, 0) == tg.TGEMM_EARG
    assert lib.tgemm_balance_plan(8, 8, 8, 8, 0, 256, 0, ctypes.byref(b), None, 4) == tg.TGEMM_EARG
