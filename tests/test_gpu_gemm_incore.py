"""GPU parity of the in-core tiled GEMM against the CPU oracle, through the C ABI.

Bars: integer-valued inputs bit-exact; uniform[-1,1) fp32 inputs relative Frobenius error <= 1e-5
(the fp32 chain of length K contributes about 2^-24 * sqrt(K) / sqrt(6), i.e. 2e-6 at K = 8000)."""
import numpy as np
import pytest
import torch

from gpu_util import announce, rel_fro, run_incore
from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs

pytestmark = pytest.mark.gpu
TOL_F32 = 1e-5


@pytest.fixture(scope="module")
def ctxs():
    made = {cfg: tg.tgemm_create(0, kernel_config=cfg) for cfg in (0, 1, 2, 3)}
    yield made
    for c in made.values():
        tg.tgemm_destroy(c)


INT_CASES = [
    # M, N, K, T
    (1, 1, 1, 1), (3, 5, 7, 2), (37, 53, 29, 16), (64, 64, 16, 1024), (257, 131, 77, 64),
    (300, 300, 300, 100), (513, 259, 1025, 256), (1000, 1000, 1000, 256), (130, 1030, 40, 512),
    (700, 36, 2050, 1024),
]


@pytest.mark.parametrize("cfg", [0, 1, 2, 3])
@pytest.mark.parametrize("M,N,K,T", INT_CASES)
def test_integer_inputs_bit_exact(ctxs, oracle, M, N, K, T, cfg):
    announce("int", M, N, K, T, "cfg", cfg)
    A = inputs.int_matrix(11, M, K)
    B = inputs.int_matrix(12, K, N)
    C0 = inputs.int_matrix(13, M, N, lo=-7, hi=7)
    ref = oracle.gemm(A.numpy(), B.numpy(), c_in=C0.numpy())
    C = C0.cuda()
    run_incore(ctxs[cfg], A.cuda(), B.cuda(), C, T)
    assert np.array_equal(C.cpu().numpy().astype(np.float64), ref)


def test_config1_full_parity(ctxs, oracle):
    """fp32 1000^3, T = 256 (232-wide edge tiles), uniform[-1,1), C = 0."""
    n, T = 1000, 256
    A = inputs.uniform_matrix(1, n, n)
    B = inputs.uniform_matrix(2, n, n)
    ref = oracle.gemm(A.numpy(), B.numpy())
    for cfg in (0, 1, 2, 3):
        announce("config1 cfg", cfg)
        C = torch.zeros(n, n, device="cuda")
        run_incore(ctxs[cfg], A.cuda(), B.cuda(), C, T)
        err = rel_fro(C.cpu().numpy(), ref)
        print("config1 cfg", cfg, "rel fro", err)
        assert err <= TOL_F32
    st = tg.tgemm_last_stats(ctxs[0])
    assert st["in_core"] == 1 and st["n_tasks"] == 16 and st["n_tile_gemms"] == 64 and st["kernel_ms"] > 0


def test_accumulates_into_c_and_unaligned_pointers(ctxs, oracle):
    """C <- C + A B with non-zero C; odd leading dimensions and a 4-byte-aligned base pointer
    force the scalar load/store paths."""
    M, N, K, T = 203, 157, 301, 64
    A = inputs.uniform_matrix(3, M, K)
    B = inputs.uniform_matrix(4, K, N)
    C0 = inputs.uniform_matrix(5, M, N)
    ref = oracle.gemm(A.numpy(), B.numpy(), c_in=C0.numpy())
    for cfg in (1, 2, 3):
        announce("unaligned cfg", cfg)
        bufA = torch.empty(M * K + 1, device="cuda")
        bufB = torch.empty(K * N + 1, device="cuda")
        bufC = torch.empty(M * N + 1, device="cuda")
        a, b, c = bufA[1:].view(M, K), bufB[1:].view(K, N), bufC[1:].view(M, N)
        a.copy_(A); b.copy_(B); c.copy_(C0)
        run_incore(ctxs[cfg], a, b, c, T)
        assert rel_fro(c.cpu().numpy(), ref) <= TOL_F32


def test_tile_size_does_not_change_integer_result(ctxs, oracle):
    M, N, K = 390, 270, 530
    A = inputs.int_matrix(21, M, K)
    B = inputs.int_matrix(22, K, N)
    ref = oracle.gemm(A.numpy(), B.numpy())
    for T in (1000, 256, 128, 100, 52, 17):
        announce("tile size", T)
        C = torch.zeros(M, N, device="cuda")
        run_incore(ctxs[0], A.cuda(), B.cuda(), C, T)
        assert np.array_equal(C.cpu().numpy().astype(np.float64), ref), T


def test_empty_dimensions(ctxs):
    C = torch.full((4, 5), 3.0, device="cuda")
    A = torch.zeros(4, 1, device="cuda")
    B = torch.zeros(1, 5, device="cuda")
    tg.tgemm_run(ctxs[0], A, B, C, 4, 5, 0, 16)        # K = 0: C unchanged
    tg.tgemm_run(ctxs[0], A, B, C, 0, 5, 1, 16)        # M = 0: nothing to do
    torch.cuda.synchronize()
    assert torch.equal(C.cpu(), torch.full((4, 5), 3.0))


def test_error_paths(ctxs):
    ctx = ctxs[0]
    A = torch.zeros(8, 8, device="cuda")
    host = torch.zeros(8, 8)                      # pageable
    pinned = torch.zeros(8, 8).pin_memory()
    with pytest.raises(tg.TgemmError) as e:
        tg.tgemm_run(ctx, host, A, A.clone(), 8, 8, 8, 4)
    assert e.value.code == tg.TGEMM_EUNPINNED
    with pytest.raises(tg.TgemmError) as e:
        tg.tgemm_run(ctx, pinned, A, A.clone(), 8, 8, 8, 4)
    assert e.value.code == tg.TGEMM_EARG          # mixed kinds
    with pytest.raises(tg.TgemmError) as e:
        tg.tgemm_run(ctx, A, A.clone(), A, 8, 8, 8, 4)
    assert e.value.code == tg.TGEMM_EARG          # C aliases A
    with pytest.raises(tg.TgemmError) as e:
        tg.tgemm_run(ctx, A, A.clone(), A.clone(), 8, 8, 8, 0)
    assert e.value.code == tg.TGEMM_EARG
    with pytest.raises(tg.TgemmError) as e:
        tg.tgemm_run(ctx, A, A.clone(), A.clone(), 8, 8, 8, 4, dtype=7)
    assert e.value.code == tg.TGEMM_EARG
    with pytest.raises(tg.TgemmError) as e:
        tg.tgemm_create(0, incore_schedule=3)
    assert e.value.code == tg.TGEMM_EARG
    # the context is still usable
    C = torch.zeros(8, 8, device="cuda")
    tg.tgemm_run(ctx, torch.eye(8, device="cuda"), torch.ones(8, 8, device="cuda"), C, 8, 8, 8, 4)
    assert torch.equal(C.cpu(), torch.ones(8, 8))


def test_config2_sampled_parity_full_size(ctxs, oracle):
    """fp32 8000^3, T = 1024 (832-wide edge tiles): the whole matrix against the oracle's untiled
    fp64 triple loop (relative Frobenius and the largest entry error), every tile-corner entry and
    4096 random entries against fp64 dot products, Freivalds' identity C x = A (B x) for random
    +-1 vectors; an integer-valued run checked bit-exact on the samples and, through the same
    identity, on every entry."""
    n, T = 8000, 1024
    A = inputs.uniform_matrix(1, n, n, device="cuda")
    B = inputs.uniform_matrix(2, n, n, device="cuda")
    C = torch.zeros(n, n, device="cuda")
    announce("config2 uniform")
    run_incore(ctxs[0], A, B, C, T)
    edges = sorted(set([0, n - 1] + [t * T for t in range(1, 8)] + [t * T - 1 for t in range(1, 8)]))
    rr, cc = np.meshgrid(edges, edges, indexing="ij")
    rnd = np.random.default_rng(0)
    rows = np.concatenate([rr.ravel(), rnd.integers(0, n, 4096)])
    cols = np.concatenate([cc.ravel(), rnd.integers(0, n, 4096)])
    An, Bn = A.cpu().numpy(), B.cpu().numpy()
    ref = oracle.gemm_samples(An, Bn, rows, cols)
    got = C.cpu().numpy()[rows, cols]
    err = rel_fro(got, ref)
    print("config2 sampled rel fro", err, "kernel ms", tg.tgemm_last_stats(ctxs[0])["kernel_ms"])
    assert err <= TOL_F32
    # the whole matrix: the oracle's definition, every one of the 6.4e7 entries (5.1e11 multiply-adds in fp64)
    announce("config2 full oracle")
    Cn = C.cpu().numpy()
    full = oracle.gemm(An, Bn)
    err_full = rel_fro(Cn, full)
    worst = float(np.max(np.abs(Cn - full)))
    print("config2 full-matrix rel fro", err_full, "largest entry error", worst, flush=True)
    assert err_full <= TOL_F32
    # no single entry is off by more than rounding: an fp32 chain of n terms wanders by about
    # 2^-24 sqrt(n) rms(C) (measured: 1.4e-4 rms, 7.6e-4 at worst over 6.4e7 entries); one dropped
    # or doubled product would be off by 0.1 or more
    assert worst <= 16 * 2.0 ** -24 * np.sqrt(n) * float(np.sqrt(np.mean(full * full))), worst
    del full
    # Freivalds: C x = A (B x) for random +-1 vectors; an error anywhere in C survives with probability 1/2 per vector
    A64, B64 = An.astype(np.float64), Bn.astype(np.float64)
    for trial in range(3):
        x = rnd.choice([-1.0, 1.0], n)
        assert rel_fro(Cn.astype(np.float64) @ x, A64 @ (B64 @ x)) <= TOL_F32, trial
    ones = np.ones(n)
    announce("config2 integer")
    Ai = inputs.int_matrix(31, n, n, device="cuda")
    Bi = inputs.int_matrix(32, n, n, device="cuda")
    Ci = torch.zeros(n, n, device="cuda")
    run_incore(ctxs[0], Ai, Bi, Ci, T)
    Ain, Bin = Ai.cpu().numpy(), Bi.cpu().numpy()
    refi = oracle.gemm_samples(Ain, Bin, rows, cols)
    assert np.array_equal(Ci.cpu().numpy()[rows, cols].astype(np.float64), refi)
    assert np.array_equal(Ci.double().sum(1).cpu().numpy(), Ain.astype(np.float64) @ (Bin.astype(np.float64) @ ones))
    Cin = Ci.cpu().numpy().astype(np.float64)
    for trial in range(3):                        # integers in fp64: both sides exact
        x = rnd.choice([-1.0, 1.0], n)
        assert np.array_equal(Cin @ x, Ain.astype(np.float64) @ (Bin.astype(np.float64) @ x)), trial


def test_seeded_random_shapes_integer_exact(ctxs, oracle):
    """Seeded random shapes and tile sizes, every kernel shape: small-integer operands make every
    partial sum exact in fp32, so the result must equal the oracle's bit for bit whatever path a
    workgroup takes (full chunks with or without a ragged last one, ragged k-steps, clamped edge
    tiles, direct-to-LDS or register staging, vector or scalar accesses)."""
    rnd = np.random.default_rng(20240611)
    for case in range(40):
        kind = case % 4
        if kind == 0:      # everything aligned: the unpredicated paths
            M, N, K = (4 * int(rnd.integers(1, 200)) for _ in range(3))
            T = int(rnd.choice([32, 64, 128, 256, 512, 1024]))
        elif kind == 1:    # K not a multiple of the chunk depth, T a multiple: ragged last chunk only
            M, N = (4 * int(rnd.integers(8, 160)) for _ in range(2))
            K = 4 * int(rnd.integers(1, 300)) + 4
            T = int(rnd.choice([64, 128, 256]))
        elif kind == 2:    # odd everything
            M, N, K = (int(rnd.integers(1, 500)) for _ in range(3))
            T = int(rnd.integers(1, 300))
        else:              # wide / tall / deep
            dims = [4 * int(rnd.integers(1, 40)), 4 * int(rnd.integers(100, 400)), 4 * int(rnd.integers(1, 40))]
            rnd.shuffle(dims)
            M, N, K = (int(d) for d in dims)
            T = int(rnd.choice([100, 128, 256, 2048]))
        A = inputs.int_matrix(100 + case, M, K)
        B = inputs.int_matrix(200 + case, K, N)
        C0 = inputs.int_matrix(300 + case, M, N, lo=-7, hi=7)
        ref = oracle.gemm(A.numpy(), B.numpy(), c_in=C0.numpy())
        Ad, Bd = A.cuda(), B.cuda()
        for cfg in (1, 2, 3):
            announce("random int", case, M, N, K, T, "cfg", cfg)
            C = C0.cuda()
            run_incore(ctxs[cfg], Ad, Bd, C, T)
            assert np.array_equal(C.cpu().numpy().astype(np.float64), ref), (M, N, K, T, cfg)


# Products for the balanced schedule (tgemm_opts.incore_schedule): interior tiles of 256 x 256 in whole
# rounds or not, a right strip, a bottom strip, both, neither; strips narrower than a small macro tile;
# K a multiple of 32 only (the strips then keep 32-k stages); a tile size that covers the whole interior.
BALANCED_CASES = [
    # M, N, K, T, launches expected in TGEMM_SCHEDULE_BALANCED mode
    (1600, 1576, 512, 256, 3),      # 36 interior tiles (no whole round): segments + fix-up + strips
    (1536, 1536, 1024, 512, 2),     # no strips
    (4376, 4352, 512, 256, 4),      # 289 interior tiles: one whole round, 33 tiles cut up; bottom strip of 24 rows
    (4352, 4452, 544, 256, 4),      # right strip of 100 columns, K = 17 chunks
    (4482, 4352, 512, 256, 4),      # bottom strip of 130 rows: three rows of small macro tiles
    (1700, 1736, 512, 256, 3),      # both strips several small macro tiles wide
    (800, 800, 1024, 1024, 3),      # one task
    (2600, 2100, 768, 512, 3),      # 5 x 4 tasks, the last ones 512 x 512 of whole tiles
    (512, 512, 800, 1024, 1),       # T is clamped to 800, no multiple of 256: one launch
    (300, 200, 512, 256, 1),        # fewer than 256 columns: one launch
]


@pytest.mark.parametrize("M,N,K,T,launches", BALANCED_CASES)
def test_balanced_schedule(oracle, M, N, K, T, launches):
    """The balanced in-core schedule (whole rounds, k segments of the partial round with their fix-up,
    strips) against the oracle: integer-valued operands bit-exact on the whole matrix, and equal to the
    one-launch schedule's result; uniform operands within the fp32 bar."""
    announce("balanced", M, N, K, T)
    cb = tg.tgemm_create(0, incore_schedule=tg.TGEMM_SCHEDULE_BALANCED)
    c1 = tg.tgemm_create(0, incore_schedule=tg.TGEMM_SCHEDULE_ONE_LAUNCH)
    try:
        A = inputs.int_matrix(41, M, K)
        B = inputs.int_matrix(42, K, N)
        C0 = inputs.int_matrix(43, M, N, lo=-7, hi=7)
        ref = oracle.gemm(A.numpy(), B.numpy(), c_in=C0.numpy())
        Ad, Bd = A.cuda(), B.cuda()
        for rep in range(2):              # the second call reuses the plan and the workspace
            Cb = C0.cuda()
            run_incore(cb, Ad, Bd, Cb, T)
            assert tg.tgemm_last_stats(cb)["kernel_launches"] == launches
            assert np.array_equal(Cb.cpu().numpy().astype(np.float64), ref), rep
        C1 = C0.cuda()
        run_incore(c1, Ad, Bd, C1, T)
        assert tg.tgemm_last_stats(c1)["kernel_launches"] == 1
        assert torch.equal(C1, Cb)
        Au = inputs.uniform_matrix(44, M, K)
        Bu = inputs.uniform_matrix(45, K, N)
        Cu0 = inputs.uniform_matrix(46, M, N)
        refu = oracle.gemm(Au.numpy(), Bu.numpy(), c_in=Cu0.numpy())
        Cu = Cu0.cuda()
        run_incore(cb, Au.cuda(), Bu.cuda(), Cu, T)
        assert rel_fro(Cu.cpu().numpy(), refu) <= TOL_F32
        # another product on the same context: the plan follows the sizes
        M2, N2 = M + 256, N
        A2 = inputs.int_matrix(47, M2, K)
        C2 = torch.zeros(M2, N2, device="cuda")
        run_incore(cb, A2.cuda(), Bd, C2, T)
        assert np.array_equal(C2.cpu().numpy().astype(np.float64), oracle.gemm(A2.numpy(), B.numpy()))
    finally:
        tg.tgemm_destroy(cb)
        tg.tgemm_destroy(c1)


def test_balanced_schedule_is_the_automatic_choice_where_it_gains(oracle):
    """7168^2 x 4096 (784 macro tiles: three whole rounds and 16 tiles more) takes the balanced schedule
    by itself, 8192^2 x 4096 (four whole rounds) one launch; sampled entries against the oracle."""
    ctx = tg.tgemm_create(0)
    try:
        for n, K, launches in ((7168, 4096, 3), (8192, 4096, 1)):
            announce("automatic schedule", n, K)
            A = inputs.uniform_matrix(51, n, K, device="cuda")
            B = inputs.uniform_matrix(52, K, n, device="cuda")
            C = torch.zeros(n, n, device="cuda")
            run_incore(ctx, A, B, C, 1024)
            assert tg.tgemm_last_stats(ctx)["kernel_launches"] == launches
            rnd = np.random.default_rng(n)
            rows = np.concatenate([rnd.integers(0, n, 2048), rnd.integers(n - 256, n, 2048)])
            cols = np.concatenate([rnd.integers(0, n, 2048), rnd.integers(n - 512, n, 2048)])
            ref = oracle.gemm_samples(A.cpu().numpy(), B.cpu().numpy(), rows, cols)
            assert rel_fro(C.cpu().numpy()[rows, cols], ref) <= TOL_F32
    finally:
        tg.tgemm_destroy(ctx)


def test_balanced_schedule_asynchronous_calls_of_changing_sizes(oracle):
    """tgemm_opts.async_incore with the balanced schedule: calls of different sizes enqueued back to back
    share one workspace and its tables (a new plan waits for the copies of the old one); results after one
    tgemm_sync, integer-valued operands bit-exact."""
    ctx = tg.tgemm_create(0, async_incore=1, incore_schedule=tg.TGEMM_SCHEDULE_BALANCED)
    try:
        jobs = []
        for i, (M, N, K, T) in enumerate([(1600, 1576, 512, 256), (800, 800, 1024, 1024), (1600, 1576, 512, 256), (1536, 1536, 1024, 512)]):
            A = inputs.int_matrix(61 + i, M, K)
            B = inputs.int_matrix(71 + i, K, N)
            C0 = inputs.int_matrix(81 + i, M, N, lo=-7, hi=7)
            jobs.append((A, B, C0, A.cuda(), B.cuda(), C0.cuda(), T))
        torch.cuda.synchronize()
        for rep in range(2):          # every C accumulates twice
            for A, B, C0, Ad, Bd, Cd, T in jobs:
                M, K = A.shape
                announce("async balanced", M, B.shape[1], K, T)
                tg.tgemm_run(ctx, Ad, Bd, Cd, M, B.shape[1], K, T, tg.TGEMM_F32, 0)
                assert tg.tgemm_last_stats(ctx)["kernel_launches"] > 1
        tg.tgemm_sync(ctx)
        for A, B, C0, Ad, Bd, Cd, T in jobs:
            ref = oracle.gemm(A.numpy(), B.numpy(), c_in=C0.numpy())
            ref = oracle.gemm(A.numpy(), B.numpy(), c_in=ref)
            assert np.array_equal(Cd.cpu().numpy().astype(np.float64), ref)
    finally:
        tg.tgemm_destroy(ctx)
