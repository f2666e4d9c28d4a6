"""GPU parity of the bf16-input / fp32-accumulate tiled GEMM (in-core and out-of-core) against the
oracle, which widens the same bf16 bit patterns exactly to fp64.  Bars: integer-valued inputs
bit-exact; random inputs relative Frobenius error <= 1e-2 (the stated bf16 bar; the inputs are
already bf16, so only the fp32 accumulation differs and the observed error is ~1e-6, which the
tests also require to stay below 1e-4 to catch indexing mistakes that a loose bar would hide)."""
import numpy as np
import pytest
import torch

from gpu_util import announce, rel_fro
from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs

pytestmark = pytest.mark.gpu
BAR, SANITY = 1e-2, 1e-4


def _bf16(t):
    return t.to(torch.bfloat16)


@pytest.fixture(scope="module")
def ctxs():
    made = {cfg: tg.tgemm_create(0, kernel_config=cfg) for cfg in (0, 2, 3, 4)}
    yield made
    for c in made.values():
        tg.tgemm_destroy(c)


CASES = [(1, 1, 1, 1), (3, 5, 7, 2), (37, 53, 29, 16), (64, 64, 16, 1024), (257, 131, 77, 64),
         (300, 300, 300, 100), (513, 259, 1025, 256), (1000, 1000, 1000, 256), (130, 1030, 40, 512),
         (700, 36, 2050, 1024), (256, 256, 64, 256), (384, 512, 200, 128),
         # shapes the direct-to-LDS kernel takes under config 3 (whole 32-k chunks, N a multiple of 8):
         # ragged edge tiles in M and N, one chunk, fewer chunks than stages, T above and below K
         (1304, 1096, 1312, 256), (520, 264, 64, 256), (1000, 1000, 992, 1000), (264, 520, 96, 2048),
         (40, 8, 32, 64), (2048, 1536, 1024, 512), (77, 640, 160, 32)]


@pytest.mark.parametrize("cfg", [0, 2, 3, 4])
@pytest.mark.parametrize("M,N,K,T", CASES)
def test_integer_inputs_bit_exact(ctxs, oracle, M, N, K, T, cfg):
    announce("bf16 int", M, N, K, T, "cfg", cfg)
    A = _bf16(inputs.int_matrix(11, M, K))
    B = _bf16(inputs.int_matrix(12, K, N))
    C0 = inputs.int_matrix(13, M, N, lo=-7, hi=7)
    ref = oracle.gemm(inputs.bf16_bits(A), inputs.bf16_bits(B), c_in=C0.numpy())
    C = C0.cuda()
    Ad, Bd = A.cuda(), B.cuda()
    torch.cuda.synchronize()
    tg.tgemm_run(ctxs[cfg], Ad, Bd, C, M, N, K, T, tg.TGEMM_BF16, 0)
    assert np.array_equal(C.cpu().numpy().astype(np.float64), ref)


def test_uniform_parity_and_unaligned(ctxs, oracle):
    for (M, N, K, T) in [(1000, 1000, 1000, 256), (203, 157, 301, 64), (520, 264, 776, 128),
                         (520, 264, 768, 128), (1304, 1096, 1312, 256)]:   # the last two: direct-to-LDS when aligned
        A = _bf16(inputs.uniform_matrix(1, M, K))
        B = _bf16(inputs.uniform_matrix(2, K, N))
        C0 = inputs.uniform_matrix(3, M, N)
        ref = oracle.gemm(inputs.bf16_bits(A), inputs.bf16_bits(B), c_in=C0.numpy())
        for cfg in (0, 2, 3, 4):
            announce("bf16 uniform", M, N, K, T, "cfg", cfg)
            # a 2-byte offset from an aligned base exercises the scalar load paths
            bufA = torch.empty(M * K + 1, dtype=torch.bfloat16, device="cuda")
            bufB = torch.empty(K * N + 1, dtype=torch.bfloat16, device="cuda")
            a, b = bufA[1:].view(M, K), bufB[1:].view(K, N)
            a.copy_(A); b.copy_(B)
            C = C0.cuda()
            torch.cuda.synchronize()
            tg.tgemm_run(ctxs[cfg], a, b, C, M, N, K, T, tg.TGEMM_BF16, 0)
            err = rel_fro(C.cpu().numpy(), ref)
            assert err <= BAR and err <= SANITY, err
            C2 = C0.cuda()
            Ad, Bd = A.cuda(), B.cuda()
            torch.cuda.synchronize()
            tg.tgemm_run(ctxs[cfg], Ad, Bd, C2, M, N, K, T, tg.TGEMM_BF16, 0)
            assert torch.equal(C2, C)        # vector and scalar load paths agree bit for bit


def test_out_of_core_bf16(oracle):
    M, N, K, T, n_ab = 1500, 1400, 1300, 256, 20
    A = _bf16(inputs.uniform_matrix(1, M, K))
    B = _bf16(inputs.uniform_matrix(2, K, N))
    C0 = inputs.uniform_matrix(3, M, N)
    ref = oracle.gemm(inputs.bf16_bits(A), inputs.bf16_bits(B), c_in=C0.numpy())
    ctx = tg.tgemm_create(0, trace=1, order=tg.TGEMM_ORDER_SERPENTINE)
    try:
        Ap, Bp, Cp = A.pin_memory(), B.pin_memory(), C0.clone().pin_memory()
        budget = 4 * T * T * 4 + n_ab * T * T * 2
        tg.tgemm_run(ctx, Ap, Bp, Cp, M, N, K, T, tg.TGEMM_BF16, budget)
        err = rel_fro(Cp.numpy(), ref)
        assert err <= BAR and err <= SANITY, err
        st = tg.tgemm_last_stats(ctx)
        seq = oracle.tgemm_access_sequence(M, N, K, T, order="serpentine")
        _, sim = oracle.lru_simulate([s[:3] for s in seq], st["n_slots"])
        assert st["n_slots"] == n_ab and (st["hits"], st["misses"]) == (sim["hits"], sim["misses"])
        Ai = _bf16(inputs.int_matrix(5, M, K)).pin_memory()
        Bi = _bf16(inputs.int_matrix(6, K, N)).pin_memory()
        Ci = torch.zeros(M, N).pin_memory()
        tg.tgemm_run(ctx, Ai, Bi, Ci, M, N, K, T, tg.TGEMM_BF16, budget)
        assert np.array_equal(Ci.numpy().astype(np.float64), oracle.gemm(inputs.bf16_bits(Ai), inputs.bf16_bits(Bi)))
    finally:
        tg.tgemm_destroy(ctx)


def test_supplementary_8192_sampled(ctxs, oracle):
    """bf16 8192^3, T = 2048, in-core: sampled entries against fp64 dot products."""
    n, T = 8192, 2048
    A = _bf16(inputs.uniform_matrix(1, n, n, device="cuda"))
    B = _bf16(inputs.uniform_matrix(2, n, n, device="cuda"))
    C = torch.zeros(n, n, device="cuda")
    torch.cuda.synchronize()
    tg.tgemm_run(ctxs[0], A, B, C, n, n, n, T, tg.TGEMM_BF16, 0)
    st = tg.tgemm_last_stats(ctxs[0])
    print("bf16 8192^3 kernel ms", st["kernel_ms"], "TFLOP/s", 2.0 * n ** 3 / st["kernel_ms"] / 1e9)
    rnd = np.random.default_rng(0)
    edges = sorted(set([0, n - 1] + [t * T for t in range(1, 4)] + [t * T - 1 for t in range(1, 4)]))
    rr, cc = np.meshgrid(edges, edges, indexing="ij")
    rows = np.concatenate([rr.ravel(), rnd.integers(0, n, 2048)])
    cols = np.concatenate([cc.ravel(), rnd.integers(0, n, 2048)])
    ref = oracle.gemm_samples(inputs.bf16_bits(A), inputs.bf16_bits(B), rows, cols)
    err = rel_fro(C.cpu().numpy()[rows, cols], ref)
    assert err <= BAR and err <= SANITY, err


def test_direct_to_lds_kernel_equals_register_staged_kernel_bitwise(ctxs, oracle):
    """Seeded random shapes that the direct-to-LDS kernel accepts (whole 32-k chunks, N a multiple
    of 8, aligned pointers): ragged edge tiles in M and N, tile sizes below, at and above the
    dimensions, 1 to 60 chunks.  Both 256 x 256 kernels run the same sequence of 16-k MFMAs per
    output element, so their results must agree bit for bit; every fourth shape is also compared with
    the oracle."""
    rnd = np.random.default_rng(20240607)
    for case in range(32):
        M = int(rnd.integers(1, 1400))
        N = 8 * int(rnd.integers(1, 170))
        K = 32 * int(rnd.integers(1, 60))
        T = int(rnd.choice([32, 64, 96, 128, 256, 512, 2048]))
        announce("bf16 dl vs staged", case, M, N, K, T)
        A = _bf16(inputs.uniform_matrix(100 + case, M, K)).cuda()
        B = _bf16(inputs.uniform_matrix(200 + case, K, N)).cuda()
        C0 = inputs.uniform_matrix(300 + case, M, N)
        outs = []
        for cfg in (3, 4):
            C = C0.cuda()
            torch.cuda.synchronize()
            tg.tgemm_run(ctxs[cfg], A, B, C, M, N, K, T, tg.TGEMM_BF16, 0)
            outs.append(C.cpu())
        assert torch.equal(outs[0], outs[1]), (M, N, K, T)
        if case % 4 == 0:
            ref = oracle.gemm(inputs.bf16_bits(A.cpu()), inputs.bf16_bits(B.cpu()), c_in=C0.numpy())
            err = rel_fro(outs[0].numpy(), ref)
            assert err <= BAR and err <= SANITY, (M, N, K, T, err)


# M, N, K, T, launches expected under TGEMM_SCHEDULE_BALANCED: the partial round's tiles cut evenly (at
# most half as many tiles as compute units) or by equal ranges (more); with whole rounds before it or not
BALANCED_CASES = [
    (1536, 1536, 1024, 512, 2),     # 36 tiles, 7 pieces each
    (4352, 4352, 512, 256, 3),      # a whole round + 33 tiles, in 4 pieces each (a piece is at least 4 chunks)
    (2560, 2048, 768, 512, 2),      # 80 tiles, 3 pieces each
    (3328, 3328, 640, 256, 2),      # 169 tiles: more than half the units, equal ranges
    (1536, 1528, 1024, 512, 1),     # N no multiple of 256: declined, one launch
]


@pytest.mark.parametrize("M,N,K,T,launches", BALANCED_CASES)
def test_balanced_schedule(oracle, M, N, K, T, launches):
    """The balanced in-core schedule with the direct-to-LDS kernel (whole rounds, k pieces of the partial
    round's tiles into a workspace, fix-up): integer-valued operands bit-exact on the whole matrix and
    equal to the one launch; uniform operands within the bars."""
    announce("bf16 balanced", M, N, K, T)
    cb = tg.tgemm_create(0, incore_schedule=tg.TGEMM_SCHEDULE_BALANCED)
    c1 = tg.tgemm_create(0, incore_schedule=tg.TGEMM_SCHEDULE_ONE_LAUNCH)
    try:
        A = _bf16(inputs.int_matrix(41, M, K))
        B = _bf16(inputs.int_matrix(42, K, N))
        C0 = inputs.int_matrix(43, M, N, lo=-7, hi=7)
        ref = oracle.gemm(inputs.bf16_bits(A), inputs.bf16_bits(B), c_in=C0.numpy())
        Ad, Bd = A.cuda(), B.cuda()
        for rep in range(2):
            Cb = C0.cuda()
            torch.cuda.synchronize()
            tg.tgemm_run(cb, Ad, Bd, Cb, M, N, K, T, tg.TGEMM_BF16, 0)
            assert tg.tgemm_last_stats(cb)["kernel_launches"] == launches
            assert np.array_equal(Cb.cpu().numpy().astype(np.float64), ref), rep
        C1 = C0.cuda()
        torch.cuda.synchronize()
        tg.tgemm_run(c1, Ad, Bd, C1, M, N, K, T, tg.TGEMM_BF16, 0)
        assert tg.tgemm_last_stats(c1)["kernel_launches"] == 1
        assert torch.equal(C1, Cb)
        Au = _bf16(inputs.uniform_matrix(44, M, K))
        Bu = _bf16(inputs.uniform_matrix(45, K, N))
        Cu0 = inputs.uniform_matrix(46, M, N)
        refu = oracle.gemm(inputs.bf16_bits(Au), inputs.bf16_bits(Bu), c_in=Cu0.numpy())
        Cu = Cu0.cuda()
        Aud, Bud = Au.cuda(), Bu.cuda()
        torch.cuda.synchronize()
        tg.tgemm_run(cb, Aud, Bud, Cu, M, N, K, T, tg.TGEMM_BF16, 0)
        err = rel_fro(Cu.cpu().numpy(), refu)
        assert err <= BAR and err <= SANITY, err
    finally:
        tg.tgemm_destroy(cb)
        tg.tgemm_destroy(c1)
