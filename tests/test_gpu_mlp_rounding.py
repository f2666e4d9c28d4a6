"""GPU parity of the stochastic rounding of updated bf16 weights (mlp_set_rounding) against the
oracle's generator and rounding rule.

Exact case: a single softmax layer started from zero weights with 256 classes, a batch of 128 and
small-integer inputs.  Probabilities (2^-8), errors and every partial sum of dW = X^T D are then
exact in bf16 / fp32, the fp32 value that gets rounded is the same on both sides, and the stored bit
patterns must agree on every entry -- for every kernel, tile size (even, odd, ragged), in-core and
out-of-core, and for later steps.  General case: a three-layer network with random weights, where
the two sides' fp32 values differ within the bf16 bar; there the result must be one of the two bf16
neighbours and must equal the oracle's wherever the decision does not depend on that difference."""
import numpy as np
import pytest
import torch

from gpu_util import announce
from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs

pytestmark = pytest.mark.gpu


def _bits(t):
    return inputs.bf16_bits(t).copy()       # a pinned host tensor would otherwise be viewed, not copied


def _val(bits):
    return (np.asarray(bits, dtype=np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def _budget(dims, batch, T, frac):
    L = len(dims) - 1
    ws = batch * 4 + batch * dims[L] * 4 + sum(batch * dims[l] * 2 * (2 if l < L else 1) for l in range(1, L + 1))
    ws += 96 * max(-(-d // T) for d in dims) * 8
    n_tiles = sum((-(-dims[l] // T)) * (-(-dims[l + 1] // T)) for l in range(L))
    n_slots = max(int(frac * n_tiles), 2 * max(-(-d // T) for d in dims) + 2)
    return ws + n_slots * T * T * 2


@pytest.mark.parametrize("ooc", [False, True])
@pytest.mark.parametrize("cfg,T", [(2, 96), (3, 96), (4, 96), (2, 75), (4, 75), (3, 2048)])
def test_exact_case_matches_the_oracle_bit_for_bit(oracle, cfg, T, ooc):
    n0, n1, batch, lr, seed = 300, 256, 128, 0.75, 0x1234567887654321
    announce("mlp stochastic rounding, exact case", cfg, T, "ooc" if ooc else "in-core")
    X = inputs.int_matrix(3, batch, n0, lo=-7, hi=7).to(torch.bfloat16)
    y = inputs.labels(4, batch, n1)
    zero = np.zeros((n0, n1), dtype=np.uint16)
    ctx = tg.tgemm_create(0, kernel_config=cfg)
    try:
        W = torch.zeros(n0, n1, dtype=torch.bfloat16)
        W = W.pin_memory() if ooc else W.cuda()
        Xd, yd = X.cuda(), y.cuda()
        torch.cuda.synchronize()
        mlp = tg.mlp_create(ctx, [n0, n1], [W], tg.TGEMM_BF16, T, hbm_budget=_budget([n0, n1], batch, T, 0.5) if ooc else 0)
        tg.mlp_set_rounding(mlp, tg.TGEMM_ROUND_STOCHASTIC, seed)
        for step in range(1 if ooc else 3):
            loss = tg.mlp_step(mlp, Xd, yd, batch, lr)
            tg.tgemm_sync(ctx)
            ref_loss, want, exact = oracle.mlp_step_stochastic(_bits(X), [zero], y.numpy(), lr, seed, step)
            assert abs(loss - ref_loss) <= 1e-6 * ref_loss
            got = _bits(W)
            assert np.array_equal(got, want[0]), (step, int((got != want[0]).sum()))
            # the rounding was exercised: a good share of the entries is not representable in bf16
            e32 = exact[0].astype(np.float32)
            assert np.array_equal(e32.astype(np.float64), exact[0])
            inexact = (e32.view(np.uint32) & 0xFFFF) != 0
            assert inexact.mean() > 0.3
            assert 0.2 < float((got != (e32.view(np.uint32) >> 16))[inexact].mean()) < 0.8      # ups and downs
            if step > 0:
                assert not np.array_equal(got, first)                                        # fresh bits per step
            else:
                first = got.copy()
            if not ooc:
                W.zero_()                      # caller-owned device weights: start the next step from zero again
                torch.cuda.synchronize()
        # back to nearest-even, and the step count restarts with a new seed
        tg.mlp_set_rounding(mlp, tg.TGEMM_ROUND_NEAREST, 0)
        if not ooc:
            tg.mlp_step(mlp, Xd, yd, batch, lr)
            tg.tgemm_sync(ctx)
            rne = torch.from_numpy(exact[0].astype(np.float32)).to(torch.bfloat16)
            assert np.array_equal(_bits(W), _bits(rne))
            W.zero_()
            torch.cuda.synchronize()
            tg.mlp_set_rounding(mlp, tg.TGEMM_ROUND_STOCHASTIC, seed)
            tg.mlp_step(mlp, Xd, yd, batch, lr)
            tg.tgemm_sync(ctx)
            assert np.array_equal(_bits(W), first)
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)


def _random_net(dims, batch):
    X = inputs.normal_matrix(1, batch, dims[0]).to(torch.bfloat16)
    Ws = [inputs.normal_matrix(10 + l, dims[l], dims[l + 1], std=0.05).to(torch.bfloat16) for l in range(len(dims) - 1)]
    return X, Ws, inputs.labels(5, batch, dims[-1])


@pytest.mark.parametrize("ooc", [False, True])
def test_general_case_neighbours_and_decided_entries(oracle, ooc):
    dims, batch, T, lr, seed = [256, 384, 320, 200], 192, 128, 0.25, 77
    announce("mlp stochastic rounding, general case", "ooc" if ooc else "in-core")
    X, Ws, y = _random_net(dims, batch)
    ctx = tg.tgemm_create(0, kernel_config=3)
    try:
        Wx = [w.clone().pin_memory() if ooc else w.cuda() for w in Ws]
        Xd, yd = X.cuda(), y.cuda()
        torch.cuda.synchronize()
        mlp = tg.mlp_create(ctx, dims, Wx, tg.TGEMM_BF16, T, hbm_budget=_budget(dims, batch, T, 0.4) if ooc else 0)
        tg.mlp_set_rounding(mlp, tg.TGEMM_ROUND_STOCHASTIC, seed)
        for step in range(3):
            before = [_bits(w) for w in Wx]
            tg.mlp_step(mlp, Xd, yd, batch, lr)
            tg.tgemm_sync(ctx)
            # the oracle starts every step from the weights the GPU holds, with the step's bits
            _, want, exact = oracle.mlp_step_stochastic(_bits(X), before, y.numpy(), lr, seed, step)
            acts, _, _ = oracle.mlp_forward(_bits(X), before)
            _, dWs, deltas = oracle.mlp_backward(_bits(X), before, y.numpy())
            for l in range(len(Ws)):
                got = _bits(Wx[l])
                # how far the GPU's fp32 value may sit from the oracle's: activations and errors are
                # stored as bf16 (2^-9 each) on the GPU, entrywise |A|^T |D| 2^-8 to first order; 4x margin
                eps = lr * 2.0 ** -6 * (np.abs(acts[l]).T @ np.abs(deltas[l]))
                e = exact[l]
                lo32, hi32 = (e - eps).astype(np.float32), (e + eps).astype(np.float32)
                b_lo = oracle.stochastic_round_matrix(lo32, seed, l + 1, step)
                b_hi = oracle.stochastic_round_matrix(hi32, seed, l + 1, step)
                decided = (b_lo == b_hi) & (b_lo == want[l])
                assert decided.mean() > 0.5, (step, l, decided.mean())
                assert np.array_equal(got[decided], want[l][decided]), (step, l, int((got != want[l])[decided].sum()))
                # everywhere: between the truncation of the smallest and the upper neighbour of the
                # largest magnitude that the fp32 value may have
                cands = np.stack([_val(lo32.view(np.uint32) >> 16), _val((lo32.view(np.uint32) >> 16) + 1),
                                  _val(hi32.view(np.uint32) >> 16), _val((hi32.view(np.uint32) >> 16) + 1)])
                g = _val(got)
                assert np.all((g >= cands.min(axis=0)) & (g <= cands.max(axis=0))), (step, l)
                # and most entries agree outright
                assert float((got == want[l]).mean()) > 0.85
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)


def test_same_bits_whatever_kernel_tile_size_or_residency():
    dims, batch, lr, seed = [256, 384, 320, 200], 192, 4.0, 5
    X, Ws, y = _random_net(dims, batch)
    Xd, yd = X.cuda(), y.cuda()
    runs = []
    for cfg, T, ooc in ((3, 128, False), (4, 128, False), (2, 128, False), (3, 64, False), (3, 128, True), (4, 96, True)):
        announce("mlp stochastic rounding, reproducibility", cfg, T, ooc)
        ctx = tg.tgemm_create(0, kernel_config=cfg)
        try:
            Wx = [w.clone().pin_memory() if ooc else w.cuda() for w in Ws]
            torch.cuda.synchronize()
            mlp = tg.mlp_create(ctx, dims, Wx, tg.TGEMM_BF16, T, hbm_budget=_budget(dims, batch, T, 0.4) if ooc else 0)
            tg.mlp_set_rounding(mlp, tg.TGEMM_ROUND_STOCHASTIC, seed)
            losses = [tg.mlp_step(mlp, Xd, yd, batch, lr) for _ in range(3)]
            tg.tgemm_sync(ctx)
            runs.append((losses, [_bits(w) for w in Wx]))
            tg.mlp_destroy(mlp)
        finally:
            tg.tgemm_destroy(ctx)
    for losses, ws in runs[1:]:
        assert losses == runs[0][0]
        for a, b in zip(ws, runs[0][1]):
            assert np.array_equal(a, b)


def test_small_updates_survive_in_expectation(oracle):
    """A learning rate that puts most updates below half an ulp: nearest-even leaves those weights
    where they were, stochastic rounding moves the sum of the weights by the sum of the updates."""
    dims, batch, T, lr = [256, 384, 200], 192, 128, 0.02
    X, Ws, y = _random_net(dims, batch)
    Xd, yd = X.cuda(), y.cuda()
    _, exact, _ = oracle.mlp_step(_bits(X), [_bits(w) for w in Ws], y.numpy(), lr)
    out = {}
    for mode in (tg.TGEMM_ROUND_NEAREST, tg.TGEMM_ROUND_STOCHASTIC):
        announce("mlp small updates, rounding mode", mode)
        ctx = tg.tgemm_create(0)
        try:
            Wd = [w.cuda() for w in Ws]
            torch.cuda.synchronize()
            mlp = tg.mlp_create(ctx, dims, Wd, tg.TGEMM_BF16, T)
            tg.mlp_set_rounding(mlp, mode, 9)
            tg.mlp_step(mlp, Xd, yd, batch, lr)
            tg.tgemm_sync(ctx)
            out[mode] = [_val(_bits(w)) for w in Wd]
            tg.mlp_destroy(mlp)
        finally:
            tg.tgemm_destroy(ctx)
    for l, w in enumerate(Ws):
        old = _val(_bits(w))
        want = exact[l] - old                                 # the update, -lr dW
        ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(old), 1e-30))) - 7)
        small = np.abs(want) < 0.25 * ulp
        assert small.mean() > 0.5, small.mean()
        rne, sr = out[tg.TGEMM_ROUND_NEAREST][l] - old, out[tg.TGEMM_ROUND_STOCHASTIC][l] - old
        assert np.all(rne[small] == 0.0)                      # lost
        # stochastic: per entry a step of one ulp with probability |update| / ulp; the sum over the
        # small entries has standard deviation sqrt(sum ulp^2 p (1 - p))
        p = np.abs(want[small]) / ulp[small]
        sd = np.sqrt(np.sum(ulp[small] ** 2 * p * (1 - p)))
        assert abs(sr[small].sum() - want[small].sum()) < 5 * sd + 0.02 * np.abs(want[small]).sum()
        assert np.abs(sr[small]).sum() > 0.5 * np.abs(want[small]).sum()
        assert set(np.unique(np.round(np.abs(sr[small]) / ulp[small], 6)).tolist()) <= {0.0, 0.5, 1.0}


def test_rounding_mode_errors():
    ctx = tg.tgemm_create(0)
    try:
        W = [torch.zeros(64, 32, device="cuda")]
        mlp = tg.mlp_create(ctx, [64, 32], W, tg.TGEMM_F32, 32)
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_set_rounding(mlp, tg.TGEMM_ROUND_STOCHASTIC, 1)
        assert e.value.code == tg.TGEMM_EARG
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_set_rounding(mlp, 5, 1)
        assert e.value.code == tg.TGEMM_EARG
        tg.mlp_set_rounding(mlp, tg.TGEMM_ROUND_NEAREST, 1)
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)
