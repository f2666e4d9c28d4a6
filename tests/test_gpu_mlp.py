"""GPU parity of the MLP passes (forward = equation 1, backward = equations 3 and 4, SGD step)
against the fp64 oracle, through the C ABI.  fp32 bar: relative Frobenius error <= 1e-5 on every
activation, the probabilities, the loss, every error matrix, every dW, and on W_new - W_old."""
import numpy as np
import pytest
import torch

from gpu_util import announce, rel_fro
from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs

pytestmark = pytest.mark.gpu
TOL = 1e-5


def _net(dims, batch, std=0.05, seed=0):
    X = inputs.normal_matrix(seed + 1, batch, dims[0])
    Ws = [inputs.normal_matrix(seed + 10 + l, dims[l], dims[l + 1], std=std) for l in range(len(dims) - 1)]
    y = inputs.labels(seed + 5, batch, dims[-1])
    return X, Ws, y


def _read(mlp, what, layer, rows, cols):
    out = torch.empty(rows, cols)
    tg.mlp_read(mlp, what, layer, out, rows * cols * 4)
    return out.numpy()


@pytest.mark.parametrize("dims,batch,T", [([5, 7, 6, 4], 3, 2), ([64, 96, 80, 50], 33, 32),
                                          ([512, 2048, 2048, 2048, 1250], 512, 1024),
                                          ([300, 700, 10], 130, 256), ([40, 30], 17, 16)])
def test_forward_backward_step_parity(oracle, dims, batch, T):
    announce("mlp", dims, batch, T)
    X, Ws, y = _net(dims, batch)
    L = len(Ws)
    acts, z, P = oracle.mlp_forward(X.numpy(), [w.numpy() for w in Ws])
    loss_ref, dW_ref, delta_ref = oracle.mlp_backward(X.numpy(), [w.numpy() for w in Ws], y.numpy())
    ctx = tg.tgemm_create(0)
    try:
        Xd, yd = X.cuda(), y.cuda()
        Wd = [w.cuda() for w in Ws]
        torch.cuda.synchronize()
        mlp = tg.mlp_create(ctx, dims, Wd, tg.TGEMM_F32, T)
        probs = torch.empty(batch, dims[-1], device="cuda")
        tg.mlp_forward(mlp, Xd, batch, probs)
        for l in range(1, L):
            assert rel_fro(_read(mlp, 0, l, batch, dims[l]), acts[l]) <= TOL, ("activation", l)
        assert rel_fro(_read(mlp, 1, 0, batch, dims[-1]), z) <= TOL
        assert rel_fro(probs.cpu().numpy(), P) <= TOL
        dWd = [torch.zeros_like(w) for w in Wd]
        torch.cuda.synchronize()
        loss = tg.mlp_backward(mlp, yd, dWd)
        assert abs(loss - loss_ref) <= TOL * abs(loss_ref)
        for l in range(1, L + 1):
            assert rel_fro(_read(mlp, 2, l, batch, dims[l]), delta_ref[l - 1]) <= TOL, ("delta", l)
        for l in range(L):
            assert rel_fro(dWd[l].cpu().numpy(), dW_ref[l]) <= TOL, ("dW", l)
            assert torch.equal(Wd[l].cpu(), Ws[l])                      # backward leaves W alone
        # one fused step: W_new - W_old against -lr * dW (all dW from the pre-update weights)
        lr = 0.01
        loss2 = tg.mlp_step(mlp, Xd, yd, batch, lr)
        assert abs(loss2 - loss_ref) <= TOL * abs(loss_ref)
        for l in range(L):
            upd = Wd[l].cpu().numpy().astype(np.float64) - Ws[l].numpy().astype(np.float64)
            # the update is rounded into fp32 weights: half an ulp of W per entry on top of the bar
            slack = np.linalg.norm(Ws[l].numpy()) * 2.0 ** -24 / np.linalg.norm(lr * dW_ref[l])
            assert rel_fro(upd, -lr * dW_ref[l]) <= TOL + slack, ("update", l)
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)


def test_training_reduces_loss_and_matches_oracle_trajectory(oracle):
    dims, batch, T, lr = [32, 48, 10], 64, 32, 0.5
    X, Ws, y = _net(dims, batch, std=0.3, seed=7)
    ctx = tg.tgemm_create(0)
    try:
        Wd = [w.cuda() for w in Ws]
        Xd, yd = X.cuda(), y.cuda()
        torch.cuda.synchronize()
        mlp = tg.mlp_create(ctx, dims, Wd, tg.TGEMM_F32, T)
        Wo = [w.numpy().astype(np.float64) for w in Ws]
        losses = []
        for step in range(5):
            losses.append(tg.mlp_step(mlp, Xd, yd, batch, lr))
            lo, Wo, _ = oracle.mlp_step(X.numpy(), Wo, y.numpy(), lr)
            assert abs(losses[-1] - lo) <= 1e-4 * abs(lo)
        assert losses[-1] < losses[0]
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)


def test_zero_weights_closed_form():
    dims, batch = [16, 24, 1000], 8
    ctx = tg.tgemm_create(0)
    try:
        Wd = [torch.zeros(dims[l], dims[l + 1], device="cuda") for l in range(2)]
        X = inputs.normal_matrix(1, batch, dims[0]).cuda()
        y = inputs.labels(2, batch, dims[-1]).cuda()
        torch.cuda.synchronize()
        mlp = tg.mlp_create(ctx, dims, Wd, tg.TGEMM_F32, 64)
        probs = torch.empty(batch, dims[-1], device="cuda")
        tg.mlp_forward(mlp, X, batch, probs)
        assert torch.allclose(probs.cpu(), torch.full((batch, dims[-1]), 1e-3), rtol=1e-6, atol=0)
        assert np.array_equal(_read(mlp, 0, 1, batch, dims[1]), np.full((batch, dims[1]), 0.5, np.float32))
        loss = tg.mlp_backward(mlp, y, None)
        assert abs(loss - np.log(1000.0)) < 1e-5
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)


def test_error_paths():
    ctx = tg.tgemm_create(0)
    try:
        W = [torch.zeros(8, 4, device="cuda")]
        torch.cuda.synchronize()
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_create(ctx, [8, 4], [torch.zeros(8, 4)], tg.TGEMM_F32, 16)
        assert e.value.code == tg.TGEMM_EUNPINNED
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_create(ctx, [8, 0], W, tg.TGEMM_F32, 16)
        assert e.value.code == tg.TGEMM_EARG
        mlp = tg.mlp_create(ctx, [8, 4], W, tg.TGEMM_F32, 16, hbm_budget=64)
        y = torch.zeros(4, dtype=torch.int32, device="cuda")
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_backward(mlp, y, None)
        assert e.value.code == tg.TGEMM_ESTATE
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_forward(mlp, torch.zeros(4, 8, device="cuda"), 4)
        assert e.value.code == tg.TGEMM_EBUDGET
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)


def test_seeded_random_networks(oracle):
    """Random depths, widths (aligned and odd), batches and tile sizes, every kernel shape: dW of every
    layer and the probabilities against the oracle at the fp32 bar.  The three layouts of the passes
    (forward NN, error NT, gradient TN) thereby meet ragged edges and ragged k-steps in all paths."""
    rnd = np.random.default_rng(20240612)
    for case in range(10):
        L = int(rnd.integers(1, 5))
        aligned = case % 2 == 0
        pick = (lambda lo, hi: 4 * int(rnd.integers(lo // 4 + 1, hi // 4))) if aligned else (lambda lo, hi: int(rnd.integers(lo, hi)))
        dims = [pick(8, 700) for _ in range(L + 1)]
        batch = pick(4, 600)
        T = int(rnd.choice([32, 64, 100, 128, 256, 1024]))
        cfg = int(rnd.integers(0, 4))
        announce("random mlp", case, dims, batch, T, "cfg", cfg)
        X, Ws, y = _net(dims, batch, seed=case)
        _, _, P = oracle.mlp_forward(X.numpy(), [w.numpy() for w in Ws])
        loss_ref, dW_ref, _ = oracle.mlp_backward(X.numpy(), [w.numpy() for w in Ws], y.numpy())
        ctx = tg.tgemm_create(0, kernel_config=cfg)
        try:
            Xd, yd = X.cuda(), y.cuda()
            Wd = [w.cuda() for w in Ws]
            dWd = [torch.zeros(w.shape, device="cuda") for w in Ws]
            probs = torch.empty(batch, dims[-1], device="cuda")
            torch.cuda.synchronize()
            mlp = tg.mlp_create(ctx, dims, Wd, tg.TGEMM_F32, T)
            tg.mlp_forward(mlp, Xd, batch, probs)
            loss = tg.mlp_backward(mlp, yd, dWd)
            assert rel_fro(probs.cpu().numpy(), P) <= TOL, (case, "probs")
            assert abs(loss - loss_ref) <= TOL * abs(loss_ref), (case, "loss")
            for l in range(L):
                assert rel_fro(dWd[l].cpu().numpy(), dW_ref[l]) <= TOL, (case, "dW", l)
            tg.mlp_destroy(mlp)
        finally:
            tg.tgemm_destroy(ctx)
