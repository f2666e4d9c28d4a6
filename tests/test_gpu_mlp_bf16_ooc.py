"""GPU parity of the MLP passes in the remaining modes -- bf16 storage with fp32 accumulation, and
out-of-core (weights in pinned host memory, staged through the bounded HBM weight-tile cache) --
against the fp64 oracle fed the same bit patterns.

Bars: fp32 out-of-core 1e-5 (and bitwise equal to the in-core run); bf16 1e-2 relative Frobenius on
activations, logits, probabilities, loss, errors and dW.  The weight update is checked on
W_new - W_old with a learning rate large enough that the update dominates the rounding of W_new
into its storage format (half an ulp per entry, allowed on top of the bar)."""
import numpy as np
import pytest
import torch

from gpu_util import announce, rel_fro
from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs

pytestmark = pytest.mark.gpu


def _net(dims, batch, dtype, std=0.05, seed=0):
    X = inputs.normal_matrix(seed + 1, batch, dims[0]).to(dtype)
    Ws = [inputs.normal_matrix(seed + 10 + l, dims[l], dims[l + 1], std=std).to(dtype) for l in range(len(dims) - 1)]
    y = inputs.labels(seed + 5, batch, dims[-1])
    return X, Ws, y


def _np(t):
    return inputs.bf16_bits(t) if t.dtype == torch.bfloat16 else t.numpy()


def _f64(t):
    return t.to(torch.float64).numpy()


def _read(mlp, what, layer, rows, cols, dtype):
    out = torch.empty(rows, cols, dtype=dtype)
    tg.mlp_read(mlp, what, layer, out, rows * cols * out.element_size())
    return _f64(out)


def _workspace_bytes(dims, batch, es, T, ooc):
    L = len(dims) - 1
    total = batch * 4 + batch * dims[L] * 4
    for l in range(1, L + 1):
        total += batch * dims[l] * es * (2 if l < L else 1)
    if ooc:
        total += 32 * max(-(-d // T) for d in dims) * 8
    return total


def _check_passes(oracle, mlp, dims, batch, X, Ws, y, Wd, Xd, yd, dtype, tol, lr):
    L = len(Ws)
    tdt = X.dtype
    acts, z, P = oracle.mlp_forward(_np(X), [_np(w) for w in Ws])
    loss_ref, dW_ref, delta_ref = oracle.mlp_backward(_np(X), [_np(w) for w in Ws], y.numpy())
    probs = torch.empty(batch, dims[-1], device="cuda")
    torch.cuda.synchronize()
    tg.mlp_forward(mlp, Xd, batch, probs)
    for l in range(1, L):
        assert rel_fro(_read(mlp, 0, l, batch, dims[l], tdt), acts[l]) <= tol, ("activation", l)
    assert rel_fro(_read(mlp, 1, 0, batch, dims[-1], torch.float32), z) <= tol
    assert rel_fro(probs.cpu().numpy(), P) <= tol
    dWd = [torch.zeros(w.shape, device="cuda") for w in Ws]
    torch.cuda.synchronize()
    loss = tg.mlp_backward(mlp, yd, dWd)
    assert abs(loss - loss_ref) <= tol * abs(loss_ref)
    for l in range(1, L + 1):
        assert rel_fro(_read(mlp, 2, l, batch, dims[l], tdt), delta_ref[l - 1]) <= tol, ("delta", l)
    for l in range(L):
        assert rel_fro(dWd[l].cpu().numpy(), dW_ref[l]) <= tol, ("dW", l)
        assert torch.equal(Wd[l].cpu(), Ws[l])                       # backward leaves W alone
    loss2 = tg.mlp_step(mlp, Xd, yd, batch, lr)
    assert abs(loss2 - loss_ref) <= tol * abs(loss_ref)
    for l in range(L):
        new = Wd[l].cpu()
        # W_new - W_old against -lr * dW; storing W_new rounds it to the weight format, which adds up
        # to half an ulp of W_new per entry (2^-9 relative for bf16, 2^-24 for fp32) on top of the bar
        upd = _f64(new) - _f64(Ws[l])
        half_ulp = 2.0 ** -9 if dtype == tg.TGEMM_BF16 else 2.0 ** -24
        slack = np.linalg.norm(_f64(new)) * half_ulp / np.linalg.norm(lr * dW_ref[l])
        assert slack < 0.05, slack                                      # the update dominates the rounding
        assert rel_fro(upd, -lr * dW_ref[l]) <= tol + slack, ("update", l)


@pytest.mark.parametrize("dims,batch,T", [([64, 96, 80, 50], 33, 32), ([512, 1024, 768, 2000], 384, 256),
                                          ([40, 30], 17, 16), ([256, 512, 264, 1000], 200, 128)])
@pytest.mark.parametrize("cfg", [0, 3, 4])      # automatic; large tiles (direct-to-LDS kernel where it applies); large, register-staged
def test_bf16_in_core(oracle, dims, batch, T, cfg):
    announce("mlp bf16 in-core", dims, batch, T, "cfg", cfg)
    X, Ws, y = _net(dims, batch, torch.bfloat16)
    ctx = tg.tgemm_create(0, kernel_config=cfg)
    try:
        Wd = [w.cuda() for w in Ws]
        Xd, yd = X.cuda(), y.cuda()
        torch.cuda.synchronize()
        mlp = tg.mlp_create(ctx, dims, Wd, tg.TGEMM_BF16, T)
        _check_passes(oracle, mlp, dims, batch, X, Ws, y, Wd, Xd, yd, tg.TGEMM_BF16, 1e-2, lr=20.0)
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)


@pytest.mark.parametrize("dtype,tdt,tol,lr", [(tg.TGEMM_F32, torch.float32, 1e-5, 0.01),
                                              (tg.TGEMM_BF16, torch.bfloat16, 1e-2, 20.0)])
@pytest.mark.parametrize("dims,batch,T,frac", [([512, 1024, 768, 2000], 384, 256, 0.4),
                                               ([300, 520, 1000], 100, 128, 0.6),
                                               ([512, 2048, 2048, 16384], 512, 256, 0.35)])
@pytest.mark.parametrize("cfg", [0, 3])
def test_out_of_core(oracle, dims, batch, T, frac, dtype, tdt, tol, lr, cfg):
    announce("mlp ooc", dims, batch, T, frac, "bf16" if dtype else "f32", "cfg", cfg)
    X, Ws, y = _net(dims, batch, tdt)
    es = 2 if dtype == tg.TGEMM_BF16 else 4
    n_tiles = sum((-(-dims[l] // T)) * (-(-dims[l + 1] // T)) for l in range(len(Ws)))
    max_tiles = max(-(-d // T) for d in dims)
    n_slots = max(int(frac * n_tiles), 2 * max_tiles + 2)
    assert n_slots < n_tiles                                         # genuinely out-of-core
    budget = _workspace_bytes(dims, batch, es, T, True) + n_slots * T * T * es
    ctx = tg.tgemm_create(0, kernel_config=cfg)
    try:
        Wp = [w.clone().pin_memory() for w in Ws]
        Xd, yd = X.cuda(), y.cuda()
        torch.cuda.synchronize()
        with pytest.raises(tg.TgemmError) as e:                      # budget below the minimum working set
            small = tg.mlp_create(ctx, dims, Wp, dtype, T, hbm_budget=_workspace_bytes(dims, batch, es, T, True))
            tg.mlp_forward(small, Xd, batch)
        assert e.value.code == tg.TGEMM_EBUDGET
        tg.mlp_destroy(small)
        mlp = tg.mlp_create(ctx, dims, Wp, dtype, T, hbm_budget=budget)
        _check_passes(oracle, mlp, dims, batch, X, Ws, y, Wp, Xd, yd, dtype, tol, lr)
        st = tg.tgemm_last_stats(ctx)                                # stats of the step
        assert st["in_core"] == 0 and st["n_slots"] == n_slots
        w_bytes = sum(w.numel() for w in Ws) * es
        assert st["d2h_bytes"] == w_bytes                            # every updated tile written back once
        assert st["evictions"] > 0 and st["h2d_bytes"] >= w_bytes - n_slots * T * T * es
        # same step in-core from the same starting weights: the host weights must hold the same bits
        Wd = [w.cuda() for w in Ws]
        torch.cuda.synchronize()
        ref = tg.mlp_create(ctx, dims, Wd, dtype, T)
        tg.mlp_step(ref, Xd, yd, batch, lr)
        for l in range(len(Ws)):
            assert torch.equal(Wd[l].cpu(), Wp[l]), ("in-core vs out-of-core weights", l)
        # a second step starts from the updated host weights and a warm cache
        l_ooc = tg.mlp_step(mlp, Xd, yd, batch, lr)
        l_ic = tg.mlp_step(ref, Xd, yd, batch, lr)
        assert l_ooc == l_ic
        for l in range(len(Ws)):
            assert torch.equal(Wd[l].cpu(), Wp[l]), ("second step", l)
        tg.mlp_destroy(ref)
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)
