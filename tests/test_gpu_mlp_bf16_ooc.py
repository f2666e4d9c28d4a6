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


def _step_sweep(dims, T):
    """Weight tiles in the order one training step touches them."""
    cd = lambda a: -(-a // T)
    L = len(dims) - 1
    seq = [(l, k, j) for l in range(1, L + 1) for j in range(cd(dims[l])) for k in range(cd(dims[l - 1]))]
    seq += [(l, r, c) for l in range(L, 0, -1) for r in range(cd(dims[l - 1])) for c in range(cd(dims[l]))]
    return seq


def _workspace_bytes(dims, batch, es, T, ooc):
    L = len(dims) - 1
    total = batch * 4 + batch * dims[L] * 4
    for l in range(1, L + 1):
        total += batch * dims[l] * es * (2 if l < L else 1)
    if ooc:
        total += 96 * max(-(-d // T) for d in dims) * 8
    return total


def _check_passes(oracle, mlp, dims, batch, X, Ws, y, Wd, Xd, yd, dtype, tol, lr, act="sigmoid"):
    L = len(Ws)
    tdt = X.dtype
    acts, z, P = oracle.mlp_forward(_np(X), [_np(w) for w in Ws], act)
    loss_ref, dW_ref, delta_ref = oracle.mlp_backward(_np(X), [_np(w) for w in Ws], y.numpy(), act=act)
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
        # steady state: the cache evicts by next use in the step's fixed sweep (forward: tile columns
        # layer by layer; backward: tile rows, layers reversed) and must not miss more often than
        # strict LRU would on the same sweep, nor less often than the tiles that cannot fit
        tg.mlp_step(mlp, Xd, yd, batch, lr)
        st = tg.tgemm_last_stats(ctx)
        sweep = _step_sweep(dims, T)
        _, lru = oracle.lru_simulate(sweep * 4, n_slots)
        _, lru3 = oracle.lru_simulate(sweep * 3, n_slots)
        lru_per_step = lru["misses"] - lru3["misses"]
        print("misses per step", st["misses"], "strict LRU", lru_per_step, "tiles", n_tiles, "slots", n_slots)
        assert st["hits"] + st["misses"] == 2 * n_tiles
        assert n_tiles - n_slots <= st["misses"] <= lru_per_step
        tg.mlp_destroy(ref)
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)


@pytest.mark.parametrize("dtype,tdt", [(tg.TGEMM_F32, torch.float32), (tg.TGEMM_BF16, torch.bfloat16)])
def test_deferred_writeback_gives_the_same_weights(dtype, tdt):
    """With deferred write-back a step returns while its updated tiles still travel to the host; they
    must be ordered before the next step's update of the same slot and before any re-fetch, so after
    tgemm_sync the host weights and the losses equal those of the synchronous mode bit for bit."""
    dims, batch, T = [512, 1024, 768, 2000], 384, 256
    announce("mlp ooc deferred write-back", dims, batch, T, "bf16" if dtype else "f32")
    X, Ws, y = _net(dims, batch, tdt)
    es = 2 if dtype == tg.TGEMM_BF16 else 4
    n_tiles = sum((-(-dims[l] // T)) * (-(-dims[l + 1] // T)) for l in range(len(Ws)))
    n_slots = max(int(0.4 * n_tiles), 2 * max(-(-d // T) for d in dims) + 2)
    budget = _workspace_bytes(dims, batch, es, T, True) + n_slots * T * T * es
    Xd, yd = X.cuda(), y.cuda()
    torch.cuda.synchronize()
    results = []
    for deferred in (0, 1):
        ctx = tg.tgemm_create(0, deferred_writeback=deferred)
        try:
            Wp = [w.clone().pin_memory() for w in Ws]
            mlp = tg.mlp_create(ctx, dims, Wp, dtype, T, hbm_budget=budget)
            losses = [tg.mlp_step(mlp, Xd, yd, batch, 0.5) for _ in range(4)]
            tg.tgemm_sync(ctx)
            results.append((losses, [w.clone() for w in Wp]))
            tg.mlp_destroy(mlp)
        finally:
            tg.tgemm_destroy(ctx)
    assert results[0][0] == results[1][0]
    for l in range(len(Ws)):
        assert torch.equal(results[0][1][l], results[1][1][l]), ("weights", l)
        assert not torch.equal(results[0][1][l], Ws[l])              # the steps did change them


ACT_CODE = {"sigmoid": tg.TGEMM_ACT_SIGMOID, "tanh": tg.TGEMM_ACT_TANH, "relu": tg.TGEMM_ACT_RELU}


def _dyadic_net(dims, batch, dtype):
    """Small integers for X and small integers / 32 for the weights: every hidden pre-activation is a
    dyadic rational that fp32 and fp64 both hold exactly, so the GPU and the oracle take the same
    relu on/off decisions (a decision taken in different precisions could flip at a pre-activation
    within rounding of zero, and one flipped unit is far above the fp32 tolerance)."""
    X = inputs.int_matrix(1, batch, dims[0]).to(dtype)
    Ws = [(inputs.int_matrix(10 + l, dims[l], dims[l + 1]) / 32.0).to(dtype) for l in range(len(dims) - 1)]
    return X, Ws, inputs.labels(5, batch, dims[-1])


@pytest.mark.parametrize("ooc", [False, True])
@pytest.mark.parametrize("dtype,tdt,tol,lr", [(tg.TGEMM_F32, torch.float32, 1e-5, 0.01),
                                              (tg.TGEMM_BF16, torch.bfloat16, 1e-2, 20.0)])
@pytest.mark.parametrize("act", ["tanh", "relu"])
def test_other_activations(oracle, act, dtype, tdt, tol, lr, ooc):
    """Forward, backward and step with tanh / relu hidden layers against the oracle, in-core and with
    the weights out-of-core (section 2 fixes only that the passes are matrix products)."""
    dims, batch, T = [512, 1024, 768, 2000], 384, 256
    announce("mlp activation", act, "bf16" if dtype else "f32", "ooc" if ooc else "in-core")
    if act == "relu":
        X, Ws, y = _dyadic_net(dims, batch, tdt)
    else:
        X, Ws, y = _net(dims, batch, tdt)
    es = 2 if dtype == tg.TGEMM_BF16 else 4
    ctx = tg.tgemm_create(0, kernel_config=3 if dtype == tg.TGEMM_BF16 else 0)
    try:
        Xd, yd = X.cuda(), y.cuda()
        if ooc:
            n_tiles = sum((-(-dims[l] // T)) * (-(-dims[l + 1] // T)) for l in range(len(Ws)))
            n_slots = max(int(0.4 * n_tiles), 2 * max(-(-d // T) for d in dims) + 2)
            Wx = [w.clone().pin_memory() for w in Ws]
            budget = _workspace_bytes(dims, batch, es, T, True) + n_slots * T * T * es
        else:
            Wx = [w.cuda() for w in Ws]
            budget = 0
        torch.cuda.synchronize()
        mlp = tg.mlp_create(ctx, dims, Wx, dtype, T, hbm_budget=budget)
        tg.mlp_set_activation(mlp, ACT_CODE[act])
        _check_passes(oracle, mlp, dims, batch, X, Ws, y, Wx, Xd, yd, dtype, tol, lr, act=act)
        # changing the function discards the pending forward pass
        tg.mlp_forward(mlp, Xd, batch)
        tg.mlp_set_activation(mlp, tg.TGEMM_ACT_SIGMOID)
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_backward(mlp, yd, None)
        assert e.value.code == tg.TGEMM_ESTATE
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_set_activation(mlp, 7)
        assert e.value.code == tg.TGEMM_EARG
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)
