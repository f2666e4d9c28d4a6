"""GPU parity of the MLP passes with bias rows (mlp_set_bias) against the fp64 oracle: activations,
logits, probabilities, loss, errors, dW, db and one SGD step, fp32 (1e-5) and bf16 (1e-2), in-core
and with the weights out-of-core, batches that span one and several column-sum bands."""
import numpy as np
import pytest
import torch

from gpu_util import announce, rel_fro
from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs

pytestmark = pytest.mark.gpu

ACT_CODE = {"sigmoid": tg.TGEMM_ACT_SIGMOID, "tanh": tg.TGEMM_ACT_TANH}


def _np(t):
    return inputs.bf16_bits(t).copy() if t.dtype == torch.bfloat16 else t.numpy().copy()


def _f64(t):
    return t.to(torch.float64).numpy()


def _read(mlp, what, layer, rows, cols, dtype):
    out = torch.empty(rows, cols, dtype=dtype)
    tg.mlp_read(mlp, what, layer, out, rows * cols * out.element_size())
    return _f64(out)


def _budget(dims, batch, T, es, frac):
    L = len(dims) - 1
    ws = batch * 4 + batch * dims[L] * 4 + sum(batch * dims[l] * es * (2 if l < L else 1) for l in range(1, L + 1))
    ws += -(-batch // 512) * max(dims[1:]) * 4                              # column-sum scratch
    ws += 96 * max(-(-d // T) for d in dims) * 8
    n_tiles = sum((-(-dims[l] // T)) * (-(-dims[l + 1] // T)) for l in range(L))
    n_slots = max(int(frac * n_tiles), 2 * max(-(-d // T) for d in dims) + 2)
    return ws + n_slots * T * T * es


@pytest.mark.parametrize("ooc", [False, True])
@pytest.mark.parametrize("dtype,tdt,tol,lr", [(tg.TGEMM_F32, torch.float32, 1e-5, 0.01),
                                              (tg.TGEMM_BF16, torch.bfloat16, 1e-2, 20.0)])
@pytest.mark.parametrize("dims,batch,T,act", [([512, 1024, 768, 2000], 384, 256, "sigmoid"),
                                              ([200, 328, 264, 1000], 1100, 128, "tanh"),
                                              ([40, 30], 17, 16, "sigmoid")])
def test_passes_with_bias_rows(oracle, dims, batch, T, act, dtype, tdt, tol, lr, ooc):
    announce("mlp bias", dims, batch, T, act, "bf16" if dtype else "f32", "ooc" if ooc else "in-core")
    L = len(dims) - 1
    es = 2 if dtype == tg.TGEMM_BF16 else 4
    X = inputs.normal_matrix(1, batch, dims[0]).to(tdt)
    Ws = [inputs.normal_matrix(10 + l, dims[l], dims[l + 1], std=0.05).to(tdt) for l in range(L)]
    bs = [inputs.normal_matrix(20 + l, 1, dims[l + 1], std=0.5).reshape(-1).contiguous() for l in range(L)]
    y = inputs.labels(5, batch, dims[-1])
    Xn, Wn, bn = _np(X), [_np(w) for w in Ws], [b.numpy().copy() for b in bs]
    acts, z, P = oracle.mlp_forward(Xn, Wn, act, bs=bn)
    loss_ref, dW_ref, delta_ref, db_ref = oracle.mlp_backward(Xn, Wn, y.numpy(), act, bs=bn)
    _, _, P_nobias = oracle.mlp_forward(Xn, Wn, act)
    assert rel_fro(P_nobias, P) > 0.05                                       # the bias rows matter here

    ctx = tg.tgemm_create(0)
    try:
        Wx = [w.clone().pin_memory() if ooc else w.cuda() for w in Ws]
        bd = [b.cuda() for b in bs]
        dbd = [torch.full((dims[l + 1],), 7.0, device="cuda") for l in range(L)]
        Xd, yd = X.cuda(), y.cuda()
        probs = torch.empty(batch, dims[-1], device="cuda")
        dWd = [torch.zeros(w.shape, device="cuda") for w in Ws]
        torch.cuda.synchronize()
        mlp = tg.mlp_create(ctx, dims, Wx, dtype, T, hbm_budget=_budget(dims, batch, T, es, 0.4) if ooc else 0)
        tg.mlp_set_activation(mlp, ACT_CODE[act])
        tg.mlp_set_bias(mlp, bd, dbd)
        tg.mlp_forward(mlp, Xd, batch, probs)
        for l in range(1, L):
            assert rel_fro(_read(mlp, 0, l, batch, dims[l], tdt), acts[l]) <= tol, ("activation", l)
        assert rel_fro(_read(mlp, 1, 0, batch, dims[-1], torch.float32), z) <= tol
        assert rel_fro(probs.cpu().numpy(), P) <= tol
        loss = tg.mlp_backward(mlp, yd, dWd)
        assert abs(loss - loss_ref) <= tol * abs(loss_ref)
        for l in range(1, L + 1):
            assert rel_fro(_read(mlp, 2, l, batch, dims[l], tdt), delta_ref[l - 1]) <= tol, ("delta", l)
        for l in range(L):
            assert rel_fro(dWd[l].cpu().numpy(), dW_ref[l]) <= tol, ("dW", l)
            assert rel_fro(dbd[l].cpu().numpy(), db_ref[l]) <= tol, ("db", l)
            assert torch.equal(bd[l].cpu(), bs[l])                           # backward leaves b alone
        # one step: weights as in the bias-free tests, bias rows against b - lr db
        for t in dbd:
            t.fill_(7.0)
        loss2 = tg.mlp_step(mlp, Xd, yd, batch, lr)
        tg.tgemm_sync(ctx)
        assert abs(loss2 - loss_ref) <= tol * abs(loss_ref)
        for l in range(L):
            upd = _f64(Wx[l].cpu()) - _f64(Ws[l])
            half_ulp = 2.0 ** -9 if dtype == tg.TGEMM_BF16 else 2.0 ** -24
            slack = np.linalg.norm(_f64(Wx[l].cpu())) * half_ulp / np.linalg.norm(lr * dW_ref[l])
            assert rel_fro(upd, -lr * dW_ref[l]) <= tol + slack, ("update", l)
            updb = _f64(bd[l].cpu()) - _f64(bs[l])
            slack_b = np.linalg.norm(_f64(bd[l].cpu())) * 2.0 ** -24 / np.linalg.norm(lr * db_ref[l])
            assert rel_fro(updb, -lr * db_ref[l]) <= tol + slack_b, ("bias update", l)
            assert rel_fro(dbd[l].cpu().numpy(), db_ref[l]) <= tol, ("db of the step", l)
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)


def test_removing_the_bias_rows_and_errors(oracle):
    dims, batch, T = [96, 160, 64], 48, 32
    X = inputs.normal_matrix(1, batch, dims[0])
    Ws = [inputs.normal_matrix(10 + l, dims[l], dims[l + 1], std=0.1) for l in range(2)]
    bs = [inputs.normal_matrix(20 + l, 1, dims[l + 1], std=0.5).reshape(-1).contiguous() for l in range(2)]
    _, _, P_b = oracle.mlp_forward(X.numpy(), [w.numpy() for w in Ws], bs=[b.numpy() for b in bs])
    _, _, P_0 = oracle.mlp_forward(X.numpy(), [w.numpy() for w in Ws])
    ctx = tg.tgemm_create(0)
    try:
        Wd, bd, Xd = [w.cuda() for w in Ws], [b.cuda() for b in bs], X.cuda()
        yd = inputs.labels(5, batch, dims[-1]).cuda()
        probs = torch.empty(batch, dims[-1], device="cuda")
        torch.cuda.synchronize()
        mlp = tg.mlp_create(ctx, dims, Wd, tg.TGEMM_F32, T)
        tg.mlp_forward(mlp, Xd, batch, probs)
        assert rel_fro(probs.cpu().numpy(), P_0) <= 1e-5
        tg.mlp_set_bias(mlp, bd)
        with pytest.raises(tg.TgemmError) as e:                              # the pending forward pass is gone
            tg.mlp_backward(mlp, yd, None)
        assert e.value.code == tg.TGEMM_ESTATE
        tg.mlp_forward(mlp, Xd, batch, probs)
        assert rel_fro(probs.cpu().numpy(), P_b) <= 1e-5
        tg.mlp_set_bias(mlp, None)
        tg.mlp_forward(mlp, Xd, batch, probs)
        assert rel_fro(probs.cpu().numpy(), P_0) <= 1e-5
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_set_bias(mlp, [bd[0], None])
        assert e.value.code == tg.TGEMM_EARG
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_set_bias(mlp, [bd[0], bs[1]])                             # host memory
        assert e.value.code == tg.TGEMM_EARG
        with pytest.raises(tg.TgemmError) as e:
            tg.mlp_set_bias(mlp, None, bd)
        assert e.value.code == tg.TGEMM_EARG
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)
