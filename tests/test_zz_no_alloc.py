"""mlp_forward_static (the entry point that allocates nothing: its activations and logits live in a
static device array) against mlp_forward, through the C ABI.

Both run the same kernels on the same shapes, so the probabilities must agree bit for bit; they are
also held to the oracle at the bar of the forward pass (fp32 1e-5, bf16 1e-2).  Two calls in a row on
one object, the second with a smaller batch (the array still holds the first call's contents), fp32
and bf16, with and without bias rows; the device's free memory does not change over the calls; a
batch beyond the array is refused before any work."""
import numpy as np
import pytest
import torch

from gpu_util import announce, rel_fro
from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs

pytestmark = pytest.mark.gpu


def _net(dims, batch, dt, std=0.05):
    X = inputs.normal_matrix(1, batch, dims[0]).to(dt)
    Ws = [inputs.normal_matrix(10 + l, dims[l], dims[l + 1], std=std).to(dt) for l in range(len(dims) - 1)]
    return X, Ws


def _np(t):
    return inputs.bf16_bits(t) if t.dtype == torch.bfloat16 else t.numpy()


@pytest.mark.parametrize("dt,tol", [(torch.float32, 1e-5), (torch.bfloat16, 1e-2)])
@pytest.mark.parametrize("bias", [False, True])
def test_static_forward_equals_allocating_forward(oracle, dt, tol, bias):
    dims, T = [300, 520, 410, 130], 128
    batches = [200, 70]                       # the second call is smaller and finds the first one's data in the array
    announce("mlp_forward_static", dt, "bias" if bias else "no bias", dims, batches)
    X, Ws = _net(dims, max(batches), dt)
    bs = [inputs.normal_matrix(30 + l, 1, dims[l + 1], std=0.1).view(-1) for l in range(3)] if bias else None
    code = tg.TGEMM_BF16 if dt == torch.bfloat16 else tg.TGEMM_F32
    ctx = tg.tgemm_create(0)
    try:
        Xd = X.cuda()
        Wd = [w.cuda() for w in Ws]
        bd = [b.cuda() for b in bs] if bias else None
        torch.cuda.synchronize()
        ref_net = tg.mlp_create(ctx, dims, Wd, code, T)          # goes through mlp_forward (allocates its workspaces)
        static_net = tg.mlp_create(ctx, dims, Wd, code, T)       # never allocates a workspace
        if bias:
            tg.mlp_set_bias(ref_net, bd)
            tg.mlp_set_bias(static_net, bd)
        outs = [(torch.empty(b, dims[-1], device="cuda"), torch.full((b, dims[-1]), -1.0, device="cuda")) for b in batches]
        torch.cuda.synchronize()
        for b, (p_ref, _) in zip(batches, outs):
            tg.mlp_forward(ref_net, Xd, b, p_ref)
        free_before, _ = torch.cuda.mem_get_info()
        for b, (_, p_static) in zip(batches, outs):
            tg.mlp_forward_static(static_net, Xd, b, p_static)
        free_after, _ = torch.cuda.mem_get_info()
        assert free_after == free_before, "mlp_forward_static changed the device's free memory"
        for b, (p_ref, p_static) in zip(batches, outs):
            assert torch.equal(p_ref, p_static), ("bitwise", b)
            _, _, P = oracle.mlp_forward(_np(X[:b]), [_np(w) for w in Ws], bs=[v.numpy() for v in bs] if bias else None)
            err = rel_fro(p_static.cpu().numpy(), P)
            print("batch", b, "rel fro vs oracle", err, flush=True)
            assert err <= tol, (b, err)
        # the object that only ever ran the static call has no pass state: backward has nothing to start from
        y = inputs.labels(5, batches[0], dims[-1]).cuda()
        with pytest.raises(tg.TgemmError) as ei:
            tg.mlp_backward(static_net, y)
        assert ei.value.code == tg.TGEMM_ESTATE
        tg.mlp_destroy(ref_net)
        tg.mlp_destroy(static_net)
    finally:
        tg.tgemm_destroy(ctx)


def test_static_forward_refuses_what_does_not_fit():
    dims, T = [256, 4096, 4096], 256
    announce("mlp_forward_static limits")
    Ws = [torch.zeros(dims[l], dims[l + 1], device="cuda") for l in range(2)]
    ctx = tg.tgemm_create(0)
    try:
        net = tg.mlp_create(ctx, dims, Ws, tg.TGEMM_F32, T)
        per_row = dims[1] * 4 + dims[2] * 4
        fits = (32 << 20) // per_row                               # 1024 rows fill the array exactly
        assert fits * per_row == 32 << 20
        X = torch.zeros(fits + 1, dims[0], device="cuda")
        probs = torch.empty(fits + 1, dims[-1], device="cuda")
        torch.cuda.synchronize()
        tg.mlp_forward_static(net, X, fits, probs)                 # the maximum size
        torch.cuda.synchronize()
        assert np.allclose(probs[:fits].cpu().numpy(), 1.0 / dims[-1], rtol=1e-6)   # zero weights: uniform rows
        with pytest.raises(tg.TgemmError) as ei:
            tg.mlp_forward_static(net, X, fits + 1, probs)
        assert ei.value.code == tg.TGEMM_EBUDGET
        with pytest.raises(tg.TgemmError) as ei:
            tg.mlp_forward_static(net, X, 8, None)
        assert ei.value.code == tg.TGEMM_EARG
        tg.mlp_destroy(net)
        # out-of-core weights are refused
        Wh = [torch.zeros(dims[l], dims[l + 1], pin_memory=True) for l in range(2)]
        net = tg.mlp_create(ctx, dims, Wh, tg.TGEMM_F32, T, hbm_budget=10 ** 9)
        with pytest.raises(tg.TgemmError) as ei:
            tg.mlp_forward_static(net, X, 8, probs)
        assert ei.value.code == tg.TGEMM_EARG
        tg.mlp_destroy(net)
    finally:
        tg.tgemm_destroy(ctx)
