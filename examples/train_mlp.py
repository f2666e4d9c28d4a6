"""Trains a small MLP on synthetic Gaussian blobs with the C ABI's MLP calls (through the ctypes
binding): bias rows, momentum, tanh hidden layers, mini-batches.  Every product, activation, error and
update runs in the library's HIP kernels; torch only allocates the device buffers and draws the data.

    python examples/train_mlp.py [--bf16 [--master-weights]] [--epochs N]

Prints the mean loss per epoch and the accuracy on held-out points."""
import argparse
import os
import sys

import torch

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
from paper_1511_04348_amd import binding as tg  # noqa: E402


def blobs(n, n_classes, dim, gen):
    centres = torch.randn(n_classes, dim, generator=gen) * 3.0
    y = torch.randint(0, n_classes, (n,), generator=gen)
    x = centres[y] + torch.randn(n, dim, generator=gen)
    return x, y.to(torch.int32)


def run(bf16=False, epochs=6, batch=512, quiet=False, master_weights=False):
    gen = torch.Generator().manual_seed(0)
    dims = [64, 256, 128, 16]
    x, y = blobs(20 * batch, dims[-1], dims[0], gen)
    xt, yt, x, y = x[: 4 * batch], y[: 4 * batch], x[4 * batch:], y[4 * batch:]      # held-out / training split
    dt = torch.bfloat16 if bf16 else torch.float32
    W = [(torch.randn(dims[l], dims[l + 1], generator=gen) * (1.0 / dims[l] ** 0.5)).to(dt).cuda() for l in range(3)]
    b = [torch.zeros(dims[l + 1], device="cuda") for l in range(3)]
    V = [torch.zeros(dims[l], dims[l + 1], device="cuda") for l in range(3)]
    Vb = [torch.zeros(dims[l + 1], device="cuda") for l in range(3)]
    xd, yd, xtd = x.to(dt).cuda(), y.cuda(), xt.to(dt).cuda()
    torch.cuda.synchronize()

    ctx = tg.tgemm_create(0)
    mlp = tg.mlp_create(ctx, dims, W, tg.TGEMM_BF16 if bf16 else tg.TGEMM_F32, 128)
    tg.mlp_set_activation(mlp, tg.TGEMM_ACT_TANH)
    tg.mlp_set_bias(mlp, b)
    tg.mlp_set_momentum(mlp, 0.9, V, Vb)
    if bf16 and master_weights:      # fp32 master copies keep the small steps; the bf16 weights are their image
        M = [w.float() for w in W]
        tg.mlp_set_master_weights(mlp, M)
    elif bf16:                       # without them, stochastic rounding keeps the steps in expectation
        tg.mlp_set_rounding(mlp, tg.TGEMM_ROUND_STOCHASTIC, 1)
    losses = []
    n_batches = x.shape[0] // batch
    for epoch in range(epochs):
        total = 0.0
        for i in range(n_batches):
            xb = xd[i * batch:(i + 1) * batch]
            yb = yd[i * batch:(i + 1) * batch]
            total += tg.mlp_step(mlp, xb, yb, batch, 0.02)
        losses.append(total / n_batches)
        if not quiet:
            print("epoch %d  mean loss %.4f" % (epoch, losses[-1]))
    probs = torch.empty(xt.shape[0], dims[-1], device="cuda")
    tg.mlp_forward(mlp, xtd, xt.shape[0], probs)
    tg.tgemm_sync(ctx)
    acc = float((probs.argmax(dim=1).cpu() == yt.to(torch.int64)).float().mean())
    if not quiet:
        print("held-out accuracy %.3f" % acc)
    tg.mlp_destroy(mlp)
    tg.tgemm_destroy(ctx)
    return losses, acc


if __name__ == "__main__":
    ap = argparse.ArgumentParser()
    ap.add_argument("--bf16", action="store_true")
    ap.add_argument("--master-weights", action="store_true", help="with --bf16: fp32 master copies instead of stochastic rounding")
    ap.add_argument("--epochs", type=int, default=6)
    a = ap.parse_args()
    run(bf16=a.bf16, epochs=a.epochs, master_weights=a.master_weights)
