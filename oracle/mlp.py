"""MLP oracle (test infrastructure only), fp64 throughout.

Section 2 of the paper reduces training to matrix products: the forward pass
feeds each layer with (previous layer's output) x (parameter matrix)
(equation 1); the backward pass forms the error derivative with respect to
the parameters (equation 3) and with respect to the layer outputs (equation
4), both again matrix products; parameters are updated after the two passes.
The equations themselves are not printed, so the textbook forms are taken:

    A_0 = X                               [batch x n_0]
    Z_l = A_{l-1} W_l                     l = 1..L      (no bias)
    A_l = sigmoid(Z_l)                    l < L
    P   = softmax over each row of Z_L;   loss = -mean_b log P[b, y_b]
    D_L = (P - onehot(y)) / batch
    dW_l     = A_{l-1}^T D_l
    dA_{l-1} = D_l W_l^T ;   D_{l-1} = dA_{l-1} * A_{l-1} * (1 - A_{l-1})
    W_l <- W_l - lr * dW_l               (every dW from the pre-update weights)

numpy's fp64 matmul is the library primitive used for the products.
"""
import numpy as np

from .gemm import bf16_to_f64


def _f64(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return bf16_to_f64(a).reshape(a.shape)
    return a.astype(np.float64)


def mlp_forward(X, Ws):
    """Returns (acts, logits, probs): acts[l] is the input of layer l+1 (acts[0] = X)."""
    a = _f64(X)
    acts = [a]
    L = len(Ws)
    z = None
    for l, W in enumerate(Ws):
        z = a @ _f64(W)
        if l < L - 1:
            a = 1.0 / (1.0 + np.exp(-z))
            acts.append(a)
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    probs = e / e.sum(axis=1, keepdims=True)
    return acts, z, probs


def mlp_loss(X, Ws, y):
    _, z, _ = mlp_forward(X, Ws)
    y = np.asarray(y, dtype=np.int64)
    zmax = z.max(axis=1)
    lse = zmax + np.log(np.exp(z - zmax[:, None]).sum(axis=1))
    return float(np.mean(lse - z[np.arange(z.shape[0]), y]))


def mlp_backward(X, Ws, y):
    """Returns (loss, dWs, deltas): deltas[l] is the error at the output of layer l+1."""
    acts, z, probs = mlp_forward(X, Ws)
    y = np.asarray(y, dtype=np.int64)
    B = z.shape[0]
    loss = mlp_loss(X, Ws, y)
    d = probs.copy()
    d[np.arange(B), y] -= 1.0
    d /= B
    L = len(Ws)
    dWs = [None] * L
    deltas = [None] * L
    for l in range(L - 1, -1, -1):
        deltas[l] = d
        dWs[l] = acts[l].T @ d
        if l > 0:
            dA = d @ _f64(Ws[l]).T
            d = dA * acts[l] * (1.0 - acts[l])
    return loss, dWs, deltas


def mlp_step(X, Ws, y, lr):
    """One SGD step.  Returns (loss before the update, new weights in fp64, dWs)."""
    loss, dWs, _ = mlp_backward(X, Ws, y)
    new = [_f64(W) - lr * g for W, g in zip(Ws, dWs)]
    return loss, new, dWs
