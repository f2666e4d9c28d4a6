"""MLP oracle (test infrastructure only), fp64 throughout.

Section 2 of the paper reduces training to matrix products: the forward pass
feeds each layer with (previous layer's output) x (parameter matrix)
(equation 1); the backward pass forms the error derivative with respect to
the parameters (equation 3) and with respect to the layer outputs (equation
4), both again matrix products; parameters are updated after the two passes.
The equations themselves are not printed, so the textbook forms are taken:

    A_0 = X                               [batch x n_0]
    Z_l = A_{l-1} W_l  (+ 1 b_l^T)        l = 1..L      (bias rows b_l optional: bs=None means none)
    A_l = act(Z_l)                        l < L      (act: sigmoid by default; tanh, relu)
    P   = softmax over each row of Z_L;   loss = -mean_b log P[b, y_b]
    D_L = (P - onehot(y)) / batch
    dW_l     = A_{l-1}^T D_l ;   db_l = 1^T D_l  (column sums over the batch)
    dA_{l-1} = D_l W_l^T ;   D_{l-1} = dA_{l-1} * act'(Z_{l-1})
             act' = A (1 - A) for the sigmoid, 1 - A^2 for tanh, [Z > 0] for relu
    W_l <- W_l - lr * dW_l ;  b_l <- b_l - lr * db_l     (every gradient from the pre-update values)
    with momentum:  V_l <- mu V_l + dW_l ;  W_l <- W_l - lr V_l
    with fp32 master copies M_l of bf16 weights:  M_l <- fp32(M_l - lr dW_l) ;  W_l <- bf16(M_l),
                    every product of the two passes taken with the bf16 W_l

numpy's fp64 matmul is the library primitive used for the products.

mlp_rows evaluates the per-sample quantities (activations, logits, probabilities, errors) for a
subset of the batch rows: each of them depends on that sample's row alone, apart from the 1 / batch
in D_L, which is passed in.  It exists for networks whose weight matrices are too large to widen to
fp64 whole (a 17 GB bf16 matrix would become 69 GB): its products walk the weight matrix in blocks of
the OUTPUT index, so every output entry is still one fp64 dot product over the whole inner dimension.
"""
import numpy as np

from .gemm import bf16_to_f64
from .rounding import stochastic_round_matrix, round_bf16_nearest


def _f64(a):
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return bf16_to_f64(a).reshape(a.shape)
    return a.astype(np.float64)


def _act(z, act):
    if act == "sigmoid":
        return 1.0 / (1.0 + np.exp(-z))
    if act == "tanh":
        return np.tanh(z)
    if act == "relu":
        return np.where(z > 0.0, z, 0.0)
    raise ValueError(act)


def _act_slope(z, a, act):
    """d act / d z at pre-activation z (a = act(z))."""
    if act == "sigmoid":
        return a * (1.0 - a)
    if act == "tanh":
        return 1.0 - a * a
    if act == "relu":
        return (z > 0.0).astype(np.float64)
    raise ValueError(act)


def mlp_forward(X, Ws, act="sigmoid", return_pre=False, bs=None):
    """Returns (acts, logits, probs): acts[l] is the input of layer l+1 (acts[0] = X).
    With return_pre also the hidden pre-activations Z_l as a fourth value."""
    a = _f64(X)
    acts = [a]
    pre = [None]
    L = len(Ws)
    z = None
    for l, W in enumerate(Ws):
        z = a @ _f64(W)
        if bs is not None:
            z = z + np.asarray(bs[l], dtype=np.float64)[None, :]
        if l < L - 1:
            a = _act(z, act)
            acts.append(a)
            pre.append(z)
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    probs = e / e.sum(axis=1, keepdims=True)
    if return_pre:
        return acts, z, probs, pre
    return acts, z, probs


def mlp_loss(X, Ws, y, act="sigmoid", bs=None):
    _, z, _ = mlp_forward(X, Ws, act, bs=bs)
    y = np.asarray(y, dtype=np.int64)
    zmax = z.max(axis=1)
    lse = zmax + np.log(np.exp(z - zmax[:, None]).sum(axis=1))
    return float(np.mean(lse - z[np.arange(z.shape[0]), y]))


def mlp_backward(X, Ws, y, act="sigmoid", bs=None):
    """Returns (loss, dWs, deltas): deltas[l] is the error at the output of layer l+1.
    With bias rows (bs) a fourth value: the bias gradients dbs."""
    acts, z, probs, pre = mlp_forward(X, Ws, act, return_pre=True, bs=bs)
    y = np.asarray(y, dtype=np.int64)
    B = z.shape[0]
    loss = mlp_loss(X, Ws, y, act, bs=bs)
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
            d = dA * _act_slope(pre[l], acts[l], act)
    if bs is not None:
        return loss, dWs, deltas, [dl.sum(axis=0) for dl in deltas]
    return loss, dWs, deltas


def mlp_step(X, Ws, y, lr, act="sigmoid", bs=None):
    """One SGD step.  Returns (loss before the update, new weights in fp64, dWs); with bias rows
    (bs) also the new bias rows and their gradients."""
    if bs is None:
        loss, dWs, _ = mlp_backward(X, Ws, y, act)
    else:
        loss, dWs, _, dbs = mlp_backward(X, Ws, y, act, bs=bs)
    new = [_f64(W) - lr * g for W, g in zip(Ws, dWs)]
    if bs is None:
        return loss, new, dWs
    new_bs = [np.asarray(b, dtype=np.float64) - lr * g for b, g in zip(bs, dbs)]
    return loss, new, dWs, new_bs, dbs


def mlp_step_momentum(X, Ws, y, lr, mu, Vs, act="sigmoid", bs=None, Vbs=None):
    """One step of SGD with (heavy-ball) momentum:  V <- mu V + dW;  W <- W - lr V, the same for the
    bias rows when they and their velocities Vbs are given (bias rows without velocities take the
    plain step).  Returns (loss, new weights, new velocities) and, with bias rows, also
    (new bias rows, new bias velocities or None)."""
    if bs is None:
        loss, dWs, _ = mlp_backward(X, Ws, y, act)
    else:
        loss, dWs, _, dbs = mlp_backward(X, Ws, y, act, bs=bs)
    new_V = [mu * np.asarray(V, dtype=np.float64) + g for V, g in zip(Vs, dWs)]
    new_W = [_f64(W) - lr * V for W, V in zip(Ws, new_V)]
    if bs is None:
        return loss, new_W, new_V
    if Vbs is None:
        return loss, new_W, new_V, [np.asarray(b, dtype=np.float64) - lr * g for b, g in zip(bs, dbs)], None
    new_Vb = [mu * np.asarray(v, dtype=np.float64) + g for v, g in zip(Vbs, dbs)]
    new_b = [np.asarray(b, dtype=np.float64) - lr * v for b, v in zip(bs, new_Vb)]
    return loss, new_W, new_V, new_b, new_Vb


def mlp_step_stochastic(X, Ws, y, lr, seed, step, act="sigmoid"):
    """One SGD step of a bf16 network whose updated weights are rounded stochastically.

    The exact update is formed in fp64, brought to fp32 (the precision in which the rounding
    decision is taken) and rounded with the bits of (seed, layer, step).  Returns (loss, new
    weights as bf16 bit patterns, new weights in fp64 before any rounding)."""
    loss, exact, _ = mlp_step(X, Ws, y, lr, act)
    bits = [stochastic_round_matrix(w.astype(np.float32), seed, l + 1, step) for l, w in enumerate(exact)]
    return loss, bits, exact


def mlp_step_master(X, Ws, y, lr, masters, act="sigmoid", mu=None, Vs=None):
    """One step of a bf16 network that keeps an fp32 master copy M_l of every weight matrix.

    Both passes use the bf16 weights Ws (bit patterns); the step is applied to the master copy, in
    fp64 here and then brought to fp32 (the precision the master copy is stored in), and the bf16
    weights become the master copy rounded to nearest even -- so steps below half a bf16 ulp are kept
    in M_l and add up instead of being lost.  With mu and Vs the step is the momentum one
    (V <- mu V + dW; M <- M - lr V).  Returns (loss, new bf16 bit patterns, new masters as fp32,
    the new masters in fp64 before the fp32 rounding[, new velocities])."""
    loss, dWs, _ = mlp_backward(X, Ws, y, act)
    vel = None if Vs is None else [g + mu * np.asarray(V, dtype=np.float64) for g, V in zip(dWs, Vs)]
    moves = dWs if Vs is None else vel
    exact = [np.asarray(M, dtype=np.float32).astype(np.float64) - lr * d for M, d in zip(masters, moves)]
    new_M = [e.astype(np.float32) for e in exact]
    bits = [round_bf16_nearest(m) for m in new_M]
    if Vs is None:
        return loss, bits, new_M, exact
    return loss, bits, new_M, exact, vel


def _rows_times(R, W, transpose=False, block=4096, workers=1):
    """R @ W (or R @ W^T with transpose) in fp64 without ever holding the fp64 image of all of W: the
    output index (columns of W; rows of W with transpose) is walked in blocks, the inner dimension
    is never split.  workers > 1 only hands the independent blocks to a thread pool."""
    W = np.asarray(W)
    n_out = W.shape[0] if transpose else W.shape[1]
    out = np.empty((R.shape[0], n_out), dtype=np.float64)

    def one_block(o0):
        o1 = min(n_out, o0 + block)
        if transpose:
            out[:, o0:o1] = R @ _f64(W[o0:o1, :]).T
        else:
            out[:, o0:o1] = R @ _f64(np.ascontiguousarray(W[:, o0:o1]))

    starts = range(0, n_out, block)
    if workers > 1:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(workers) as pool:
            list(pool.map(one_block, starts))
    else:
        for o0 in starts:
            one_block(o0)
    return out


def mlp_rows(X_rows, Ws, y_rows, batch, act="sigmoid", block=4096, workers=1):
    """Forward and backward quantities of the batch rows given (X_rows: r x n_0, y_rows: r labels) of a
    step whose whole batch has `batch` samples.  Returns (acts, logits, probs, loss_rows, deltas):
    acts[l] the input of layer l+1 (acts[0] = X_rows), loss_rows[b] = -log P[b, y_b], deltas[l] the
    error at the output of layer l+1, with D_L = (P - onehot(y)) / batch."""
    a = _f64(X_rows)
    acts, pre = [a], [None]
    L = len(Ws)
    z = None
    for l, W in enumerate(Ws):
        z = _rows_times(a, W, block=block, workers=workers)
        if l < L - 1:
            a = _act(z, act)
            acts.append(a)
            pre.append(z)
    zmax = z.max(axis=1, keepdims=True)
    e = np.exp(z - zmax)
    probs = e / e.sum(axis=1)[:, None]
    y = np.asarray(y_rows, dtype=np.int64)
    r = np.arange(z.shape[0])
    loss_rows = zmax[:, 0] + np.log(e.sum(axis=1)) - z[r, y]
    d = probs.copy()
    d[r, y] -= 1.0
    d /= batch
    deltas = [None] * L
    for l in range(L - 1, -1, -1):
        deltas[l] = d
        if l > 0:
            d = _rows_times(d, Ws[l], transpose=True, block=block, workers=workers) * _act_slope(pre[l], acts[l], act)
    return acts, z, probs, loss_rows, deltas
