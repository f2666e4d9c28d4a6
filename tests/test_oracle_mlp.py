"""Pins of the MLP oracle: finite differences, closed forms for zero weights and for the
single-layer (softmax regression) case, invariants, first-order descent."""
import math

import numpy as np


def _net(seed, dims, B):
    r = np.random.default_rng(seed)
    X = r.normal(0, 1, (B, dims[0])).astype(np.float32)
    Ws = [r.normal(0, 0.5, (a, b)).astype(np.float32) for a, b in zip(dims[:-1], dims[1:])]
    y = r.integers(0, dims[-1], B)
    return X, Ws, y


def test_finite_differences_every_weight(oracle):
    X, Ws, y = _net(0, [5, 7, 6, 4], 3)
    loss, dWs, _ = oracle.mlp_backward(X, Ws, y)
    assert abs(loss - oracle.mlp_loss(X, Ws, y)) < 1e-15
    h = 1e-5
    W64 = [w.astype(np.float64) for w in Ws]
    for l, W in enumerate(W64):
        num = np.zeros_like(W)
        for idx in np.ndindex(*W.shape):
            old = W[idx]
            W[idx] = old + h
            lp = oracle.mlp_loss(X, W64, y)
            W[idx] = old - h
            lm = oracle.mlp_loss(X, W64, y)
            W[idx] = old
            num[idx] = (lp - lm) / (2 * h)
        err = np.linalg.norm(num - dWs[l]) / np.linalg.norm(dWs[l])
        assert err < 1e-6, (l, err)


def test_zero_weights_closed_form(oracle):
    dims = [6, 8, 5, 10]
    X, Ws, y = _net(1, dims, 4)
    Ws = [np.zeros_like(w) for w in Ws]
    acts, z, P = oracle.mlp_forward(X, Ws)
    assert np.array_equal(acts[1], np.full((4, 8), 0.5)) and np.array_equal(acts[2], np.full((4, 5), 0.5))
    assert np.allclose(P, 0.1, rtol=0, atol=1e-16)
    assert abs(oracle.mlp_loss(X, Ws, y) - math.log(10)) < 1e-15
    # the benchmark output widths
    assert abs(math.log(10000) - 9.210340371976184) < 1e-12
    loss, dWs, _ = oracle.mlp_backward(X, Ws, y)
    # with zero weights no error reaches the earlier layers
    assert np.array_equal(dWs[0], np.zeros_like(dWs[0])) and np.array_equal(dWs[1], np.zeros_like(dWs[1]))
    # last layer: 0.5 * column sums of (P - Y)/B
    D = np.full((4, 10), 0.1)
    D[np.arange(4), y] -= 1
    assert np.allclose(dWs[2], 0.5 * np.ones((5, 1)) * D.sum(0, keepdims=True) / 4, atol=1e-16)


def test_single_layer_is_softmax_regression(oracle):
    X, Ws, y = _net(2, [9, 6], 7)
    loss, dWs, deltas = oracle.mlp_backward(X, Ws, y)
    X64, W64 = X.astype(np.float64), Ws[0].astype(np.float64)
    z = X64 @ W64
    P = np.exp(z) / np.exp(z).sum(1, keepdims=True)   # no max shift: small logits
    Y = np.eye(6)[y]
    assert np.allclose(dWs[0], X64.T @ (P - Y) / 7, atol=1e-14)
    assert abs(loss + np.mean(np.log(P[np.arange(7), y]))) < 1e-14


def test_invariants_and_orientation(oracle):
    dims = [5, 9, 4]
    X, Ws, y = _net(3, dims, 6)
    acts, z, P = oracle.mlp_forward(X, Ws)
    assert [a.shape for a in acts] == [(6, 5), (6, 9)] and z.shape == (6, 4)
    assert np.allclose(P.sum(1), 1, atol=1e-15)
    loss, dWs, deltas = oracle.mlp_backward(X, Ws, y)
    assert [g.shape for g in dWs] == [w.shape for w in Ws]
    assert np.allclose(deltas[-1].sum(1), 0, atol=1e-16)
    assert loss > 0
    # softmax is shift invariant: a huge common offset on the logits must not overflow
    big = [Ws[0], Ws[1] * 0]
    acts2, z2, P2 = oracle.mlp_forward(X, big)
    assert np.allclose(P2, 0.25)


def test_step_descends_first_order(oracle):
    X, Ws, y = _net(4, [6, 8, 5], 8)
    lr = 1e-4
    loss, newW, dWs = oracle.mlp_step(X, Ws, y, lr)
    g2 = sum(float((g * g).sum()) for g in dWs)
    loss_after = oracle.mlp_loss(X, newW, y)
    assert abs((loss_after - loss) + lr * g2) < 50 * lr * lr * g2 + 1e-12
    # all updates use the pre-update weights: W_new - W == -lr * dW exactly in fp64
    for w, nw, g in zip(Ws, newW, dWs):
        assert np.array_equal(nw, w.astype(np.float64) - lr * g)


def test_bf16_inputs_widen_exactly(oracle):
    X, Ws, y = _net(5, [4, 5, 3], 2)
    def bits(a):
        u = a.view(np.uint32).astype(np.uint64)
        return ((u + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    Xb, Wb = bits(X), [bits(w) for w in Ws]
    Xf = oracle.bf16_to_f64(Xb).reshape(X.shape).astype(np.float32)
    Wf = [oracle.bf16_to_f64(w).reshape(w.shape).astype(np.float32) for w in Wb]
    l1 = oracle.mlp_backward(Xb, Wb, y)
    l2 = oracle.mlp_backward(Xf, Wf, y)
    assert l1[0] == l2[0] and all(np.array_equal(a, b) for a, b in zip(l1[1], l2[1]))


# ---- other hidden activations (tanh, relu) ---------------------------------------------------------

def _fd_check(oracle, act, seed):
    X, Ws, y = _net(seed, [5, 7, 6, 4], 3)
    loss, dWs, _ = oracle.mlp_backward(X, Ws, y, act=act)
    h = 1e-6
    W64 = [w.astype(np.float64) for w in Ws]
    for l, W in enumerate(W64):
        num = np.zeros_like(W)
        for idx in np.ndindex(*W.shape):
            old = W[idx]
            W[idx] = old + h
            lp = oracle.mlp_loss(X, W64, y, act=act)
            W[idx] = old - h
            lm = oracle.mlp_loss(X, W64, y, act=act)
            W[idx] = old
            num[idx] = (lp - lm) / (2 * h)
        err = np.linalg.norm(num - dWs[l]) / np.linalg.norm(dWs[l])
        assert err < 1e-6, (act, l, err)


def test_finite_differences_tanh_and_relu(oracle):
    _fd_check(oracle, "tanh", 3)
    # relu has a kink at 0; with these seeded weights no pre-activation lies within 1e-3 of it
    X, Ws, y = _net(4, [5, 7, 6, 4], 3)
    _, _, _, pre = oracle.mlp_forward(X, Ws, "relu", return_pre=True)
    assert min(np.abs(z).min() for z in pre[1:]) > 1e-3
    _fd_check(oracle, "relu", 4)


def test_activation_values_written_out(oracle):
    """One input row through an identity first layer: the hidden activations are the function's
    values at 1, -2 and 0.5 (tanh(1) = 0.76159415595576, tanh(2) = 0.96402758007582,
    tanh(0.5) = 0.46211715726001; logistic function at 1, -2, 0.5: 0.73105857863000,
    0.11920292202212, 0.62245933120185 -- standard table values)."""
    X = np.array([[1.0, -2.0, 0.5]], dtype=np.float32)
    Ws = [np.eye(3, dtype=np.float32), np.ones((3, 2), dtype=np.float32)]
    acts, z, P = oracle.mlp_forward(X, Ws, "tanh")
    assert np.allclose(acts[1], [[0.76159415595576, -0.96402758007582, 0.46211715726001]], rtol=0, atol=1e-13)
    acts, z, P = oracle.mlp_forward(X, Ws, "relu")
    assert np.array_equal(acts[1], [[1.0, 0.0, 0.5]]) and np.array_equal(z, [[1.5, 1.5]])
    acts, z, P = oracle.mlp_forward(X, Ws, "sigmoid")
    assert np.allclose(acts[1], [[0.73105857863000, 0.11920292202212, 0.62245933120185]], rtol=0, atol=1e-13)


def test_activation_symmetries(oracle):
    """tanh is odd: without biases the logits change sign with the input.  relu is positively
    homogeneous: the logits scale with the input.  Zero weights: tanh and relu hidden layers are 0."""
    X, Ws, y = _net(5, [6, 9, 7, 5], 4)
    X = X.astype(np.float64)          # so that -X and 3 X are exact
    _, z, _ = oracle.mlp_forward(X, Ws, "tanh")
    _, zn, _ = oracle.mlp_forward(-X, Ws, "tanh")
    assert np.allclose(zn, -z, rtol=0, atol=1e-14) and np.abs(z).max() > 0.1
    _, z, _ = oracle.mlp_forward(X, Ws, "relu")
    _, z3, _ = oracle.mlp_forward(3.0 * X, Ws, "relu")
    assert np.allclose(z3, 3.0 * z, rtol=1e-13, atol=1e-13) and np.abs(z).max() > 0.1
    _, zneg, _ = oracle.mlp_forward(-X, Ws, "relu")
    assert not np.allclose(zneg, z) and not np.allclose(zneg, -z)        # neither even nor odd
    Z0 = [np.zeros_like(w) for w in Ws]
    for act in ("tanh", "relu"):
        acts, _, P = oracle.mlp_forward(X, Z0, act)
        assert all(np.array_equal(a, np.zeros_like(a)) for a in acts[1:])
        assert np.allclose(P, 0.2, rtol=0, atol=1e-16)
    # the relu slope is 0 or 1: the error reaching layer 1 vanishes exactly where the unit is off
    acts, _, _, pre = oracle.mlp_forward(X, Ws, "relu", return_pre=True)
    _, _, deltas = oracle.mlp_backward(X, Ws, y, act="relu")
    assert np.array_equal(deltas[0] == 0.0, pre[1] <= 0.0)


def test_step_descends_for_every_activation(oracle):
    for act in ("tanh", "relu"):
        X, Ws, y = _net(6, [8, 10, 6], 5)
        loss, dWs, _ = oracle.mlp_backward(X, Ws, y, act=act)
        lr = 1e-4
        l0, new, _ = oracle.mlp_step(X, Ws, y, lr, act=act)
        assert l0 == loss
        l1 = oracle.mlp_loss(X, new, y, act=act)
        g2 = sum((g ** 2).sum() for g in dWs)
        assert abs((l1 - l0) + lr * g2) < 5e-2 * lr * g2


# ---- bias rows -----------------------------------------------------------------------------------

def _biases(seed, dims):
    r = np.random.default_rng(seed)
    return [r.normal(0, 0.5, n).astype(np.float32) for n in dims[1:]]


def test_bias_finite_differences(oracle):
    for act in ("sigmoid", "tanh"):
        dims = [5, 6, 6, 4]          # two layers of one width: a bias row taken from the wrong layer still fits
        X, Ws, y = _net(20, dims, 3)
        bs = [b.astype(np.float64) for b in _biases(21, dims)]
        loss, dWs, _, dbs = oracle.mlp_backward(X, Ws, y, act, bs=bs)
        assert abs(loss - oracle.mlp_loss(X, Ws, y, act, bs=bs)) < 1e-15
        h = 1e-5
        for l, b in enumerate(bs):
            num = np.zeros_like(b)
            for i in range(b.size):
                old = b[i]
                b[i] = old + h
                lp = oracle.mlp_loss(X, Ws, y, act, bs=bs)
                b[i] = old - h
                lm = oracle.mlp_loss(X, Ws, y, act, bs=bs)
                b[i] = old
                num[i] = (lp - lm) / (2 * h)
            assert np.linalg.norm(num - dbs[l]) / np.linalg.norm(dbs[l]) < 1e-6, (act, l)
        # the weight gradients with bias rows present, one layer by finite differences
        W64 = [w.astype(np.float64) for w in Ws]
        num = np.zeros_like(W64[1])
        for idx in np.ndindex(*W64[1].shape):
            old = W64[1][idx]
            W64[1][idx] = old + h
            lp = oracle.mlp_loss(X, W64, y, act, bs=bs)
            W64[1][idx] = old - h
            lm = oracle.mlp_loss(X, W64, y, act, bs=bs)
            W64[1][idx] = old
            num[idx] = (lp - lm) / (2 * h)
        assert np.linalg.norm(num - dWs[1]) / np.linalg.norm(dWs[1]) < 1e-6


def test_bias_is_a_constant_one_input_column(oracle):
    """A bias row equals one more weight row fed by an input that is always 1 (layer by layer: the
    augmented activation is [A_l, 1])."""
    X, Ws, y = _net(22, [6, 5], 8)
    b = _biases(23, [6, 5])
    X1 = np.concatenate([X, np.ones((8, 1), dtype=np.float32)], axis=1)
    W1 = [np.concatenate([Ws[0], b[0][None, :]], axis=0)]
    loss_b, dW_b, _, db = oracle.mlp_backward(X, Ws, y, bs=b)
    loss_1, dW_1, _ = oracle.mlp_backward(X1, W1, y)
    assert abs(loss_b - loss_1) < 1e-15
    assert np.allclose(dW_1[0][:-1], dW_b[0], atol=1e-16) and np.allclose(dW_1[0][-1], db[0], atol=1e-16)
    # two layers, by hand: hidden activations of the biased net feed an augmented second layer
    X, Ws, y = _net(24, [4, 6, 3], 5)
    b = _biases(25, [4, 6, 3])
    acts, z, P = oracle.mlp_forward(X, Ws, bs=b)
    h = 1.0 / (1.0 + np.exp(-(X.astype(np.float64) @ Ws[0] + b[0])))
    assert np.allclose(acts[1], h, atol=1e-15)
    assert np.allclose(z, np.concatenate([h, np.ones((5, 1))], 1) @ np.concatenate([Ws[1], b[1][None, :]], 0), atol=1e-14)


def test_bias_closed_forms(oracle):
    # zero weights: the logits are the last bias row whatever the input; P = softmax(b_L)
    dims = [6, 8, 5]
    X, Ws, y = _net(26, dims, 4)
    Ws = [np.zeros_like(w) for w in Ws]
    b = _biases(27, dims)
    acts, z, P = oracle.mlp_forward(X, Ws, bs=b)
    sm = np.exp(b[1].astype(np.float64))
    sm /= sm.sum()
    assert np.allclose(z, np.tile(b[1].astype(np.float64), (4, 1)), atol=0) and np.allclose(P, np.tile(sm, (4, 1)), atol=1e-16)
    assert np.allclose(acts[1], np.tile(1 / (1 + np.exp(-b[0].astype(np.float64))), (4, 1)), atol=1e-16)
    loss, dWs, deltas, dbs = oracle.mlp_backward(X, Ws, y, bs=b)
    # db_L = softmax(b_L) - class frequencies
    freq = np.bincount(y, minlength=5) / 4.0
    assert np.allclose(dbs[1], sm - freq, atol=1e-15)
    assert abs(dbs[1].sum()) < 1e-15                       # rows of D_L sum to zero
    assert np.array_equal(dbs[0], np.zeros(8))             # nothing flows back through zero weights
    # zero bias rows change nothing
    X, Ws, y = _net(28, [5, 7, 4], 6)
    zb = [np.zeros(7), np.zeros(4)]
    l0, g0, d0 = oracle.mlp_backward(X, Ws, y)
    l1, g1, d1, db1 = oracle.mlp_backward(X, Ws, y, bs=zb)
    assert l0 == l1 and all(np.array_equal(a, c) for a, c in zip(g0, g1))
    assert all(np.array_equal(d.sum(axis=0), g) for d, g in zip(d1, db1)) and db1[0].shape == (7,) and db1[1].shape == (4,)


def test_bias_step(oracle):
    dims = [6, 9, 5]
    X, Ws, y = _net(29, dims, 16)
    b = _biases(30, dims)
    loss, new, dWs, new_b, dbs = oracle.mlp_step(X, Ws, y, 0.05, bs=b)
    _, g, _, gb = oracle.mlp_backward(X, Ws, y, bs=b)
    for l in range(2):
        assert np.array_equal(new[l], Ws[l].astype(np.float64) - 0.05 * g[l])
        assert np.array_equal(new_b[l], b[l].astype(np.float64) - 0.05 * gb[l]) and np.array_equal(dbs[l], gb[l])
    # first-order descent including the bias part of the gradient
    after = oracle.mlp_loss(X, new, y, bs=new_b)
    pred = loss - 0.05 * (sum((x ** 2).sum() for x in g) + sum((x ** 2).sum() for x in gb))
    assert after < loss and abs(after - pred) < 0.05 * (loss - pred) + 1e-6
    # moving only the bias rows along -db lowers the loss too
    assert oracle.mlp_loss(X, Ws, y, bs=new_b) < loss


# ---- momentum --------------------------------------------------------------------------------------

def test_momentum_reduces_to_sgd_and_heavy_ball_identity(oracle):
    dims = [6, 9, 5]
    X, Ws, y = _net(40, dims, 12)
    r = np.random.default_rng(41)
    V0 = [r.normal(0, 0.1, w.shape) for w in Ws]
    lr, mu = 0.05, 0.8
    # mu = 0: the plain step whatever the old velocity, and the velocity becomes the gradient
    loss, W1, V1 = oracle.mlp_step_momentum(X, Ws, y, lr, 0.0, V0)
    loss_s, W_s, g = oracle.mlp_step(X, Ws, y, lr)
    assert loss == loss_s
    assert all(np.array_equal(a, b) for a, b in zip(W1, W_s)) and all(np.array_equal(a, b) for a, b in zip(V1, g))
    # one step written out
    _, W1, V1 = oracle.mlp_step_momentum(X, Ws, y, lr, mu, V0)
    for l in range(2):
        assert np.allclose(V1[l], mu * V0[l] + g[l], rtol=0, atol=1e-16)
        assert np.allclose(W1[l], Ws[l].astype(np.float64) - lr * mu * V0[l] - lr * g[l], rtol=0, atol=1e-15)
    # two steps from rest: the heavy-ball form  W2 - W1 = mu (W1 - W0) - lr grad(W1)
    zero = [np.zeros(w.shape) for w in Ws]
    _, Wa, Va = oracle.mlp_step_momentum(X, Ws, y, lr, mu, zero)
    _, Wb, Vb = oracle.mlp_step_momentum(X, Wa, y, lr, mu, Va)
    _, g1, _ = oracle.mlp_backward(X, Wa, y)
    for l in range(2):
        assert np.allclose(Wb[l] - Wa[l], mu * (Wa[l] - Ws[l].astype(np.float64)) - lr * g1[l], rtol=0, atol=1e-15)
    # a constant gradient direction accumulates: from rest, step 2 moves further than step 1 along -g
    assert sum(((Wb[l] - Wa[l]) * g[l]).sum() for l in range(2)) < sum(((Wa[l] - Ws[l]) * g[l]).sum() for l in range(2)) < 0


def test_momentum_with_bias_rows(oracle):
    dims = [5, 7, 4]
    X, Ws, y = _net(42, dims, 9)
    b = _biases(43, dims)
    r = np.random.default_rng(44)
    V0 = [r.normal(0, 0.1, w.shape) for w in Ws]
    Vb0 = [r.normal(0, 0.1, x.shape) for x in b]
    lr, mu = 0.1, 0.5
    _, g, _, gb = oracle.mlp_backward(X, Ws, y, bs=b)
    loss, W1, V1, b1, Vb1 = oracle.mlp_step_momentum(X, Ws, y, lr, mu, V0, bs=b, Vbs=Vb0)
    for l in range(2):
        assert np.allclose(V1[l], mu * V0[l] + g[l], atol=1e-16) and np.allclose(Vb1[l], mu * Vb0[l] + gb[l], atol=1e-16)
        assert np.allclose(W1[l], Ws[l] - lr * V1[l], atol=1e-16) and np.allclose(b1[l], b[l] - lr * Vb1[l], atol=1e-16)
    # bias rows without velocities take the plain step
    _, W2, V2, b2, none = oracle.mlp_step_momentum(X, Ws, y, lr, mu, V0, bs=b)
    assert none is None and all(np.array_equal(a, c) for a, c in zip(W2, W1))
    assert all(np.allclose(b2[l], b[l] - lr * gb[l], atol=1e-16) for l in range(2))


def test_rows_equal_the_whole_batch_pass(oracle):
    """mlp_rows on a subset of the batch rows = those rows of the whole-batch passes, for block sizes
    that split the output index raggedly, one by one, or not at all; fp32 and bf16 bit patterns."""
    dims, B = [9, 13, 11, 7], 10
    X, Ws, y = _net(21, dims, B)
    rows = [0, 3, 4, 9]
    for conv in (lambda a: a.astype(np.float32), lambda a: (a.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)):
        Xc, Wc = conv(X), [conv(w) for w in Ws]
        for act in ("sigmoid", "tanh", "relu"):
            acts, z, P = oracle.mlp_forward(Xc, Wc, act)
            _, _, deltas = oracle.mlp_backward(Xc, Wc, y, act)
            for block in (1, 4, 5, 64):
                a_r, z_r, P_r, loss_r, d_r = oracle.mlp_rows(Xc[rows], Wc, y[rows], B, act, block=block, workers=1 + block % 3)
                for l in range(len(dims) - 1):
                    assert np.allclose(a_r[l], acts[l][rows], rtol=1e-13, atol=1e-15), ("act", l, block)
                    assert np.allclose(d_r[l], deltas[l][rows], rtol=1e-12, atol=1e-18), ("delta", l, block)
                assert np.allclose(z_r, z[rows], rtol=1e-13, atol=1e-15) and np.allclose(P_r, P[rows], rtol=1e-13)
    # the row losses average to the loss when every row is given
    _, _, _, loss_r, _ = oracle.mlp_rows(X.astype(np.float32), [w.astype(np.float32) for w in Ws], y, B)
    assert abs(loss_r.mean() - oracle.mlp_loss(X.astype(np.float32), [w.astype(np.float32) for w in Ws], y)) < 1e-13


def test_rows_closed_forms_and_input_gradient(oracle):
    """Independent of the whole-batch functions: zero weights (P = 1/C, row loss = ln C, hidden 0.5,
    D_L = (1/C - onehot) / batch, earlier errors vanish), and the first error times W_1^T is the
    gradient of sum(row losses) / batch with respect to the rows' inputs (central differences)."""
    dims, B = [6, 8, 5, 4], 7
    X, Ws, y = _net(22, dims, B)
    rows = [1, 2, 6]
    Z = [np.zeros_like(w, dtype=np.float32) for w in Ws]
    a_r, z_r, P_r, loss_r, d_r = oracle.mlp_rows(X[rows].astype(np.float32), Z, y[rows], B)
    C = dims[-1]
    assert np.all(P_r == 1.0 / C) and np.allclose(loss_r, np.log(C), rtol=1e-15) and np.all(a_r[1] == 0.5) and np.all(a_r[2] == 0.5)
    want = np.full((len(rows), C), 1.0 / C)
    want[np.arange(len(rows)), y[rows]] -= 1.0
    assert np.allclose(d_r[-1], want / B, rtol=1e-15) and np.all(d_r[0] == 0.0) and np.all(d_r[1] == 0.0)
    Wf = [w.astype(np.float32) for w in Ws]
    Xr = X[rows].astype(np.float32).astype(np.float64)
    for act in ("sigmoid", "tanh"):
        _, _, _, _, d_r = oracle.mlp_rows(Xr.astype(np.float32), Wf, y[rows], B, act, block=3)
        grad = d_r[0] @ Wf[0].astype(np.float64).T
        h = 1e-5
        for r in range(len(rows)):
            for c in range(dims[0]):
                def total(v):
                    Xp = Xr.copy()
                    Xp[r, c] = v
                    # inputs stay fp64 here: the check is on the mathematics, not on storage rounding
                    a = Xp
                    for l, W in enumerate(Wf):
                        zz = a @ W.astype(np.float64)
                        if l < len(Wf) - 1:
                            a = 1.0 / (1.0 + np.exp(-zz)) if act == "sigmoid" else np.tanh(zz)
                    m = zz.max(axis=1)
                    lse = m + np.log(np.exp(zz - m[:, None]).sum(axis=1))
                    return float((lse - zz[np.arange(len(rows)), y[rows]]).sum() / B)
                fd = (total(Xr[r, c] + h) - total(Xr[r, c] - h)) / (2 * h)
                assert abs(fd - grad[r, c]) <= 1e-6 * max(1e-3, abs(grad[r, c])), (act, r, c, fd, grad[r, c])


def test_products_equal_the_triple_loop(oracle):
    """The MLP oracle takes its products from numpy's fp64 matmul; the GEMM oracle is a triple loop in
    C.  On fp32 inputs (which both widen exactly) the first layer's pre-activations, the last layer's
    dW = A^T D and the error D W^T must agree between the two to fp64 rounding."""
    dims, B = [6, 9, 5], 8
    X, Ws, y = _net(31, dims, B)
    acts, z, P, pre = oracle.mlp_forward(X, Ws, return_pre=True)
    _, dWs, deltas = oracle.mlp_backward(X, Ws, y)
    assert np.allclose(pre[1], oracle.gemm(X, Ws[0]), rtol=1e-13, atol=1e-15)
    a1 = acts[1].astype(np.float32)                       # what a device would hold; both sides get the same bits
    d2 = deltas[1].astype(np.float32)
    assert np.allclose(a1.astype(np.float64).T @ d2.astype(np.float64), oracle.gemm(a1, d2, trans_a=True), rtol=1e-13, atol=1e-18)
    assert np.allclose(d2.astype(np.float64) @ Ws[1].astype(np.float64).T, oracle.gemm(d2, Ws[1], trans_b=True), rtol=1e-13, atol=1e-18)
