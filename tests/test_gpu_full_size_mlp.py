"""Full-size parity of the MLP configurations, through the C ABI, against oracle results computed
from the same seeded inputs only (nothing the GPU produced is fed to the oracle).

Config 4 (fp32, 4096 -> 16384 -> 16384 -> 16384 -> 10000, batch 4096, in-core): the whole fp64
oracle pass is affordable on the host, so every activation, the probabilities, the loss, every
error matrix and every dW are compared in full (relative Frobenius <= 1e-5), and W_new - W_old
after the fused step.

Config 5 (bf16, 8192 -> 32768 -> 32768 -> 262144, batch 8192, weights in pinned host memory, budget
32e9 bytes): the full oracle is out of reach (2.4e14 multiply-adds).
  (i)  Every per-sample quantity depends on that sample's row alone, so for sampled batch rows spread
       over all batch tiles oracle.mlp_rows computes the row's activations, logits, probabilities,
       loss and back-propagated errors from the seeded inputs alone (fp64); compared at the bf16 bar
       (1e-2).
  (ii) dW_l = A_{l-1}^T D_l sums over the whole batch, so an entry needs whole columns of A_{l-1} and
       D_l: those are read back from the device (mlp_read) and oracle.gemm_samples forms >= 4096
       entries of every dW_l from them in fp64, tile corners included.  This part is teacher-forced:
       it checks the dW product (and, after mlp_step, the fused update and the write-back) on the
       operands the device holds, and (i) is what ties those operands to the oracle.
  (iii) One mlp_step with the configuration's learning rate and one with a learning rate large
       enough to move bf16 weights by many ulps: W_new must be the correctly rounded image of
       W_old - lr dW on the sampled entries, W_new - W_old must meet the bar, every weight byte is
       written back once (d2h_bytes), and the weight-tile cache's trace is valid with its misses
       between the oracle's furthest-next-use count and +5 %."""
import numpy as np
import pytest
import torch

from gpu_util import announce, rel_fro
from test_gpu_mlp_cache_trace import replay_trace
from paper_1511_04348_amd import binding as tg
from paper_1511_04348_amd import inputs

pytestmark = pytest.mark.gpu


def test_config4_full_parity(oracle):
    dims, batch, T, lr = [4096, 16384, 16384, 16384, 10000], 4096, 1024, 0.01
    L = 4
    announce("config4 inputs")
    X = inputs.normal_matrix(1, batch, dims[0], device="cuda")
    y = inputs.labels(5, batch, dims[-1], device="cuda")
    W = [inputs.normal_matrix(10 + l, dims[l], dims[l + 1], std=0.01, device="cuda") for l in range(L)]
    torch.cuda.synchronize()
    Xn, yn, Wn = X.cpu().numpy(), y.cpu().numpy(), [w.cpu().numpy() for w in W]
    ctx = tg.tgemm_create(0)
    try:
        mlp = tg.mlp_create(ctx, dims, W, tg.TGEMM_F32, T)
        probs = torch.empty(batch, dims[-1], device="cuda")
        dW = [torch.empty_like(w) for w in W]
        torch.cuda.synchronize()
        announce("config4 gpu passes")
        tg.mlp_forward(mlp, X, batch, probs)
        loss = tg.mlp_backward(mlp, y, dW)
        acts = []
        for l in range(1, L):
            a = torch.empty(batch, dims[l])
            tg.mlp_read(mlp, 0, l, a, a.numel() * 4)
            acts.append(a.numpy())
        deltas = []
        for l in range(1, L + 1):
            d = torch.empty(batch, dims[l])
            tg.mlp_read(mlp, 2, l, d, d.numel() * 4)
            deltas.append(d.numpy())
        dWn = [g.cpu().numpy() for g in dW]
        probs_n = probs.cpu().numpy()
        del dW, probs
        torch.cuda.empty_cache()
        loss_step = tg.mlp_step(mlp, X, y, batch, lr)
        W_new = [w.cpu().numpy() for w in W]
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)
    announce("config4 oracle (fp64, full size)")
    loss_ref, dW_ref, delta_ref = oracle.mlp_backward(Xn, Wn, yn)
    acts_ref, _, P_ref = oracle.mlp_forward(Xn, Wn)
    tol = 1e-5
    assert abs(loss - loss_ref) <= tol * abs(loss_ref) and abs(loss_step - loss_ref) <= tol * abs(loss_ref)
    for l in range(1, L):
        assert rel_fro(acts[l - 1], acts_ref[l]) <= tol, ("activation", l)
    assert rel_fro(probs_n, P_ref) <= tol
    for l in range(L):
        assert rel_fro(deltas[l], delta_ref[l]) <= tol, ("delta", l + 1)
        e = rel_fro(dWn[l], dW_ref[l])
        print("config4 dW", l + 1, "rel fro", e)
        assert e <= tol, ("dW", l + 1)
        upd = W_new[l].astype(np.float64) - Wn[l].astype(np.float64)
        slack = np.linalg.norm(W_new[l]) * 2.0 ** -24 / np.linalg.norm(lr * dW_ref[l])
        assert rel_fro(upd, -lr * dW_ref[l]) <= tol + slack, ("update", l + 1, slack)


def _read_matrix(mlp, what, layer, rows, cols, dt):
    buf = torch.empty(rows, cols, dtype=dt)
    tg.mlp_read(mlp, what, layer, buf, buf.numel() * buf.element_size())
    return buf


def _sample_entries(n_rows, n_cols, T, n_random, seed):
    """Entry indices: the four corners of every tile on a coarse grid of tiles plus random entries."""
    rng = np.random.default_rng(seed)
    edges_r = sorted(set(e for t in range(0, n_rows, T) for e in (t, min(n_rows, t + T) - 1)))
    edges_c = sorted(set(e for t in range(0, n_cols, T) for e in (t, min(n_cols, t + T) - 1)))
    pick_r = edges_r if len(edges_r) <= 8 else [edges_r[i] for i in sorted(rng.choice(len(edges_r), 8, replace=False))]
    pick_c = edges_c if len(edges_c) <= 8 else [edges_c[i] for i in sorted(rng.choice(len(edges_c), 8, replace=False))]
    ri = [r for r in pick_r for _ in pick_c] + list(rng.integers(0, n_rows, n_random))
    ci = [c for _ in pick_r for c in pick_c] + list(rng.integers(0, n_cols, n_random))
    return np.asarray(ri, dtype=np.int64), np.asarray(ci, dtype=np.int64)


def _bf16_spacing(v):
    """Distance between neighbouring bf16 values at |v| (v: float64 array of bf16-representable or nearby values)."""
    a = np.maximum(np.abs(v), 2.0 ** -126).astype(np.float32)
    return np.spacing(a).astype(np.float64) * 65536.0


def test_config5_full_size(oracle):
    dims, batch, T, budget = [8192, 32768, 32768, 262144], 8192, 2048, 32 * 10 ** 9
    L = 3
    announce("config5 inputs")
    X = inputs.normal_matrix(1, batch, dims[0], device="cuda").to(torch.bfloat16)
    y = inputs.labels(5, batch, dims[-1], device="cuda")
    W = []
    for l in range(L):
        w = torch.empty(dims[l], dims[l + 1], dtype=torch.bfloat16, pin_memory=True)
        inputs.fill(w, 10 + l, "normal", gen_device="cuda", std=0.01)
        W.append(w)
    torch.cuda.synchronize()
    rows = sorted(set([0, 1, 2047, 2048, 4095, 4096, 6143, 6144, 8191] +
                      list(np.random.default_rng(0).integers(0, batch, 7))))
    samples = [_sample_entries(dims[l], dims[l + 1], T, 4096, 100 + l) for l in range(L)]
    w_bytes = sum(w.numel() for w in W) * 2
    assert w_bytes == 19864223744
    ctx = tg.tgemm_create(0, trace=1)
    got = {}
    try:
        mlp = tg.mlp_create(ctx, dims, W, tg.TGEMM_BF16, T, hbm_budget=budget)
        dW = [torch.empty(dims[l], dims[l + 1], device="cuda") for l in range(L)]      # 1.1 + 4.3 + 34.4 GB, the caller's
        torch.cuda.synchronize()
        announce("config5 gpu forward + backward with dW")
        calls = []
        tg.mlp_forward(mlp, X, batch)
        st_f = tg.tgemm_last_stats(ctx)
        calls.append(tg.mlp_trace(mlp))
        loss = tg.mlp_backward(mlp, y, dW)
        st_b = tg.tgemm_last_stats(ctx)
        calls.append(tg.mlp_trace(mlp))
        print("config5 forward stats", st_f, "backward stats", st_b, flush=True)
        n_slots = st_f["n_slots"]
        assert st_f["in_core"] == 0 and st_f["misses"] == 2368 and n_slots < 2368
        assert st_f["h2d_bytes"] == w_bytes                                          # forward fetches every tile once
        assert st_b["d2h_bytes"] == 0                                                 # backward without update writes nothing back
        for name, what, layer, n, dt in [("a1", 0, 1, dims[1], torch.bfloat16), ("a2", 0, 2, dims[2], torch.bfloat16),
                                         ("z", 1, 0, dims[3], torch.float32), ("d3", 2, 3, dims[3], torch.bfloat16),
                                         ("d2", 2, 2, dims[2], torch.bfloat16), ("d1", 2, 1, dims[1], torch.bfloat16)]:
            buf = torch.empty(len(rows), n, dtype=dt)
            es = buf.element_size()
            for i, r in enumerate(rows):
                tg.mlp_read(mlp, what, layer, buf[i], n * es, offset=r * n * es)
            got[name] = buf.to(torch.float64).numpy()
        # (ii) the operands of the dW products as the device holds them, and the sampled entries of dW
        announce("config5 teacher-forced dW samples")
        A = [inputs.bf16_bits(X)] + [inputs.bf16_bits(_read_matrix(mlp, 0, l, batch, dims[l], torch.bfloat16)) for l in (1, 2)]
        D = [inputs.bf16_bits(_read_matrix(mlp, 2, l, batch, dims[l], torch.bfloat16)) for l in (1, 2, 3)]
        dW_ref = []
        for l in range(L):
            ri, ci = samples[l]
            ref = oracle.gemm_samples(A[l], D[l], ri, ci, trans_a=True)               # entries of A_{l-1}^T D_l, fp64
            gpu = dW[l][torch.as_tensor(ri, device="cuda"), torch.as_tensor(ci, device="cuda")].cpu().numpy().astype(np.float64)
            err = rel_fro(gpu, ref)
            print("config5 dW", l + 1, "sampled rel fro", err, "entries", len(ri), flush=True)
            assert err <= 1e-2, ("dW", l + 1, err)
            dW_ref.append(ref)
        del dW
        torch.cuda.empty_cache()
        # (i) the oracle's rows, from the seeded inputs and the weights as they are before any step
        announce("config5 oracle rows")
        yr = y.cpu().numpy()[rows]
        acts, z, P, loss_rows, deltas = oracle.mlp_rows(inputs.bf16_bits(X[rows]), [inputs.bf16_bits(w) for w in W], yr, batch,
                                                        workers=8)
        # (iii) the fused update at the configuration's learning rate: same inputs, same weights, so the same dW
        announce("config5 mlp_step, lr 0.01")
        W_old = [W[l][torch.as_tensor(samples[l][0]), torch.as_tensor(samples[l][1])].to(torch.float64).numpy() for l in range(L)]
        lr = 0.01
        loss_step = tg.mlp_step(mlp, X, y, batch, lr)
        st = tg.tgemm_last_stats(ctx)
        calls.append(tg.mlp_trace(mlp))
        print("config5 step stats", st, flush=True)
        assert loss_step == loss
        assert st["d2h_bytes"] == w_bytes and st["hits"] + st["misses"] == 2 * 2368
        for l in range(L):
            W_new = W[l][torch.as_tensor(samples[l][0]), torch.as_tensor(samples[l][1])].to(torch.float64).numpy()
            exact = W_old[l] - lr * dW_ref[l]
            # correctly rounded: within half a bf16 spacing of the exact value (plus the dW product's own error)
            off = np.abs(W_new - exact)
            assert np.all(off <= 0.5 * _bf16_spacing(exact) * (1 + 1e-3) + 1e-2 * np.abs(lr * dW_ref[l])), ("lr 0.01 rounding", l + 1)
            moved = int(np.count_nonzero(W_new != W_old[l]))
            print("config5 lr 0.01: layer", l + 1, "sampled weights that moved:", moved, "of", len(W_new), flush=True)
        # steady state of the weight-tile cache: two more steps, the trace of the last one replayed
        announce("config5 mlp_step, large lr; cache trace")
        lr2 = 4096.0
        W_old = [W[l][torch.as_tensor(samples[l][0]), torch.as_tensor(samples[l][1])].to(torch.float64).numpy() for l in range(L)]
        tg.mlp_step(mlp, X, y, batch, lr2)
        st2 = tg.tgemm_last_stats(ctx)
        trace = tg.mlp_trace(mlp)
        calls.append(trace)
        A = [inputs.bf16_bits(X)] + [inputs.bf16_bits(_read_matrix(mlp, 0, l, batch, dims[l], torch.bfloat16)) for l in (1, 2)]
        D = [inputs.bf16_bits(_read_matrix(mlp, 2, l, batch, dims[l], torch.bfloat16)) for l in (1, 2, 3)]
        for l in range(L):
            ri, ci = samples[l]
            ref = oracle.gemm_samples(A[l], D[l], ri, ci, trans_a=True)
            W_new = W[l][torch.as_tensor(ri), torch.as_tensor(ci)].to(torch.float64).numpy()
            exact = W_old[l] - lr2 * ref
            off = np.abs(W_new - exact)
            assert np.all(off <= 0.5 * _bf16_spacing(exact) * (1 + 1e-3) + 1e-2 * np.abs(lr2 * ref)), ("large lr rounding", l + 1)
            upd, want = W_new - W_old[l], -lr2 * ref
            slack = np.linalg.norm(0.5 * _bf16_spacing(exact)) / np.linalg.norm(want)
            err = rel_fro(upd, want)
            print("config5 W_new - W_old layer", l + 1, "rel fro", err, "half-ulp slack", slack, flush=True)
            assert err <= 1e-2 + slack, ("update", l + 1, err, slack)
            assert np.count_nonzero(upd) > 0.9 * len(upd)                               # the step really moved the weights
        assert st2["d2h_bytes"] == w_bytes
        tg.mlp_destroy(mlp)
    finally:
        tg.tgemm_destroy(ctx)
    # the cache trace of a steady-state step: lookup order unique, the rest valid, misses near the minimum
    announce("config5 cache trace")
    groups = oracle.mlp_sweep_groups(dims, T)
    flat = [k for g in groups for k in g]
    assert [(r["layer"], r["r"], r["c"]) for r in trace] == flat
    n_miss = sum(1 for r in trace if not r["hit"])
    assert n_miss == st2["misses"]
    _, two = oracle.next_use_simulate(groups, n_slots, 2)
    _, one = oracle.next_use_simulate(groups, n_slots, 1)
    steady = two["misses"] - one["misses"]
    print("config5 misses per steady-state step", n_miss, "furthest-next-use", steady, "slots", n_slots, flush=True)
    assert steady <= n_miss <= int(1.05 * steady)
    assert st2["h2d_bytes"] == n_miss * T * T * 2
    total = replay_trace(oracle, dims, T, n_slots, calls)         # every call since the object was created, from the cold cache
    assert total == st_f["misses"] + st_b["misses"] + st["misses"] + st2["misses"]
    tol = 1e-2
    for name, ref in [("a1", acts[1]), ("a2", acts[2]), ("z", z), ("d3", deltas[2]), ("d2", deltas[1]), ("d1", deltas[0])]:
        err = rel_fro(got[name], ref)
        print("config5", name, "rel fro", err, flush=True)
        assert err <= tol, name
    assert np.isfinite(loss) and abs(loss - 12.97) < 0.2      # ln(262144) = 12.48 plus the logit variance term
    assert abs(float(np.mean(loss_rows)) - loss) < 0.3         # 16 sampled rows against the batch mean
