"""Pins of the stochastic-rounding oracle.

What fixes it from outside: the published values of MurmurHash3's 32-bit finalizer, the closed-form
inverse of that finalizer, and the defining properties of stochastic rounding checked by brute
force over all 65536 values of the random bits (neighbours only, exact up-count = dropped fraction,
exact expectation, fixed points, odd symmetry)."""
import numpy as np


def _bf16_val(bits):
    return (np.asarray(bits, dtype=np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


def test_mix32_known_answers(oracle):
    # MurmurHash3 fmix32 of 0..5
    want = [0x0, 0x514E28B7, 0x30F4C306, 0x85F0B427, 0x249CB285, 0xCC0D53CD]
    got = [int(oracle.mix32(i)) for i in range(6)]
    assert got == want
    assert [int(v) for v in oracle.mix32(np.arange(6))] == want


def test_mix32_is_inverted_by_the_closed_form_inverse(oracle):
    # x ^= x >> s is undone by xoring the shifted copies back; an odd multiplier by its inverse mod 2^32
    inv1, inv2 = pow(0x85EBCA6B, -1, 1 << 32), pow(0xC2B2AE35, -1, 1 << 32)

    def unmix(h):
        h ^= h >> 16
        h = (h * inv2) & 0xFFFFFFFF
        h ^= (h >> 13) ^ (h >> 26)
        h = (h * inv1) & 0xFFFFFFFF
        h ^= h >> 16
        return h

    r = np.random.default_rng(5)
    xs = [0, 1, 0xFFFFFFFF, 0x80000000] + [int(v) for v in r.integers(0, 1 << 32, 2000)]
    hs = oracle.mix32(np.array(xs, dtype=np.uint64))
    assert [unmix(int(h)) for h in hs] == xs


def test_step_key_depends_on_every_argument(oracle):
    base = oracle.step_key(0x123456789ABCDEF0, 2, 7)
    assert 0 <= base < 1 << 32
    others = {oracle.step_key(0x123456789ABCDEF1, 2, 7), oracle.step_key(0x123456799ABCDEF0, 2, 7),
              oracle.step_key(0x123456789ABCDEF0, 3, 7), oracle.step_key(0x123456789ABCDEF0, 2, 8)}
    assert base not in others and len(others) == 4
    # written out with python integers
    k = int(oracle.mix32(0x9ABCDEF0))
    k = int(oracle.mix32(k ^ 0x12345678))
    k = int(oracle.mix32(k ^ 2))
    k = int(oracle.mix32(k ^ 7))
    assert base == k


def test_rounding_over_all_random_values_is_exactly_unbiased(oracle):
    r16 = np.arange(65536, dtype=np.uint32)
    r = np.random.default_rng(1)
    xs = np.concatenate([r.normal(0, 1, 40), [1.0, -1.0, 1.0 + 2.0 ** -8, 255.99999, -3.0e-30, 2.0 ** -130, 3.3895e38 * 0.99]])
    for x in xs.astype(np.float32):
        u = int(np.float32(x).view(np.uint32))
        lo = u >> 16
        frac = u & 0xFFFF
        out = oracle.stochastic_round_bf16(np.full(65536, x, dtype=np.float32), r16).astype(np.int64)
        assert set(np.unique(out).tolist()) <= {lo, lo + 1}                      # the two neighbours only
        assert int((out == lo + 1).sum()) == frac                                # up-count = dropped fraction
        if ((lo + 1) & 0x7F80) != 0x7F80:                                        # upper neighbour finite
            mean = _bf16_val(out).mean()
            assert mean == float(x), (x, mean)                                   # expectation, exactly
        # magnitude rounding: the mirror image of -x
        neg = oracle.stochastic_round_bf16(np.full(65536, -x, dtype=np.float32), r16).astype(np.int64)
        assert np.array_equal(neg ^ 0x8000, out)


def test_rounding_special_values(oracle):
    r16 = np.array([0, 1, 0x8000, 0xFFFF], dtype=np.uint32)
    for v, want in ((0.0, 0x0000), (-0.0, 0x8000), (1.0, 0x3F80), (-2.5, 0xC020), (np.inf, 0x7F80), (-np.inf, 0xFF80)):
        out = oracle.stochastic_round_bf16(np.full(4, v, dtype=np.float32), r16)
        assert out.tolist() == [want] * 4, v
    nan = oracle.stochastic_round_bf16(np.full(4, np.nan, dtype=np.float32), r16)
    assert all((int(b) & 0x7F80) == 0x7F80 and (int(b) & 0x7F) != 0 for b in nan)
    snan = np.array([0x7F800001], dtype=np.uint32).view(np.float32)            # payload below the cut
    assert np.isnan(_bf16_val(oracle.stochastic_round_bf16(snan, np.array([0xFFFF]))))[0]
    big = np.array([0x7F7FFFFF], dtype=np.uint32).view(np.float32)             # largest finite fp32
    assert oracle.stochastic_round_bf16(big, np.array([0]))[0] == 0x7F7F
    assert oracle.stochastic_round_bf16(big, np.array([1]))[0] == 0x7F80       # overflows like nearest-even does


def test_rounding_bits_layout_and_statistics(oracle):
    key = oracle.step_key(99, 1, 0)
    rows = np.arange(512, dtype=np.uint64)[:, None]
    cols = np.arange(1024, dtype=np.uint64)[None, :]
    bits = oracle.rounding_bits(key, rows, cols)
    assert bits.shape == (512, 1024) and bits.dtype == np.uint32 and int(bits.max()) < 65536
    # the two columns of a pair are the halves of one 32-bit word: mix32(mix32(row + key) + pair * golden)
    for (rr, cc) in ((0, 0), (3, 10), (511, 1022), (77, 500)):
        h = int(oracle.mix32((rr + key) & 0xFFFFFFFF))
        w = int(oracle.mix32((h + (cc // 2) * 0x9E3779B9) & 0xFFFFFFFF))
        assert int(bits[rr, cc]) == w & 0xFFFF and int(bits[rr, cc + 1]) == w >> 16
    # uniform: chi-square over 256 buckets of the high and of the low byte (255 dof: mean 255, sd 22.6)
    n = bits.size
    for part in (bits >> 8, bits & 0xFF):
        cnt = np.bincount(part.ravel().astype(np.int64), minlength=256)
        chi2 = float(((cnt - n / 256.0) ** 2 / (n / 256.0)).sum())
        assert 150 < chi2 < 380, chi2
    # mean and neighbour correlations at the level of sampling noise (sd of the mean: 18900 / sqrt(n) = 26)
    f = bits.astype(np.float64)
    assert abs(f.mean() - 32767.5) < 130
    z = (f - f.mean()) / f.std()
    for a, b in ((z[:, :-1], z[:, 1:]), (z[:-1, :], z[1:, :]), (z[:, :-2], z[:, 2:])):
        assert abs(float((a * b).mean())) < 6.0 / np.sqrt(a.size)
    # another step, layer or seed gives unrelated bits
    for other in (oracle.step_key(99, 1, 1), oracle.step_key(99, 2, 0), oracle.step_key(100, 1, 0)):
        g = oracle.rounding_bits(other, rows, cols).astype(np.float64)
        zg = (g - g.mean()) / g.std()
        assert abs(float((z * zg).mean())) < 6.0 / np.sqrt(z.size)
        assert float((g == f).mean()) < 1e-3


def test_rounding_a_matrix_is_unbiased_where_nearest_loses_the_update(oracle):
    # weights near 1 (ulp 2^-7), update of a twentieth of an ulp: nearest-even returns the old weights,
    # stochastic rounding moves the mean by the update
    r = np.random.default_rng(3)
    W = (1.0 + r.integers(1, 64, (256, 512)) * 2.0 ** -7).astype(np.float32)      # bf16-exact, in (1, 1.5)
    upd = np.float32(2.0 ** -7 / 20)
    new32 = (W - upd).astype(np.float32)
    rne = ((new32.view(np.uint32).astype(np.uint64) + 0x7FFF + ((new32.view(np.uint32) >> 16) & 1)) >> 16).astype(np.uint16)
    assert np.array_equal(_bf16_val(rne), W.astype(np.float64))
    out = _bf16_val(oracle.stochastic_round_matrix(new32, seed=11, layer=1, step=0))
    moved = out - W
    assert set(np.unique(moved).tolist()) <= {0.0, -(2.0 ** -7)}
    # mean step = -upd; sd of one entry = ulp * sqrt(p (1 - p)), p = 1/20
    sd = 2.0 ** -7 * np.sqrt(0.05 * 0.95) / np.sqrt(W.size)
    assert abs(moved.mean() + float(upd)) < 5 * sd
    # successive steps draw fresh bits
    out2 = _bf16_val(oracle.stochastic_round_matrix(new32, seed=11, layer=1, step=1))
    assert 0.02 < float((out2 != out).mean()) < 0.2


def test_mlp_step_stochastic_brackets_the_exact_update(oracle):
    r = np.random.default_rng(8)
    dims, B = [12, 20, 9], 16
    to_bits = lambda a: (a.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    X = to_bits(r.normal(0, 1, (B, dims[0])))
    Ws = [to_bits(r.normal(0, 0.3, (a, b))) for a, b in zip(dims[:-1], dims[1:])]
    y = r.integers(0, dims[-1], B)
    loss, bits, exact = oracle.mlp_step_stochastic(X, Ws, y, 0.5, seed=4, step=3)
    loss0, exact0, _ = oracle.mlp_step(X, Ws, y, 0.5)
    assert loss == loss0 and all(np.array_equal(a, b) for a, b in zip(exact, exact0))
    for l, (b, e) in enumerate(zip(bits, exact)):
        v = _bf16_val(b)
        e32 = e.astype(np.float32)
        lo = _bf16_val(e32.view(np.uint32) >> 16)                                  # truncation
        hi = _bf16_val((e32.view(np.uint32) >> 16) + 1)
        assert np.all((v == lo) | (v == hi))
        assert np.array_equal(b, oracle.stochastic_round_matrix(e32, 4, l + 1, 3))
        assert not np.array_equal(b, oracle.stochastic_round_matrix(e32, 4, l + 1, 2))


# ---- round to nearest even, and the step with fp32 master copies -----------------------------------

def test_nearest_even_against_torch_and_by_brute_force(oracle):
    import torch
    r = np.random.default_rng(21)
    # every exponent, random mantissas, plus the midpoints and their neighbours
    u = r.integers(0, 2 ** 32, 200000, dtype=np.uint64).astype(np.uint32)
    mid = (r.integers(0, 2 ** 16, 4096, dtype=np.uint64).astype(np.uint32) << 16) | np.uint32(0x8000)
    u = np.concatenate([u, mid, mid - 1, mid + 1, np.array([0, 0x80000000, 0x7F7FFFFF, 0x00000001, 0x3F808000, 0x3F818000], dtype=np.uint32)])
    x = u.view(np.float32)
    finite = np.isfinite(x)
    got = oracle.round_bf16_nearest(x)
    # a library's conversion (independent of the oracle's arithmetic)
    ref = torch.from_numpy(x.copy()).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(got[finite], ref[finite])
    # brute force on the value line: the result is the nearer neighbour; at a tie the even pattern
    sel = np.flatnonzero(finite)
    sel = np.concatenate([sel[:20000], sel[-12000:]])            # random values, and the midpoints with their neighbours
    xs, g = x[sel].astype(np.float64), got[sel]
    lo_bits = (u[sel] >> 16).astype(np.uint16)
    lo, hi = _bf16_val(lo_bits), _bf16_val(lo_bits + np.uint16(1))
    hi_ok = np.isfinite(hi)
    v = _bf16_val(g)
    with np.errstate(invalid="ignore"):
        d_lo, d_hi = np.abs(xs - lo), np.abs(hi - xs)
    nearer_lo, nearer_hi = hi_ok & (d_lo < d_hi), hi_ok & (d_hi < d_lo)
    assert np.array_equal(g[nearer_lo], lo_bits[nearer_lo]) and np.array_equal(v[nearer_hi], hi[nearer_hi])
    tie = hi_ok & (d_lo == d_hi) & (d_lo > 0)
    assert tie.sum() > 100 and np.all((g[tie] & 1) == 0)
    # written-out cases: 1 + 2^-8 is a tie between 1 (even) and 1 + 2^-7 (odd); 1 + 3 * 2^-8 ties upwards
    assert oracle.round_bf16_nearest(np.float32(1 + 2.0 ** -8)).item() == 0x3F80
    assert oracle.round_bf16_nearest(np.float32(1 + 3 * 2.0 ** -8)).item() == 0x3F82
    assert oracle.round_bf16_nearest(np.float32(-(1 + 2.0 ** -8 + 2.0 ** -20))).item() == 0xBF81
    # infinities stay, NaNs stay NaNs, the largest finite fp32 overflows to infinity
    sp = oracle.round_bf16_nearest(np.array([np.inf, -np.inf, np.nan], dtype=np.float32))
    assert sp[0] == 0x7F80 and sp[1] == 0xFF80 and (sp[2] & 0x7F80) == 0x7F80 and (sp[2] & 0x7F) != 0
    assert oracle.round_bf16_nearest(np.array([0x7F7FFFFF], dtype=np.uint32).view(np.float32))[0] == 0x7F80


def _small_net(seed, dims, B):
    r = np.random.default_rng(seed)
    to_bits = lambda a: (a.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    X = to_bits(r.normal(0, 1, (B, dims[0])))
    Ws = [to_bits(r.normal(0, 0.3, (a, b))) for a, b in zip(dims[:-1], dims[1:])]
    return X, Ws, r.integers(0, dims[-1], B)


def test_master_step_written_out(oracle):
    dims, B, lr = [7, 11, 5], 13, 0.25
    X, Ws, y = _small_net(31, dims, B)
    r = np.random.default_rng(32)
    # master copies that differ from the bf16 weights by less than half an ulp of them
    M = [(_bf16_val(w) * (1 + r.uniform(-1, 1, w.shape) * 2.0 ** -10)).astype(np.float32) for w in Ws]
    assert all(np.array_equal(oracle.round_bf16_nearest(m), w) for m, w in zip(M, Ws))
    loss, bits, M1, exact = oracle.mlp_step_master(X, Ws, y, lr, M)
    # the gradient is that of the bf16 weights, not of the master copies
    loss_w, g, _ = oracle.mlp_backward(X, Ws, y)
    _, g_m, _ = oracle.mlp_backward(X, [m.astype(np.float64) for m in M], y)
    assert loss == loss_w
    for l in range(2):
        assert np.array_equal(exact[l], M[l].astype(np.float64) - lr * g[l])
        assert not np.allclose(exact[l], M[l].astype(np.float64) - lr * g_m[l], rtol=0, atol=1e-9)
        assert M1[l].dtype == np.float32 and np.all(np.abs(M1[l].astype(np.float64) - exact[l]) <= np.abs(exact[l]) * 2.0 ** -24)
        v = _bf16_val(bits[l])
        assert np.all(np.abs(v - M1[l]) <= np.abs(M1[l]) * 2.0 ** -8)           # within half a bf16 ulp (2^-8 relative at most)
        assert np.array_equal(bits[l], oracle.round_bf16_nearest(M1[l]))
    # with momentum the master copy moves by the velocity
    V0 = [r.normal(0, 0.1, w.shape) for w in Ws]
    _, bits_m, M1m, exact_m, V1 = oracle.mlp_step_master(X, Ws, y, lr, M, mu=0.5, Vs=V0)
    for l in range(2):
        assert np.allclose(V1[l], 0.5 * V0[l] + g[l], rtol=0, atol=1e-16)
        assert np.allclose(exact_m[l], M[l].astype(np.float64) - lr * (0.5 * V0[l] + g[l]), rtol=0, atol=1e-15)
        assert np.array_equal(bits_m[l], oracle.round_bf16_nearest(exact_m[l].astype(np.float32)))


def test_master_copies_keep_the_steps_that_bf16_storage_loses(oracle):
    # steps far below half a bf16 ulp of the weights: the plain bf16 step returns the old weights every
    # time; with master copies the steps add up and the bf16 weights start to move
    dims, B = [6, 8, 4], 10
    X, Ws, y = _small_net(33, dims, B)
    W0 = [_bf16_val(w) for w in Ws]
    _, g0, _ = oracle.mlp_backward(X, Ws, y)
    lr = min(float(np.min(np.abs(w[w != 0])) * 2.0 ** -10 / np.max(np.abs(g))) for w, g in zip(W0, g0))
    _, plain, _ = oracle.mlp_step(X, Ws, y, lr)
    assert all(np.array_equal(oracle.round_bf16_nearest(p.astype(np.float32)), w) for p, w in zip(plain, Ws))
    M = [w.astype(np.float32) for w in W0]
    W, total, n = list(Ws), [np.zeros(w.shape) for w in Ws], 0
    while n < 2000 and all(np.array_equal(a, b) for a, b in zip(W, Ws)):
        _, g, _ = oracle.mlp_backward(X, W, y)
        _, W, M, _ = oracle.mlp_step_master(X, W, y, lr, M)
        total = [t + x for t, x in zip(total, g)]
        n += 1
    assert 2 < n < 2000                                   # no single step could move a weight; their sum does
    for l in range(2):
        # the master copy holds the sum of all steps (fp32 rounding of n additions aside)
        assert np.allclose(M[l].astype(np.float64), W0[l] - lr * total[l], rtol=n * 2.0 ** -24, atol=0)
        # and the weights that moved went one bf16 neighbour in the direction of -gradient
        moved = W[l] != Ws[l]
        if moved.any():
            step = _bf16_val(W[l])[moved] - W0[l][moved]
            assert np.all(np.sign(step) == -np.sign(total[l][moved]))
