"""Pins of the GEMM oracle against facts it does not compute itself: closed forms,
numpy's fp64 matmul, a pure-Python triple loop, exact integer arithmetic."""
import itertools

import numpy as np
import pytest


def _rng(seed):
    return np.random.default_rng(seed)


def _to_bf16_bits(x):
    """Round-to-nearest-even fp32 -> bf16 bit patterns, done with integer arithmetic."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    r = ((u >> 16) & 1) + 0x7FFF
    return ((u + r) >> 16).astype(np.uint16)


def test_identity_zero_ones(oracle):
    n = 37
    B = _rng(0).uniform(-1, 1, (n, n)).astype(np.float32)
    Cin = _rng(1).uniform(-1, 1, (n, n)).astype(np.float32)
    eye = np.eye(n, dtype=np.float32)
    out = oracle.gemm(eye, B, c_in=Cin)
    assert np.array_equal(out, Cin.astype(np.float64) + B.astype(np.float64))
    assert np.array_equal(oracle.gemm(np.zeros((n, n), np.float32), B, c_in=Cin), Cin.astype(np.float64))
    ones = oracle.gemm(np.ones((5, 23), np.float32), np.ones((23, 9), np.float32))
    assert np.array_equal(ones, np.full((5, 9), 23.0))


def test_rank1_closed_form(oracle):
    r = _rng(2)
    u, v, w, z = (r.integers(-3, 4, n).astype(np.float32) for n in (11, 17, 17, 13))
    A = np.outer(u, v).astype(np.float32)
    B = np.outer(w, z).astype(np.float32)
    expect = float(np.dot(v.astype(np.float64), w.astype(np.float64))) * np.outer(u, z).astype(np.float64)
    assert np.array_equal(oracle.gemm(A, B), expect)


@pytest.mark.parametrize("dt", ["f32", "bf16"])
def test_brute_force_vs_numpy_all_small_shapes(oracle, dt):
    r = _rng(3)
    for M, N, K in itertools.product([1, 2, 3, 5, 8], repeat=3):
        A32 = r.uniform(-1, 1, (M, K)).astype(np.float32)
        B32 = r.uniform(-1, 1, (K, N)).astype(np.float32)
        Cin = r.uniform(-1, 1, (M, N)).astype(np.float32)
        if dt == "bf16":
            A, B = _to_bf16_bits(A32), _to_bf16_bits(B32)
            A64, B64 = oracle.bf16_to_f64(A).reshape(M, K), oracle.bf16_to_f64(B).reshape(K, N)
        else:
            A, B = A32, B32
            A64, B64 = A32.astype(np.float64), B32.astype(np.float64)
        ref = Cin.astype(np.float64) + A64 @ B64
        for ta, tb in itertools.product([False, True], repeat=2):
            Aa = np.ascontiguousarray(A.T) if ta else A
            Bb = np.ascontiguousarray(B.T) if tb else B
            got = oracle.gemm(Aa, Bb, c_in=Cin, trans_a=ta, trans_b=tb)
            assert got.shape == (M, N)
            assert np.allclose(got, ref, rtol=0, atol=1e-13), (M, N, K, ta, tb)


def test_bf16_widening_is_exact(oracle):
    bits = np.array([0x3F80, 0xBF80, 0x4000, 0x3F00, 0x0000, 0x4049], dtype=np.uint16)
    # 1, -1, 2, 0.5, 0, 3.140625 (bf16 nearest below pi)
    assert np.array_equal(oracle.bf16_to_f64(bits), [1.0, -1.0, 2.0, 0.5, 0.0, 3.140625])


def test_pure_python_triple_loop(oracle):
    r = _rng(4)
    M, N, K = 4, 3, 6
    A = r.uniform(-1, 1, (M, K)).astype(np.float32)
    B = r.uniform(-1, 1, (K, N)).astype(np.float32)
    got = oracle.gemm(A, B)
    for m in range(M):
        for n in range(N):
            s = 0.0
            for k in range(K):
                s += float(A[m, k]) * float(B[k, n])
            assert got[m, n] == s  # same order, same fp64 arithmetic


def test_integer_inputs_exact(oracle):
    r = _rng(5)
    M, N, K = 45, 31, 300
    A = r.integers(-2, 3, (M, K)).astype(np.float32)
    B = r.integers(-2, 3, (K, N)).astype(np.float32)
    Cin = r.integers(-5, 6, (M, N)).astype(np.float32)
    ref = Cin.astype(np.int64) + A.astype(np.int64) @ B.astype(np.int64)
    assert np.array_equal(oracle.gemm(A, B, c_in=Cin), ref.astype(np.float64))
    assert np.array_equal(oracle.gemm_tiled(A, B, 7, c_in=Cin), ref.astype(np.float64))


def test_tiled_equals_untiled_any_T(oracle):
    r = _rng(6)
    M, N, K = 23, 19, 29
    A = r.uniform(-1, 1, (M, K)).astype(np.float32)
    B = r.uniform(-1, 1, (K, N)).astype(np.float32)
    Cin = r.uniform(-1, 1, (M, N)).astype(np.float32)
    ref = oracle.gemm(A, B, c_in=Cin)
    for T in [1, 2, 3, 7, K, K + 1, 64]:
        got = oracle.gemm_tiled(A, B, T, c_in=Cin)
        assert np.allclose(got, ref, rtol=0, atol=1e-13), T
    # transposed storage through the tiled walker as well
    got = oracle.gemm_tiled(np.ascontiguousarray(A.T), np.ascontiguousarray(B.T), 5, c_in=Cin,
                            trans_a=True, trans_b=True)
    assert np.allclose(got, ref, rtol=0, atol=1e-13)


def test_samples_match_full(oracle):
    r = _rng(7)
    M, N, K = 33, 27, 41
    A = r.uniform(-1, 1, (M, K)).astype(np.float32)
    B = r.uniform(-1, 1, (K, N)).astype(np.float32)
    Cin = r.uniform(-1, 1, (M, N)).astype(np.float32)
    full = oracle.gemm(A, B, c_in=Cin)
    rows = r.integers(0, M, 50)
    cols = r.integers(0, N, 50)
    assert np.array_equal(oracle.gemm_samples(A, B, rows, cols, c_in=Cin), full[rows, cols])
    fullt = oracle.gemm(np.ascontiguousarray(A.T), B, trans_a=True)
    assert np.array_equal(oracle.gemm_samples(np.ascontiguousarray(A.T), B, rows, cols, trans_a=True),
                          fullt[rows, cols])


def test_empty_dims(oracle):
    Cin = np.ones((3, 4), np.float32)
    out = oracle.gemm(np.zeros((3, 0), np.float32), np.zeros((0, 4), np.float32), c_in=Cin)
    assert np.array_equal(out, np.ones((3, 4)))
    assert oracle.gemm(np.zeros((0, 5), np.float32), np.zeros((5, 4), np.float32)).shape == (0, 4)
