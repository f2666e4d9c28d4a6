"""ctypes front end of oracle_gemm.c (test infrastructure only).

All results are fp64.  Operands are numpy arrays: float32, or uint16 holding
bf16 bit patterns.  ``trans_a`` / ``trans_b`` select the stored orientation:
with trans_a the array holds op(A) transposed (shape K x M), as in the
backward-pass products of section 2 (equations 3 and 4).
"""
import ctypes

import numpy as np

from .build import build_oracle

_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build_oracle())
        i64, vp, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_int
        lib.oracle_gemm.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, i64, ci]
        lib.oracle_gemm.restype = ci
        lib.oracle_gemm_tiled.argtypes = [vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, i64, i64, ci]
        lib.oracle_gemm_tiled.restype = ci
        lib.oracle_gemm_samples.argtypes = [vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, i64, i64, i64, ci]
        lib.oracle_gemm_samples.restype = ci
        lib.oracle_num_threads.restype = ci
        _lib = lib
    return _lib


def num_threads():
    return int(_load().oracle_num_threads())


def bf16_to_f64(u16):
    """Exact widening of bf16 bit patterns (uint16 array) to fp64."""
    u = np.ascontiguousarray(u16, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return u.view(np.float32).astype(np.float64)


def _dtype_code(a):
    if a.dtype == np.float32:
        return 0
    if a.dtype == np.uint16:
        return 1
    raise TypeError("oracle operands must be float32 or uint16 (bf16 bits), got %s" % a.dtype)


def _prep(A, B, c_in, trans_a, trans_b):
    A = np.ascontiguousarray(A)
    B = np.ascontiguousarray(B)
    if A.ndim != 2 or B.ndim != 2:
        raise ValueError("2-D operands required")
    code = _dtype_code(A)
    if _dtype_code(B) != code:
        raise TypeError("A and B must share a dtype")
    if trans_a:
        K, M = A.shape
        sam, sak = 1, A.shape[1]
    else:
        M, K = A.shape
        sam, sak = A.shape[1], 1
    if trans_b:
        N, Kb = B.shape
        sbk, sbn = 1, B.shape[1]
    else:
        Kb, N = B.shape
        sbk, sbn = B.shape[1], 1
    if K != Kb:
        raise ValueError("inner dimensions differ: %d vs %d" % (K, Kb))
    if c_in is not None:
        c_in = np.ascontiguousarray(c_in, dtype=np.float32)
        if c_in.shape != (M, N):
            raise ValueError("c_in shape")
    return A, B, c_in, code, M, N, K, sam, sak, sbk, sbn


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def gemm(A, B, c_in=None, trans_a=False, trans_b=False):
    """C_in + op(A) @ op(B), untiled definition, fp64 result."""
    A, B, c_in, code, M, N, K, sam, sak, sbk, sbn = _prep(A, B, c_in, trans_a, trans_b)
    out = np.empty((M, N), dtype=np.float64)
    rc = _load().oracle_gemm(_ptr(A), _ptr(B), _ptr(c_in), _ptr(out), M, N, K,
                             sam, sak, sbk, sbn, N, code)
    if rc != 0:
        raise RuntimeError("oracle_gemm failed: %d" % rc)
    return out


def gemm_tiled(A, B, T, c_in=None, trans_a=False, trans_b=False):
    """Same value via the tile algorithm of section 3.1 with tile size T."""
    A, B, c_in, code, M, N, K, sam, sak, sbk, sbn = _prep(A, B, c_in, trans_a, trans_b)
    out = np.empty((M, N), dtype=np.float64)
    rc = _load().oracle_gemm_tiled(_ptr(A), _ptr(B), _ptr(c_in), _ptr(out), M, N, K, int(T),
                                   sam, sak, sbk, sbn, N, code)
    if rc != 0:
        raise RuntimeError("oracle_gemm_tiled failed: %d" % rc)
    return out


def gemm_samples(A, B, rows, cols, c_in=None, trans_a=False, trans_b=False):
    """Entries (rows[s], cols[s]) of C_in + op(A) @ op(B), each a full fp64 dot product."""
    A, B, c_in, code, M, N, K, sam, sak, sbk, sbn = _prep(A, B, c_in, trans_a, trans_b)
    rows = np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.ascontiguousarray(cols, dtype=np.int64)
    if rows.shape != cols.shape or rows.ndim != 1:
        raise ValueError("rows/cols")
    if rows.size and (rows.min() < 0 or rows.max() >= M or cols.min() < 0 or cols.max() >= N):
        raise IndexError("sample index out of range")
    out = np.empty(rows.shape, dtype=np.float64)
    rc = _load().oracle_gemm_samples(_ptr(A), _ptr(B), _ptr(c_in), _ptr(out), _ptr(rows), _ptr(cols),
                                     rows.size, K, sam, sak, sbk, sbn, N, code)
    if rc != 0:
        raise RuntimeError("oracle_gemm_samples failed: %d" % rc)
    return out
