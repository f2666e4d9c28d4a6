"""Stochastic rounding of fp32 values to bf16 (test infrastructure only).

The paper's update (section 2: parameters change by the error derivative
after the two passes) is silent on storage precision.  For bf16 weights the
library offers, besides round-to-nearest-even, the classical stochastic
rounding: of the two bf16 neighbours of the fp32 result take the one of
larger magnitude with probability equal to the dropped fraction, so that the
stored value equals the fp32 result in expectation and a value bf16 holds
exactly never moves.  Written out on bit patterns (sign-magnitude, so adding
to the pattern moves the magnitude): add 16 uniform random bits below the cut
and truncate.

The random bits are those the C ABI documents (``mlp_set_rounding``): a
counter-based generator built from the 32-bit finalizer of MurmurHash3, all
arithmetic modulo 2^32.  This module implements it on its own, in numpy uint64
arithmetic with explicit masks (no reliance on wrap-around of a narrower type).
"""
import numpy as np

_M32 = np.uint64(0xFFFFFFFF)


def _u64(x):
    return np.asarray(x, dtype=np.uint64) & _M32


def mix32(x):
    """MurmurHash3's 32-bit finalizer, a bijection of the integers modulo 2^32."""
    x = _u64(x)
    x = x ^ (x >> np.uint64(16))
    x = (x * np.uint64(0x85EBCA6B)) & _M32
    x = x ^ (x >> np.uint64(13))
    x = (x * np.uint64(0xC2B2AE35)) & _M32
    x = x ^ (x >> np.uint64(16))
    return x


def step_key(seed, layer, step):
    """Key of one update of one layer (layer counts from 1, step from 0)."""
    seed = int(seed)
    k = mix32(seed & 0xFFFFFFFF)
    k = mix32(k ^ np.uint64((seed >> 32) & 0xFFFFFFFF))
    k = mix32(k ^ np.uint64(int(layer) & 0xFFFFFFFF))
    k = mix32(k ^ np.uint64(int(step) & 0xFFFFFFFF))
    return int(k)


def rounding_bits(key, rows, cols):
    """16 random bits for every (row, col) pair; rows and cols broadcast against each other."""
    rows = _u64(rows)
    cols = np.asarray(cols, dtype=np.uint64)
    hrow = mix32((rows + np.uint64(key)) & _M32)
    pair = (hrow + (((cols >> np.uint64(1)) * np.uint64(0x9E3779B9)) & _M32)) & _M32
    bits = mix32(pair)
    odd = (cols & np.uint64(1)).astype(bool)
    return np.where(odd, bits >> np.uint64(16), bits & np.uint64(0xFFFF)).astype(np.uint32)


def stochastic_round_bf16(x, r16):
    """fp32 array -> bf16 bit patterns (uint16), given 16 random bits per entry.

    Infinities are unchanged and NaNs stay NaNs (quiet bit set), as under nearest-even."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    r = np.asarray(r16, dtype=np.uint64)
    out = ((u + r) >> np.uint64(16)) & np.uint64(0xFFFF)
    special = (u & np.uint64(0x7F800000)) == np.uint64(0x7F800000)
    is_nan = special & ((u & np.uint64(0x007FFFFF)) != 0)
    keep = (u >> np.uint64(16)) | np.where(is_nan, np.uint64(0x40), np.uint64(0))
    return np.where(special, keep, out).astype(np.uint16)


def round_bf16_nearest(x):
    """fp32 array -> bf16 bit patterns (uint16), round to nearest, ties to the even bf16 pattern.

    Written from the definition on the two neighbours, not as an add-and-shift: the candidate below
    (in magnitude) is the pattern with the low 16 bits cut, the one above is the next bf16 pattern;
    the nearer wins, and at the midpoint the one whose last kept bit is 0.  Infinities are unchanged
    and NaNs stay NaNs (quiet bit set)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    low = u & np.uint64(0xFFFF)
    down = u >> np.uint64(16)
    up = down + np.uint64(1)              # sign-magnitude: the next pattern is the next magnitude
    half = np.uint64(0x8000)
    take_up = (low > half) | ((low == half) & ((down & np.uint64(1)) == np.uint64(1)))
    out = np.where(take_up, up, down) & np.uint64(0xFFFF)
    special = (u & np.uint64(0x7F800000)) == np.uint64(0x7F800000)
    is_nan = special & ((u & np.uint64(0x007FFFFF)) != 0)
    keep = np.where(is_nan, down | np.uint64(0x40), down)
    return np.where(special, keep, out).astype(np.uint16)


def stochastic_round_matrix(W32, seed, layer, step):
    """Rounds a whole weight matrix (fp32, 2-D) for update `step` of `layer`."""
    W32 = np.ascontiguousarray(W32, dtype=np.float32)
    n_r, n_c = W32.shape
    key = step_key(seed, layer, step)
    bits = rounding_bits(key, np.arange(n_r, dtype=np.uint64)[:, None], np.arange(n_c, dtype=np.uint64)[None, :])
    return stochastic_round_bf16(W32, bits)
