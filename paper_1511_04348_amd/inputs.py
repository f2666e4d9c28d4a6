"""Seeded synthetic inputs (no GEMM / MLP arithmetic lives here).

A counter-based generator: element ``idx`` of stream ``seed`` is a pure
function of (seed, idx), so any entry of a 17 GB matrix can be regenerated
without the matrix, on the CPU or on the GPU, with identical bits.  The mixer
is the splitmix64 finaliser (Steele, Lea, Flood 2014), evaluated with torch's
wrapping int64 arithmetic so the same code runs on either device.

Distributions follow the workloads: GEMM operands i.i.d. uniform on [-1, 1)
(the square single-precision products of section 4.1 of the paper), MLP
inputs N(0,1), weights N(0, std 0.01), labels uniform integers (stand-ins
for the image data set of section 4.2, which is not used).
"""
import math

import torch

_MASK64 = (1 << 64) - 1


def _s64(v):
    """Python int (mod 2^64) -> the signed value torch.int64 holds for the same bits."""
    v &= _MASK64
    return v - (1 << 64) if v >= (1 << 63) else v


_GOLD = _s64(0x9E3779B97F4A7C15)
_M1 = _s64(0xBF58476D1CE4E5B9)
_M2 = _s64(0x94D049BB133111EB)


def _lsr(x, s):
    """Logical shift right of int64 bit patterns."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix(x):
    x = (x ^ _lsr(x, 30)) * _M1
    x = (x ^ _lsr(x, 27)) * _M2
    return x ^ _lsr(x, 31)


def _mix_py(v):
    v &= _MASK64
    v = ((v ^ (v >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    v = ((v ^ (v >> 27)) * 0x94D049BB133111EB) & _MASK64
    return v ^ (v >> 31)


def hash64(seed, idx, lane=0):
    """64 random bits (as int64) for each flat index in ``idx`` (int64 tensor)."""
    base = _s64(_mix_py(seed * 2 + 1 + (lane << 32)))
    return _mix(idx * _GOLD + base)


def uniform_pm1_at(seed, idx):
    """U[-1,1) values on a 2^-23 grid (exact in fp32) at flat indices ``idx``."""
    u = _lsr(hash64(seed, idx), 40)                 # 24 bits
    return (u - (1 << 23)).to(torch.float32) * (1.0 / (1 << 23))


def small_int_at(seed, idx, lo=-2, hi=2):
    """Integer-valued fp32 entries in [lo, hi]: sums of products stay exact in fp32."""
    u = _lsr(hash64(seed, idx), 33) % (hi - lo + 1)
    return (u + lo).to(torch.float32)


def _chunks(total, chunk):
    for s in range(0, total, chunk):
        yield s, min(total, s + chunk)


def fill(out, seed, kind="uniform", chunk=1 << 26, gen_device=None, **kw):
    """Fills a contiguous tensor ``out`` (any device, possibly pinned host memory) in
    chunks; generation runs on ``gen_device`` (default: out's device)."""
    flat = out.view(-1)
    dev = torch.device(gen_device) if gen_device is not None else out.device
    for s, e in _chunks(flat.numel(), chunk):
        idx = torch.arange(s, e, dtype=torch.int64, device=dev)
        if kind == "uniform":
            v = uniform_pm1_at(seed, idx)
        elif kind == "int":
            v = small_int_at(seed, idx, **kw)
        elif kind == "normal":
            v = normal_at(seed, idx, **kw)
        else:
            raise ValueError(kind)
        flat[s:e].copy_(v.to(out.dtype))
    return out


def uniform_matrix(seed, rows, cols, device="cpu", dtype=torch.float32):
    return fill(torch.empty(rows, cols, dtype=dtype, device=device), seed, "uniform")


def int_matrix(seed, rows, cols, device="cpu", dtype=torch.float32, lo=-2, hi=2):
    return fill(torch.empty(rows, cols, dtype=dtype, device=device), seed, "int", lo=lo, hi=hi)


def normal_at(seed, idx, std=1.0):
    """N(0, std) by Box-Muller in fp64 from two 53-bit uniforms."""
    u1 = (_lsr(hash64(seed, idx, lane=1), 11) + 1).to(torch.float64) * (1.0 / (1 << 53))
    u2 = _lsr(hash64(seed, idx, lane=2), 11).to(torch.float64) * (1.0 / (1 << 53))
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2) * std


def normal_matrix(seed, rows, cols, std=1.0, device="cpu", dtype=torch.float32):
    return fill(torch.empty(rows, cols, dtype=dtype, device=device), seed, "normal", std=std)


def labels(seed, n, n_classes, device="cpu"):
    idx = torch.arange(n, dtype=torch.int64, device=device)
    return (_lsr(hash64(seed, idx, lane=3), 1) % n_classes).to(torch.int32)


def bf16_bits(t):
    """numpy uint16 view of a bfloat16 tensor's bit patterns (CPU copy)."""
    import numpy as np
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)
