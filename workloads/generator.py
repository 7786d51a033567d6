"""Counter-based input generator: v_{q,n}[i] is a pure function of (seed, job, q, n, i).

Recipe: h = splitmix64-finaliser(seed + GOLDEN * (1 + counter)) with
counter = (((job*Q + q)*N + n)*T + i).  uint32 payload = top 32 bits of h.
fp32 payload = Box-Muller on two 24-bit uniforms cut from h, evaluated in fp64
and rounded once to fp32.  Output layout [J][N][Q][T] (file-major).

16-bit payloads ("bf16", "f16") are the fp32 payload rounded once more, to nearest
even, to bfloat16 / IEEE binary16; the numpy backend hands them out as uint16
bit patterns, the torch backend as tensors of that dtype.

Two backends produce the same recipe: numpy (host) and torch (any device).
The uint32 payload is bit-identical across backends; the fp32 payload may
differ in the last bit between backends (log/cos implementations), so a test
always generates once and hands the same array to both sides.
"""
from __future__ import annotations

import math

import numpy as np

_GOLDEN = 0x9E3779B97F4A7C15
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_MASK64 = (1 << 64) - 1


def _mix64_np(z):
    z = (z ^ (z >> np.uint64(30))) * np.uint64(_M1)
    z = (z ^ (z >> np.uint64(27))) * np.uint64(_M2)
    return z ^ (z >> np.uint64(31))


def generate_numpy(J, N, Q, T, seed, mode, sigma=1.0):
    """Host arrays: float32 (mode "f32"), uint32 (mode "u32") or uint16 bit patterns
    (modes "bf16", "f16"), shape (J, N, Q, T)."""
    if mode in ("bf16", "f16"):
        return to_half_bits(generate_numpy(J, N, Q, T, seed, "f32", sigma), mode)
    out = np.empty((J, N, Q, T), dtype=np.float32 if mode == "f32" else np.uint32)
    i = np.arange(T, dtype=np.uint64)[None, :]
    q = np.arange(Q, dtype=np.uint64)[:, None]
    with np.errstate(over="ignore"):
        for j in range(J):
            for n in range(N):
                ctr = ((np.uint64(j * Q) + q) * np.uint64(N) + np.uint64(n)) * np.uint64(T) + i
                h = _mix64_np(np.uint64(seed & _MASK64) + np.uint64(_GOLDEN) * (np.uint64(1) + ctr))
                if mode == "u32":
                    out[j, n] = (h >> np.uint64(32)).astype(np.uint32)
                else:
                    u1 = ((h >> np.uint64(40)).astype(np.float64) + 1.0) / 16777216.0
                    u2 = ((h >> np.uint64(16)) & np.uint64(0xFFFFFF)).astype(np.float64) / 16777216.0
                    z = sigma * np.sqrt(-2.0 * np.log(u1)) * np.cos(2.0 * math.pi * u2)
                    out[j, n] = z.astype(np.float32)
    return out


def to_half_bits(values, mode):
    """uint16 patterns of float32 values rounded to nearest even, by the array libraries'
    own conversions: numpy's float16 for "f16", torch's bfloat16 for "bf16"."""
    values = np.ascontiguousarray(values, dtype=np.float32)
    if mode == "f16":
        with np.errstate(over="ignore"):
            return values.astype(np.float16).view(np.uint16)
    import torch
    return torch.from_numpy(values).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)


def half_bits_to_float(bits, mode):
    """Exact float32 values of uint16 patterns."""
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    if mode == "f16":
        return bits.view(np.float16).astype(np.float32)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _s64(x):
    """Two's-complement reinterpretation of an unsigned 64-bit constant."""
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def generate_torch(J, N, Q, T, seed, mode, sigma=1.0, device="cpu"):
    """Same recipe with torch ops (int64 arithmetic wraps mod 2^64).

    Returns float32 for "f32"; for "u32" returns an int32 tensor holding the
    uint32 bit patterns (torch has no arithmetic uint32 type); bfloat16 / float16
    tensors for "bf16" / "f16"."""
    import torch

    half = {"bf16": torch.bfloat16, "f16": torch.float16}.get(mode)

    def lsr(z, s):
        return (z >> s) & ((1 << (64 - s)) - 1)

    def mix(z):
        z = (z ^ lsr(z, 30)) * _s64(_M1)
        z = (z ^ lsr(z, 27)) * _s64(_M2)
        return z ^ lsr(z, 31)

    out = torch.empty((J, N, Q, T), dtype=half or (torch.float32 if mode == "f32" else torch.int32), device=device)
    i = torch.arange(T, dtype=torch.int64, device=device)[None, :]
    q = torch.arange(Q, dtype=torch.int64, device=device)[:, None]
    q = q[None]                                       # (1, Q, 1)
    i = i[None]                                       # (1, 1, T)
    step = max(1, (1 << 24) // (Q * T))               # files per block: about 16M elements at a time
    for j in range(J):
        for n0 in range(0, N, step):
            n = torch.arange(n0, min(N, n0 + step), dtype=torch.int64, device=device)[:, None, None]
            ctr = ((j * Q + q) * N + n) * T + i
            h = mix(_s64(seed) + _s64(_GOLDEN) * (1 + ctr))
            if mode == "u32":
                out[j, n0:n0 + step] = lsr(h, 32).to(torch.int32)   # wraps: keeps the low 32 bits
            else:
                u1 = (lsr(h, 40).to(torch.float64) + 1.0) / 16777216.0
                u2 = (lsr(h, 16) & 0xFFFFFF).to(torch.float64) / 16777216.0
                z = sigma * torch.sqrt(-2.0 * torch.log(u1)) * torch.cos(2.0 * math.pi * u2)
                z = z.to(torch.float32)
                out[j, n0:n0 + step] = z.to(half) if half else z
    return out
