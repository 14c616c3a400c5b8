"""Counter-based seeded random streams for the synthetic workloads.

Every value is a pure function of (seed, stream id, element index), so a tensor can be
generated in pieces, in any order and on any torch device.  The integer part (the 64-bit
mix) is bit-identical everywhere; the float part (Box-Muller in fp32) may differ in the
last ulp between devices, which is why every consumer of a generated tensor, the CPU
oracle included, is always fed the bytes of one realised tensor and never a second
generation of it.

This module holds no arithmetic of the attention method itself.
"""
from __future__ import annotations

import math

import torch

_MASK64 = (1 << 64) - 1
# Odd 64-bit constants of the splitmix64 finaliser, written as signed int64.
_GOLDEN = 0x9E3779B97F4A7C15 - (1 << 64)
_MUL1 = 0xBF58476D1CE4E5B9 - (1 << 64)
_MUL2 = 0x94D049BB133111EB - (1 << 64)


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    """Logical right shift of an int64 tensor (torch's >> is arithmetic)."""
    return (x >> s) & ((1 << (64 - s)) - 1)


def _mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on int64 tensors (two's-complement wrap-around)."""
    x = (x ^ _lsr(x, 30)) * _MUL1
    x = (x ^ _lsr(x, 27)) * _MUL2
    return x ^ _lsr(x, 31)


def _mix64_int(x: int) -> int:
    x &= _MASK64
    x = ((x ^ (x >> 30)) * 0xBF58476D1CE4E5B9) & _MASK64
    x = ((x ^ (x >> 27)) * 0x94D049BB133111EB) & _MASK64
    return x ^ (x >> 31)


def stream_key(seed: int, *ids: int) -> int:
    """Fold a seed and a tuple of small integers (tensor id, layer, ...) into one key."""
    k = _mix64_int(seed ^ 0x5851F42D4C957F2D)
    for i in ids:
        k = _mix64_int(k ^ ((int(i) + 1) * 0x9E3779B97F4A7C15))
    return k


def _signed(k: int) -> int:
    return k - (1 << 64) if k >= (1 << 63) else k


def random_bits(key: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """64 random bits for each of the element indices [start, start+count)."""
    ctr = torch.arange(start, start + count, dtype=torch.int64, device=device)
    return _mix64(ctr * _GOLDEN + _signed(key))


def uniform(key: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """fp32 uniforms in [0, 1): the top 24 bits of the stream, exactly representable."""
    bits = random_bits(key, start, count, device)
    return _lsr(bits, 40).to(torch.float32) * (1.0 / (1 << 24))


def normal(key: int, start: int, count: int, device="cpu") -> torch.Tensor:
    """fp32 standard normals by Box-Muller from two 24-bit slices of one 64-bit draw."""
    bits = random_bits(key, start, count, device)
    u1 = (_lsr(bits, 40).to(torch.float32) + 0.5) * (1.0 / (1 << 24))  # (0, 1)
    u2 = ((_lsr(bits, 16) & 0xFFFFFF).to(torch.float32)) * (1.0 / (1 << 24))  # [0, 1)
    r = torch.sqrt(-2.0 * torch.log(u1))
    return r * torch.cos((2.0 * math.pi) * u2)


def choice_without_replacement(key: int, n: int, k: int) -> list[int]:
    """k distinct integers in [0, n), ascending, drawn by rejection from the stream."""
    out: list[int] = []
    i = 0
    while len(out) < k:
        v = _mix64_int((key + i * 0x9E3779B97F4A7C15) & _MASK64) % n
        if v not in out:
            out.append(v)
        i += 1
    return sorted(out)
