"""Stateless counter-based random numbers (splitmix64 finaliser + Box-Muller).

Every draw is a pure function of (seed, tag, row id, component), so a tensor can
be produced in any chunking, on any device, in any order.
"""
from __future__ import annotations

import math

import torch

_MASK64 = (1 << 64) - 1
_M1 = 0xBF58476D1CE4E5B9
_M2 = 0x94D049BB133111EB
_GOLD = 0x9E3779B97F4A7C15
_ALT = 0xD6E8FEB86659FD93


def _signed(x: int) -> int:
    x &= _MASK64
    return x - (1 << 64) if x >= (1 << 63) else x


def mix64_int(x: int) -> int:
    """splitmix64 finaliser on a Python int (unsigned 64-bit result)."""
    x &= _MASK64
    x ^= x >> 30
    x = (x * _M1) & _MASK64
    x ^= x >> 27
    x = (x * _M2) & _MASK64
    x ^= x >> 31
    return x


def _lsr(x: torch.Tensor, s: int) -> torch.Tensor:
    # logical shift right on int64 (torch's >> is arithmetic)
    return (x >> s) & ((1 << (64 - s)) - 1)


def mix64(x: torch.Tensor) -> torch.Tensor:
    """splitmix64 finaliser on an int64 tensor (two's-complement wrap-around)."""
    x = x ^ _lsr(x, 30)
    x = x * _signed(_M1)
    x = x ^ _lsr(x, 27)
    x = x * _signed(_M2)
    x = x ^ _lsr(x, 31)
    return x


def stream_key(seed: int, tag: int) -> int:
    """Scalar key of one random stream (one tensor kind of one sequence)."""
    return mix64_int(mix64_int(seed) ^ ((tag * _GOLD) & _MASK64))


def uniform_u64(seed: int, tag: int, counter: int) -> int:
    """One unsigned 64-bit draw on the host (scalar processes: centres, lengths)."""
    return mix64_int(stream_key(seed, tag) ^ ((counter * _GOLD) & _MASK64))


def normal_rows(seed: int, tag: int, row_ids: torch.Tensor, d: int) -> torch.Tensor:
    """N(0,1) draws, one row of ``d`` components per entry of ``row_ids``.

    row_ids: int64 tensor of any shape (unique id per row within the stream).
    Returns float64 of shape row_ids.shape + (d,).
    """
    dev = row_ids.device
    rk = mix64(row_ids.to(torch.int64) * _signed(_GOLD) ^ _signed(stream_key(seed, tag)))
    comp = (torch.arange(1, d + 1, device=dev, dtype=torch.int64) * _signed(_ALT))
    x1 = mix64(rk.unsqueeze(-1) + comp)
    x2 = mix64(x1 ^ _signed(_GOLD))
    u1 = (_lsr(x1, 11).to(torch.float64) + 1.0) * (2.0 ** -53)      # (0, 1]
    u2 = _lsr(x2, 11).to(torch.float64) * (2.0 ** -53)              # [0, 1)
    return torch.sqrt(-2.0 * torch.log(u1)) * torch.cos((2.0 * math.pi) * u2)
