"""Small test-side helpers: bf16 bit handling and exact rational rounding.

Nothing here is shared with the oracle or with the HIP library; the exact
rational routines exist so that the oracle's binary32 arithmetic can be checked
against the mathematical definition of IEEE rounding rather than against
another floating-point implementation.
"""
from __future__ import annotations

from fractions import Fraction

import numpy as np
import torch


def to_bf16_bits(x) -> np.ndarray:
    """float array -> uint16 bf16 bit patterns (torch's round-to-nearest-even conversion)."""
    t = torch.as_tensor(np.asarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def bits_to_f32(u16: np.ndarray) -> np.ndarray:
    return (np.asarray(u16, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def torch_bits(t: torch.Tensor) -> np.ndarray:
    """bf16 torch tensor (any device) -> uint16 numpy bit patterns."""
    assert t.dtype == torch.bfloat16
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def bits_to_torch(u16: np.ndarray, device="cpu") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).view(torch.bfloat16).to(device)


def _round_half_even(fr: Fraction) -> int:
    fl = fr.numerator // fr.denominator
    rem = fr - fl
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def round_to_binary(fr: Fraction, mant_bits: int, emin: int) -> Fraction:
    """Round an exact rational to the nearest value of a binary format with `mant_bits`
    explicit mantissa bits and minimum normal exponent `emin`, ties to even (no overflow
    handling: callers stay in range)."""
    if fr == 0:
        return Fraction(0)
    sign = -1 if fr < 0 else 1
    a = abs(fr)
    e = a.numerator.bit_length() - a.denominator.bit_length()
    if Fraction(2) ** e > a:
        e -= 1
    if Fraction(2) ** (e + 1) <= a:
        e += 1
    e = max(e, emin)
    quantum = Fraction(2) ** (e - mant_bits)
    return sign * _round_half_even(a / quantum) * quantum


def fl32(fr: Fraction) -> Fraction:
    return round_to_binary(fr, 23, -126)


def flbf16(fr: Fraction) -> Fraction:
    return round_to_binary(fr, 7, -126)


def rint_even(fr: Fraction) -> int:
    sign = -1 if fr < 0 else 1
    return sign * _round_half_even(abs(fr))


def frac_of_f32(x) -> Fraction:
    return Fraction(float(np.float32(x)))
