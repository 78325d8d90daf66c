"""CPU oracle for the non-uniform codebook variant of the block format (TEST INFRASTRUCTURE, not product code; parity
pinned by tests/test_codebook_oracle_pins.py).

What it follows (Section 3, "Weight quantization", Eq. 1 and the sentence after it: the codes of a format come from a
format-specific codebook of representable values that may be uniform or non-uniform): a block b of B = 32 consecutive
weights of a row has one binary16 scale s_b, a code q_i of `bits` bits selects one of 2^bits levels of a table L that
belongs to the matrix's format,

    w_hat_i = s_b * L[q_i],        q_i = argmin over the table of |w_i - s_b L[q]|   (right part of Eq. 1).

The base format is the table L[q] = q - 2^(bits-1).  Reading (the paper names no non-uniform table): L is any list of
2^bits real numbers given with the matrix; the 4-bit minifloat grid E2M1 (one sign, two exponent, one mantissa bit) is
provided as the table the target hardware multiplies natively.

Canonical arrays (what the library's pack entry point takes):
    stream  uint8 [N][K/32][4*bits]   the code bitstream of the base format
    scales  uint16[N][K/32]           binary16 bit patterns of s_b
    levels  float [2^bits]            the table L

Plain numpy in float64, one step after the other.
"""
from __future__ import annotations

import numpy as np

from . import aq_oracle as ao

BLOCK = 32


def e2m1_value(pattern: int) -> float:
    """The number a 4-bit pattern s e1 e0 m denotes: (-1)^s * 2^(e-1) * (1 + m/2) for e > 0, (-1)^s * m/2 for e = 0
    (exponent bias 1, one subnormal)."""
    s, e, m = (pattern >> 3) & 1, (pattern >> 1) & 3, pattern & 1
    mag = 0.5 * m if e == 0 else 2.0 ** (e - 1) * (1.0 + 0.5 * m)
    return -mag if s else mag


def e2m1_levels() -> np.ndarray:
    """float64[16]: level of code q = the E2M1 number with bit pattern q."""
    return np.array([e2m1_value(p) for p in range(16)], dtype=np.float64)


def uniform_levels(bits: int) -> np.ndarray:
    """The base format as a table: L[q] = q - 2^(bits-1)."""
    return np.arange(1 << bits, dtype=np.float64) - float(1 << (bits - 1))


def dequant(stream: np.ndarray, scales: np.ndarray, levels, N: int, K: int, bits: int) -> np.ndarray:
    """w_hat float64 [N, K] = s_b * L[q]."""
    L = np.asarray(levels, dtype=np.float64).reshape(1 << bits)
    q = ao.unpack(stream, N, K, bits)
    s = ao.f16_to_f64(np.asarray(scales, dtype=np.uint16).reshape(N, K // BLOCK))
    return np.repeat(s, BLOCK, axis=1) * L[q]


def qmatmul(stream, scales, levels, N: int, K: int, bits: int, X_bits: np.ndarray, x_dtype: str) -> np.ndarray:
    """Y[M, N] = X W_hat^T for activations given as uint16 bit patterns of `x_dtype`, [M, K]."""
    X = ao.activations_to_f64(np.asarray(X_bits, dtype=np.uint16).reshape(-1, K), x_dtype)
    return X @ dequant(stream, scales, levels, N, K, bits).T


def nearest_codes(w: np.ndarray, s: float, levels) -> np.ndarray:
    """q_i = the first table entry that minimises |w_i - s L[q]| (uint8, same shape as w)."""
    L = np.asarray(levels, dtype=np.float64)
    w = np.asarray(w, dtype=np.float64)
    err = np.abs(w[..., None] - s * L)
    return np.argmin(err, axis=-1).astype(np.uint8)          # argmin returns the first minimiser
