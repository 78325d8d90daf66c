"""CPU oracle for the two-level variant of the block format (TEST INFRASTRUCTURE, not product code; parity pinned
by tests/test_affine_oracle_pins.py).

What it follows (Section 3, "Weight quantization", Eq. 1 in its general form): a block b of B = 32 consecutive
weights of a row has its own scale s_b and its own real zero point z_b,

    w_hat_i = s_b (q_i - z_b),      q_i in {0 .. 2^bits - 1},

and S = 8 consecutive blocks form a super-block whose own parameters compress the per-block (s_b, z_b).
Reading (the paragraph does not say how): the block's scale and the block's offset s_b z_b are each stored as a
4-bit code, multiplied by one binary16 number of the super-block:

    s_b = D_S * a_b,    s_b z_b = M_S * c_b,    a_b, c_b in {0 .. 15}
    w_hat_i = D_S a_b q_i - M_S c_b.

Stored bits per weight: bits + 8/32 + 32/256 = bits + 0.375.

Canonical arrays (what the library's pack entry point takes):
    stream  uint8 [N][K/32][4*bits]   the code bitstream of the base format
    sub     uint8 [N][K/32]           a_b in the low nibble, c_b in the high nibble
    sup     uint16[N][ceil(K/256)][2] binary16 bit patterns of D_S, M_S

Plain numpy in float64, one step after the other.
"""
from __future__ import annotations

import numpy as np

from . import aq_oracle as ao

BLOCK = 32
SUPER = 8          # blocks per super-block


def stored_bits_per_weight(bits: int) -> float:
    return bits + 8.0 / BLOCK + 32.0 / (BLOCK * SUPER)


def block_parameters(sub: np.ndarray, sup: np.ndarray, N: int, K: int):
    """(s_b, s_b z_b) per block, float64 [N, K/32]."""
    nb = K // BLOCK
    sub = np.asarray(sub, dtype=np.uint8).reshape(N, nb)
    sup = np.asarray(sup, dtype=np.uint16).reshape(N, -1, 2)
    a = (sub & 15).astype(np.float64)
    c = (sub >> 4).astype(np.float64)
    D = ao.f16_to_f64(sup[:, :, 0])
    M = ao.f16_to_f64(sup[:, :, 1])
    which = np.arange(nb) // SUPER                       # super-block of every block
    return D[:, which] * a, M[:, which] * c


def dequant(stream: np.ndarray, sub: np.ndarray, sup: np.ndarray, N: int, K: int, bits: int) -> np.ndarray:
    """w_hat float64 [N, K]."""
    q = ao.unpack(stream, N, K, bits).astype(np.float64)
    s, sz = block_parameters(sub, sup, N, K)
    return np.repeat(s, BLOCK, axis=1) * q - np.repeat(sz, BLOCK, axis=1)


def qmatvec(stream, sub, sup, N: int, K: int, bits: int, x_bits: np.ndarray, x_dtype: str) -> np.ndarray:
    """y = W_hat x for one activation vector given as uint16 bit patterns of `x_dtype`."""
    x = ao.activations_to_f64(np.asarray(x_bits, dtype=np.uint16).reshape(1, K), x_dtype)[0]
    return dequant(stream, sub, sup, N, K, bits) @ x
