"""Pins of the oracle of the two-level format variant (oracle/aq_affine_oracle.py) against things other than
itself: a hand-worked row, the base format's own oracle (the variant with M = D z and c = a IS the base format), Eq. 1
in its (s_b, z_b) form, and a brute-force loop.  No GPU."""
import os

import numpy as np
import pytest

import aq_workloads as wl
from oracle import aq_affine_oracle as af
from oracle import aq_oracle as ao

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "affine_format_example.txt")


def f16(v):
    return wl.f32_to_f16_bits(np.asarray(v, dtype=np.float32))


def test_hand_worked_row():
    g = {l.split()[0]: [float(v) for v in l.split()[1:]] for l in open(GOLDEN) if l.strip() and not l.startswith("#")}
    q = np.array([[k % 4 for k in range(32)] + [3 - k % 4 for k in range(32)]], dtype=np.uint8)
    stream = ao.pack(q, 2)
    sub = np.array([[int(g["a"][0]) | (int(g["c"][0]) << 4), int(g["a"][1]) | (int(g["c"][1]) << 4)]], dtype=np.uint8)
    sup = np.array([[[f16(g["D"][0]), f16(g["M"][0])]]], dtype=np.uint16).reshape(1, 1, 2)
    W = af.dequant(stream, sub, sup, 1, 64, 2)
    assert W[0, :4].tolist() == g["w_block0"] and W[0, 32:36].tolist() == g["w_block1"]
    ones = f16(np.ones(64))
    ramp = f16(np.arange(64) % 4)
    assert af.qmatvec(stream, sub, sup, 1, 64, 2, ones, "f16")[0] == g["y_ones"][0]
    assert af.qmatvec(stream, sub, sup, 1, 64, 2, ramp, "f16")[0] == g["y_ramp"][0]
    assert af.stored_bits_per_weight(2) == g["bpw"][0]


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_reduces_to_the_base_format(bits):
    """c = a and M = D * 2^(bits-1): w_hat = D a (q - 2^(bits-1)), the base format with d = D a."""
    N, K = 24, 544
    rng = np.random.default_rng(bits)
    codes = wl.draw_codes(N, K, bits, 61, bits)
    a = rng.integers(0, 16, size=(N, K // 32)).astype(np.uint8)
    D = (rng.integers(1, 64, size=(N, 3)) * 2.0 ** rng.integers(-12, -4, size=(N, 3))).astype(np.float32)   # 6-bit mantissas
    sup = np.stack([f16(D), f16(D * (1 << (bits - 1)))], axis=2)
    sub = (a | (a << 4)).astype(np.uint8)
    d = D[:, np.arange(K // 32) // 8] * a                        # exact in binary16: 6 + 4 bits
    base = ao.dequant(codes, f16(d), N, K, bits)
    assert np.array_equal(af.dequant(codes, sub, sup, N, K, bits), base)


def test_general_form_of_eq1_and_brute_force():
    N, K, bits = 5, 320, 3
    codes = wl.draw_codes(N, K, bits, 62)
    sub, sup = wl.draw_affine_params(N, K, bits, 62)
    W = af.dequant(codes, sub, sup, N, K, bits)
    q = ao.unpack(codes, N, K, bits)
    s, sz = af.block_parameters(sub, sup, N, K)
    for n in range(N):
        for k in range(K):
            b, S = k // 32, k // 256
            D = float(ao.f16_to_f64(sup[n, S, 0:1])[0]); M = float(ao.f16_to_f64(sup[n, S, 1:2])[0])
            a_, c_ = int(sub[n, b]) & 15, int(sub[n, b]) >> 4
            assert W[n, k] == D * a_ * int(q[n, k]) - M * c_
            if s[n, b] != 0.0:                                   # Eq. 1: s_b (q - z_b)
                z = sz[n, b] / s[n, b]
                assert abs(W[n, k] - s[n, b] * (int(q[n, k]) - z)) <= 1e-15 * max(1.0, abs(sz[n, b]))
    x = wl.draw_activations(1, K, "bf16", 62)[0]
    xf = ao.activations_to_f64(x.reshape(1, K), "bf16")[0]
    y = af.qmatvec(codes, sub, sup, N, K, bits, x, "bf16")
    for n in range(N):
        acc = 0.0
        for k in range(K):
            acc += W[n, k] * xf[k]
        assert abs(y[n] - acc) <= 1e-12 * np.abs(W[n] * xf).sum()
