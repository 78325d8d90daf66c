"""Pins of the oracle of the non-uniform codebook variant (oracle/aq_codebook_oracle.py) against things other than
itself: the published E2M1 value list, a hand-worked block, the base format's own (pinned) oracle for the uniform
table, an exact rational brute force, and closed-form properties of the nearest-level assignment.  No GPU."""
import os
from fractions import Fraction

import numpy as np
import pytest

import aq_workloads as wl
from oracle import aq_codebook_oracle as cb
from oracle import aq_oracle as ao

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "e2m1_levels.txt")


def golden():
    return {l.split()[0]: [float(v) for v in l.split()[1:]] for l in open(GOLDEN) if l.strip() and not l.startswith("#")}


def f16(v):
    return wl.f32_to_f16_bits(np.asarray(v, dtype=np.float32))


def test_e2m1_levels_are_the_published_ones():
    want = np.array(golden()["levels"])
    got = cb.e2m1_levels()
    assert np.array_equal(got, want)
    assert np.array_equal(np.signbit(got), np.signbit(want))            # pattern 8 is the negative zero
    assert got.max() == 6.0 and np.min(np.abs(got[np.abs(got) >= 1.0])) == 1.0
    assert sorted(set(np.abs(got))) == [0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0]


def test_hand_worked_block():
    g = golden()
    q = np.array([[k % 4 for k in range(32)]], dtype=np.uint8)
    stream = ao.pack(q, 2)
    scales = f16([[0.5]])
    W = cb.dequant(stream, scales, g["table2"], 1, 32, 2)
    assert W[0, :4].tolist() == g["w_first4"]
    assert cb.qmatmul(stream, scales, g["table2"], 1, 32, 2, f16(np.ones(32)), "f16")[0, 0] == g["y_ones"][0]
    assert cb.qmatmul(stream, scales, g["table2"], 1, 32, 2, f16(np.arange(32) % 4), "f16")[0, 0] == g["y_ramp"][0]


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_uniform_table_is_the_base_format(bits):
    N, K = 9, 352
    codes, scales = wl.draw_matrix(N, K, bits, 71, bits)
    assert np.array_equal(cb.dequant(codes, scales, cb.uniform_levels(bits), N, K, bits), ao.dequant(codes, scales, N, K, bits))
    X = wl.draw_activations(3, K, "bf16", 71, bits)
    assert np.array_equal(cb.qmatmul(codes, scales, cb.uniform_levels(bits), N, K, bits, X, "bf16"),
                          ao.activations_to_f64(X, "bf16") @ ao.dequant(codes, scales, N, K, bits).T)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_rational_brute_force(bits):
    """Every weight and every dot product in exact rational arithmetic on a tiny case (levels with short binary
    expansions, so that float64 is exact too and the comparison can be for equality)."""
    N, K, M = 3, 64, 2
    rng = np.random.default_rng(72 + bits)
    levels = (rng.integers(-40, 41, size=1 << bits) / 8.0).astype(np.float64)
    codes, scales = wl.draw_matrix(N, K, bits, 72, bits)
    X = wl.draw_int_activations(M, K, "f16", 72, bits)
    q = ao.unpack(codes, N, K, bits)
    s = ao.f16_to_f64(scales)
    Xf = ao.activations_to_f64(X, "f16")
    Y = cb.qmatmul(codes, scales, levels, N, K, bits, X, "f16")
    for m in range(M):
        for n in range(N):
            acc = Fraction(0)
            for k in range(K):
                acc += Fraction(float(Xf[m, k])) * Fraction(float(s[n, k // 32])) * Fraction(float(levels[q[n, k]]))
            assert Fraction(float(Y[m, n])) == acc


def test_a_permuted_table_with_permuted_codes_gives_the_same_weights():
    N, K, bits = 4, 96, 4
    codes, scales = wl.draw_matrix(N, K, bits, 73)
    levels = cb.e2m1_levels() * 0.37
    perm = np.random.default_rng(73).permutation(16)                     # new code of old code q: perm[q]
    q = ao.unpack(codes, N, K, bits)
    new_levels = np.empty(16); new_levels[perm] = levels
    W0 = cb.dequant(codes, scales, levels, N, K, bits)
    W1 = cb.dequant(ao.pack(perm[q].astype(np.uint8), bits), scales, new_levels, N, K, bits)
    assert np.array_equal(W0, W1)


def test_nearest_codes():
    levels = cb.e2m1_levels()[:8]                                        # 0 .. 6, ascending
    s = 0.25
    assert cb.nearest_codes(s * levels, s, levels).tolist() == list(range(8))         # a level maps to itself
    # midpoints go to the first (lower) entry; just above them to the upper one
    mids = s * (levels[:-1] + levels[1:]) / 2
    assert cb.nearest_codes(mids, s, levels).tolist() == list(range(7))
    assert cb.nearest_codes(np.nextafter(mids, np.inf), s, levels).tolist() == list(range(1, 8))
    assert cb.nearest_codes(np.array([-9.0, 9.0]), s, levels).tolist() == [0, 7]      # beyond the table: its ends
    # against a loop, on an unsorted table with a duplicate
    table = np.array([0.3, -1.0, 0.3, 2.5])
    w = np.random.default_rng(74).normal(size=50)
    want = [min(range(4), key=lambda c: (abs(x - 0.7 * table[c]), c)) for x in w]
    assert cb.nearest_codes(w, 0.7, table).tolist() == want
