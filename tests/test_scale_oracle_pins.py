"""Pins of the scale-optimisation oracle (oracle/aq_scale_oracle.c) against what Section 4.2 and the
mathematics fix: a hand-worked block, the rounds = 0 special case (plain nearest-code quantisation of Eq. 1),
descent of Phi_b, least-squares optimality of the scale update, exhaustive search on 4-element blocks,
invariances, and the double -> binary16 rounding.  No GPU."""
import itertools
import os

import numpy as np
import pytest

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "scale_opt_example.txt")


def phi(w, F, q, s):
    """Eq. 10: sum_i omega_i (w_i - s q_i)^2 with omega_i = F_i sqrt(sigma_b^2 + w_i^2), one block, fp64."""
    w = np.asarray(w, dtype=np.float64)
    om = np.asarray(F, dtype=np.float64) * np.sqrt(np.mean(w * w) + w * w)
    return float(np.sum(om * (w - s * np.asarray(q, dtype=np.float64)) ** 2))


def read_golden():
    d = {}
    for line in open(GOLDEN):
        if line.startswith("#") or not line.strip():
            continue
        k, *v = line.split()
        d[k] = v
    return d


def test_hand_worked_equal_magnitude_block(oracle):
    g = read_golden()
    B, bits = int(g["block"][0]), int(g["bits"][0])
    w = np.array([float(x) for x in g["w"]], dtype=np.float32)[None, :]
    codes, scales, tr = oracle.scale_optimize(w, None, bits, 2, block=B, trace=True)
    assert list(codes[0]) == [int(x) for x in g["codes"]]
    assert int(scales[0, 0]) == int(g["scale_bits"][0], 16)
    assert tr[0, 0] == pytest.approx(float(g["phi0"][0]), rel=1e-14)
    # after round 1's scale update the 5 positive elements miss by 0.5 - 7 s1, the 3 negative by 0.5 - 8 s1
    s1 = float(g["s1"][0])
    assert tr[0, 1] == pytest.approx(np.sqrt(0.5) * (5 * (0.5 - 7 * s1) ** 2 + 3 * (0.5 - 8 * s1) ** 2), rel=1e-12)
    assert tr[0, 3] == pytest.approx(0.0, abs=1e-30) and tr[0, 4] == pytest.approx(0.0, abs=1e-30)   # s2 = a / 7 fits exactly
    # one round only: stored scale = binary16(s1), codes re-assigned against it
    codes1, scales1 = oracle.scale_optimize(w, None, bits, 1, block=B)
    assert int(scales1[0, 0]) == oracle.f64_to_f16_bits(s1)
    assert list(codes1[0]) == [15, 15, 15, 1, 1, 15, 15, 1]


def test_a_tie_between_two_codes_goes_to_the_smaller_one(oracle):
    """Eq. 11's nearest-code step leaves ties open; the stated reading is the smaller entry.  max|w| = 2 at 2 bits
    gives s = 1 exactly, so the half-integers below are true ties."""
    w = np.zeros((1, 32), dtype=np.float32)
    w[0, :6] = [-2.0, 0.5, -1.5, -0.5, 1.0, 1.5]
    codes, scales = oracle.scale_optimize(w, None, 2, 0)
    assert int(scales[0, 0]) == 0x3C00                                       # binary16 1.0
    assert codes[0, :6].tolist() == [0, 2, 0, 1, 3, 3] and not np.any(codes[0, 6:] != 2)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_zero_rounds_is_nearest_code_quantisation_at_the_absmax_scale(oracle, bits):
    """rounds = 0: d = binary16(max|w| / 2^(bits-1)) and the codes are Eq. 1's argmin for that d."""
    rng = np.random.default_rng(bits)
    W = (rng.standard_normal((6, 96)) * 0.02).astype(np.float32)
    codes, scales = oracle.scale_optimize(W, None, bits, 0)
    z = float(1 << (bits - 1))
    for n in range(6):
        for j in range(3):
            blk = W[n, 32 * j:32 * j + 32].astype(np.float64)
            d_bits = int(np.float16(np.max(np.abs(blk)) / z).view(np.uint16))      # numpy's own double -> half rounding
            assert int(scales[n, j]) == d_bits
            d = float(np.uint16(d_bits).view(np.float16))
            assert np.array_equal(codes[n, 32 * j:32 * j + 32], oracle.rtn_codes(blk, d, z, bits))


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_phi_never_increases_and_matches_the_definition(oracle, bits):
    rng = np.random.default_rng(10 + bits)
    W = (rng.standard_normal((16, 128)) * 0.02).astype(np.float32)
    F = rng.gamma(0.5, 2.0, size=W.shape).astype(np.float32)            # heavy-tailed positive sensitivities
    rounds = 6
    codes, scales, tr = oracle.scale_optimize(W, F, bits, rounds, trace=True)
    steps = tr[:, :2 * rounds + 1]
    assert np.all(steps[:, 1:] <= steps[:, :-1] * (1 + 1e-12) + 1e-300)
    # the last entry is Phi of the stored pair, recomputed here from Eq. 10
    z = 1 << (bits - 1)
    d = oracle.f16_to_f64(scales)
    for b in range(0, tr.shape[0], 7):
        n, j = divmod(b, 4)
        sl = slice(32 * j, 32 * j + 32)
        assert tr[b, -1] == pytest.approx(phi(W[n, sl], F[n, sl], codes[n, sl].astype(int) - z, d[n, j]), rel=1e-12)
    # optimising never ends worse than where it started, up to the binary16 rounding of the scale
    assert np.mean(tr[:, -1] <= tr[:, 0] * (1 + 1e-9)) > 0.97
    assert np.sum(tr[:, -1]) < np.sum(tr[:, 0])


def test_scale_update_is_the_weighted_least_squares_solution(oracle):
    """At a fixed point (many rounds) the stored scale is, up to binary16 rounding, the minimiser of Phi over s for
    the stored codes, and every stored code is the codebook entry nearest to w / d."""
    rng = np.random.default_rng(3)
    bits, z = 3, 4
    W = (rng.standard_normal((32, 64)) * 0.05).astype(np.float32)
    F = rng.uniform(0.1, 3.0, size=W.shape).astype(np.float32)
    codes, scales = oracle.scale_optimize(W, F, bits, 30)
    d = oracle.f16_to_f64(scales)
    close = 0
    for n in range(32):
        for j in range(2):
            sl = slice(32 * j, 32 * j + 32)
            w, f, q = W[n, sl].astype(np.float64), F[n, sl].astype(np.float64), codes[n, sl].astype(np.float64) - z
            assert np.array_equal(q, np.clip(np.rint(w / d[n, j]), -z, z - 1))
            om = f * np.sqrt(np.mean(w * w) + w * w)
            s_ls = np.sum(om * w * q) / np.sum(om * q * q)
            for eps in (1e-4, -1e-4):
                assert phi(w, f, q, s_ls) <= phi(w, f, q, s_ls * (1 + eps))
            close += abs(d[n, j] - s_ls) <= 2.0 ** -11 * s_ls * 1.01
    assert close >= 60          # of 64 blocks; the rest moved a code when d was rounded


def test_exhaustive_search_on_four_element_blocks(oracle):
    """2-bit codebook {-2..1}, blocks of 4: all 256 code vectors with their least-squares scale give the global
    minimum of Phi; the alternating scheme is a descent from the absmax start, so it can only end at or above it,
    and it must get there in most cases."""
    rng = np.random.default_rng(4)
    W = (rng.standard_normal((40, 4)) * 0.1).astype(np.float32)
    F = rng.uniform(0.5, 2.0, size=W.shape).astype(np.float32)
    codes, scales, tr = oracle.scale_optimize(W, F, 2, 20, block=4, trace=True)
    hits, ratios = 0, []
    for n in range(40):
        w, f = W[n].astype(np.float64), F[n].astype(np.float64)
        om = f * np.sqrt(np.mean(w * w) + w * w)
        best = np.inf
        for q in itertools.product(range(-2, 2), repeat=4):
            q = np.array(q, dtype=np.float64)
            den = np.sum(om * q * q)
            s = np.sum(om * w * q) / den if den > 0 else 0.0
            best = min(best, float(np.sum(om * (w - s * q) ** 2)))
        unrounded = tr[n, 40]                      # Phi after the last re-assignment, before the binary16 rounding
        assert unrounded >= best * (1 - 1e-12)
        assert unrounded <= tr[n, 0] * (1 + 1e-12)
        hits += unrounded <= best * (1 + 1e-9)
        ratios.append(unrounded / best)
    # a local method: it finds the global optimum on a good share of the blocks and is typically close to it
    assert hits >= 12
    assert np.median(ratios) <= 1.25


def test_invariances(oracle):
    rng = np.random.default_rng(5)
    W = (rng.standard_normal((8, 64)) * 0.02).astype(np.float32)
    F = rng.uniform(0.1, 2.0, size=W.shape).astype(np.float32)
    c0, s0 = oracle.scale_optimize(W, F, 4, 4)
    c1, s1 = oracle.scale_optimize(W, F * np.float32(8.0), 4, 4)           # a common factor on F cancels in Eq. 11
    assert np.array_equal(c0, c1) and np.array_equal(s0, s1)
    c2, s2 = oracle.scale_optimize(W * np.float32(4.0), F, 4, 4)           # powers of two pass through exactly
    assert np.array_equal(c0, c2)
    assert np.array_equal(oracle.f16_to_f64(s2), 4.0 * oracle.f16_to_f64(s0))
    c3, s3 = oracle.scale_optimize(-W, F, 3, 4)                            # the codebook is not symmetric: -8..7
    c4, s4 = oracle.scale_optimize(W, F, 3, 4)
    assert not np.array_equal(c3, (7 - c4))
    z = np.zeros((2, 32), dtype=np.float32)
    cz, sz = oracle.scale_optimize(z, None, 4, 4)
    assert np.all(cz == 8) and np.all(sz == 0)                              # all-zero block: zero scale, zero codes


def test_double_to_binary16_rounding(oracle):
    rng = np.random.default_rng(6)
    xs = np.concatenate([rng.standard_normal(4000) * 10.0 ** rng.integers(-9, 5, 4000),
                         [0.0, -0.0, 65504.0, 65519.9, 65520.0, 1e9, 2.0 ** -24, 2.0 ** -25, 2.0 ** -25 * 1.0000001,
                          1.5 * 2.0 ** -24, 2.5 * 2.0 ** -24, 1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11, 2.0 ** -14 - 2.0 ** -25]])
    with np.errstate(over="ignore"):
        want = xs.astype(np.float16).view(np.uint16)
    got = np.array([oracle.f64_to_f16_bits(x) for x in xs], dtype=np.uint16)
    assert np.array_equal(got, want)
