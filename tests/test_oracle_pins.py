"""Pins of the CPU oracle against what the paper and the mathematics fix.

None of these compares the oracle with itself or with the GPU path: they use
hand-worked bitstreams, numpy's own half-precision conversion, exact rational
arithmetic on tiny cases, integer matmul, the Eq. 1 argmin round trip and the
footprint figures printed in Table 1.
"""
import os
from fractions import Fraction

import numpy as np
import pytest

import aq_workloads as wl

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# ---------------------------------------------------------------- bitstreams
def _bitstream_examples():
    out = []
    for line in open(os.path.join(GOLDEN, "bitstream_examples.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        b, codes, hexbytes = [t.strip() for t in line.split(";")]
        out.append((int(b), [int(c) for c in codes.split()], bytes.fromhex(hexbytes.replace(" ", ""))))
    return out


@pytest.mark.parametrize("bits,codes,raw", _bitstream_examples())
def test_unpack_hand_worked_bitstreams(oracle, bits, codes, raw):
    """Worked examples (tests/golden/bitstream_examples.txt): the first bytes of a
    block decode to the listed codes and the listed codes encode to those bytes."""
    blk = np.zeros(4 * bits, dtype=np.uint8)
    blk[:len(raw)] = np.frombuffer(raw, dtype=np.uint8)
    q = oracle.unpack(blk.reshape(1, 1, -1), 1, 32, bits)
    assert q[0, :len(codes)].tolist() == codes
    full = np.zeros((1, 32), dtype=np.uint8)
    full[0, :len(codes)] = codes
    s = oracle.pack(full, bits).ravel()
    assert bytes(s[:len(raw)]) == raw


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_unpack_every_value_at_every_position(oracle, bits):
    """One code set, all others zero: exactly bits [i*b, i*b+b) of the block's
    little-endian number are set (checked with Python big integers)."""
    for i in range(32):
        for v in range(1, 1 << bits):
            q = np.zeros((1, 32), dtype=np.uint8)
            q[0, i] = v
            s = oracle.pack(q, bits).ravel()
            assert len(s) == 4 * bits
            assert int.from_bytes(bytes(s), "little") == v << (i * bits)
            assert np.array_equal(oracle.unpack(s, 1, 32, bits), q)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_unpack_blocks_never_share_a_byte(oracle, bits):
    """Random bytes: block j of row n only depends on its own 4b bytes, and the codes
    are the b-bit digits of the block's little-endian integer."""
    rng = np.random.default_rng(7)
    N, K = 3, 96
    s = rng.integers(0, 256, size=(N, K // 32, 4 * bits), dtype=np.uint8)
    q = oracle.unpack(s, N, K, bits)
    for n in range(N):
        for j in range(K // 32):
            big = int.from_bytes(bytes(s[n, j]), "little")
            want = [(big >> (i * bits)) & ((1 << bits) - 1) for i in range(32)]
            assert q[n, 32 * j:32 * j + 32].tolist() == want


# ---------------------------------------------------------------- conversions
def test_f16_conversion_all_patterns(oracle):
    """All 65536 binary16 patterns against numpy's float16 -> float64 cast."""
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    got = oracle.f16_to_f64(bits)
    want = bits.view(np.float16).astype(np.float64)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))


def test_bf16_conversion_all_patterns(oracle):
    """All 65536 bfloat16 patterns against 'upper half of a float32'."""
    bits = np.arange(65536, dtype=np.uint32)
    want = (bits << 16).astype(np.uint32).view(np.float32).astype(np.float64)
    got = oracle.bf16_to_f64(bits.astype(np.uint16))
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])


# ---------------------------------------------------------------- Eq. 1
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_dequant_grid_values(oracle, bits):
    """With d = 1 the dequantised values are the integers q - 2^(b-1): the grid is
    {-2..1}, {-4..3}, {-8..7}; with d = 0.5 they halve (Eq. 1, left part)."""
    q = (np.arange(32, dtype=np.uint8) % (1 << bits)).reshape(1, 32)
    s = oracle.pack(q, bits)
    one = np.array([[0x3C00]], dtype=np.uint16)    # 1.0
    half = np.array([[0x3800]], dtype=np.uint16)   # 0.5
    W1 = oracle.dequant(s, one, 1, 32, bits)
    assert W1.min() == -(1 << (bits - 1)) and W1.max() == (1 << (bits - 1)) - 1
    assert np.array_equal(W1[0], q[0].astype(np.float64) - (1 << (bits - 1)))
    assert np.array_equal(oracle.dequant(s, half, 1, 32, bits), W1 / 2)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_grid_round_trip_through_argmin(oracle, bits):
    """Codes on the grid round-trip exactly: for d > 0 the Eq. 1 argmin applied to
    w_hat = d (q - z) returns q (the error is zero only at the true code)."""
    N, K = 16, 256
    codes, scales = wl.draw_matrix(N, K, bits, 11, bits)
    W = oracle.dequant(codes, scales, N, K, bits)
    q = oracle.unpack(codes, N, K, bits)
    d = oracle.f16_to_f64(scales)
    z = float(1 << (bits - 1))
    checked = 0
    for n in range(N):
        for j in range(K // 32):
            if d[n, j] == 0.0:
                continue
            got = oracle.rtn_codes(W[n, 32 * j:32 * j + 32], d[n, j], z, bits)
            assert np.array_equal(got, q[n, 32 * j:32 * j + 32])
            checked += 1
    assert checked > 100


def test_argmin_rounds_to_nearest_level(oracle):
    """Off-grid values go to the nearest level and saturate at the ends (Eq. 1, right part)."""
    w = np.array([-100.0, -1.26, -0.74, 0.24, 0.26, 0.76, 100.0])
    got = oracle.rtn_codes(w, 0.5, 2.0, 2)      # levels -1, -0.5, 0, 0.5
    assert got.tolist() == [0, 0, 1, 2, 3, 3, 3]
    # Eq. 1's argmin leaves a tie open; the oracle's stated reading is that the first (lowest) minimiser wins.
    # The midpoints of a power-of-two grid are exact in binary, so these are true ties.
    mid = np.array([-0.75, -0.25, 0.25])
    assert oracle.rtn_codes(mid, 0.5, 2.0, 2).tolist() == [0, 1, 2]


# ---------------------------------------------------------------- brute force
def _frac_f16(h: int) -> Fraction:
    s, e, m = (h >> 15) & 1, (h >> 10) & 31, h & 1023
    assert e != 31
    v = Fraction(m, 1 << 24) if e == 0 else Fraction(1024 + m, 1024) * Fraction(2) ** (e - 15)
    return -v if s else v


def _frac_bf16(h: int) -> Fraction:
    s, e, m = (h >> 15) & 1, (h >> 7) & 255, h & 127
    assert e != 255
    v = Fraction(m, 128) * Fraction(2) ** (-126) if e == 0 else Fraction(128 + m, 128) * Fraction(2) ** (e - 127)
    return -v if s else v


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("M,dtype", [(1, "f16"), (3, "bf16")])
def test_brute_force_exact_rationals_8x32(oracle, bits, M, dtype):
    """N = 8, K = 32 (one block per row): the whole path against exact rational
    arithmetic written from the format definition with Python integers."""
    N, K = 8, 32
    codes, scales = wl.draw_matrix(N, K, bits, 21, bits, M)
    X = wl.draw_activations(M, K, dtype, 21, bits, M)
    Y = oracle.qmatmul(codes, scales, N, K, bits, X, dtype)
    conv = _frac_f16 if dtype == "f16" else _frac_bf16
    for n in range(N):
        big = int.from_bytes(bytes(codes[n, 0]), "little")
        d = _frac_f16(int(scales[n, 0]))
        w = [d * (((big >> (i * bits)) & ((1 << bits) - 1)) - (1 << (bits - 1))) for i in range(K)]
        for m in range(M):
            exact = sum(conv(int(X[m, k])) * w[k] for k in range(K))
            got = Y[m, n]
            if exact == 0:
                assert got == 0.0
            else:
                assert abs(Fraction(got) - exact) <= abs(exact) * Fraction(1, 10 ** 13) + Fraction(1, 10 ** 18)


def test_integer_matmul_special_case(oracle):
    """All scales 1 and b = 4: the path is the integer matrix product x (Q - 8)^T,
    compared exactly with numpy's int64 matmul."""
    N, K, M = 24, 128, 5
    codes = wl.draw_codes(N, K, 4, 31)
    ones = np.full((N, K // 32), 0x3C00, dtype=np.uint16)
    X = wl.draw_int_activations(M, K, "f16", 31)
    xi = X.view(np.float16).astype(np.int64)
    q = codes.reshape(N, -1)
    Q = np.empty((N, K), dtype=np.int64)
    Q[:, 0::2] = q & 15
    Q[:, 1::2] = q >> 4
    want = xi @ (Q - 8).T
    got = oracle.qmatmul(codes, ones, N, K, 4, X, "f16")
    assert np.array_equal(got, want.astype(np.float64))


def test_matmul_against_numpy(oracle):
    rng = np.random.default_rng(3)
    X = rng.standard_normal((7, 160))
    W = rng.standard_normal((13, 160))
    got = oracle.matmul_nt(X, W)
    assert got.shape == (7, 13)          # Y is [M, N]: a transposed operand would fail here
    np.testing.assert_allclose(got, X @ W.T, rtol=1e-12, atol=1e-12)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_path_invariants(oracle, bits):
    """Doubling every scale doubles Y exactly; zero activations give zero; moving whole
    K-blocks of W and x together leaves Y unchanged up to fp64 rounding."""
    N, K, M = 12, 192, 2
    codes, scales = wl.draw_matrix(N, K, bits, 41, bits)
    X = wl.draw_activations(M, K, "f16", 41, bits)
    Y = oracle.qmatmul(codes, scales, N, K, bits, X, "f16")
    d2 = (scales.view(np.float16).astype(np.float32) * 2).astype(np.float16).view(np.uint16)
    normal = (scales >> 10) & 31 > 0            # doubling a subnormal is exact too, but keep it simple
    assert normal.mean() > 0.9
    Y2 = oracle.qmatmul(codes, d2, N, K, bits, X, "f16")
    assert np.array_equal(Y2, 2 * Y)
    assert not np.any(oracle.qmatmul(codes, scales, N, K, bits, np.zeros_like(X), "f16"))
    perm = np.array([3, 0, 5, 1, 4, 2])
    Xp = X.reshape(M, 6, 32)[:, perm].reshape(M, K)
    Yp = oracle.qmatmul(codes[:, perm], scales[:, perm], N, K, bits, Xp, "f16")
    np.testing.assert_allclose(Yp, Y, rtol=1e-12, atol=1e-15)


def test_one_hot_activation_reads_a_weight(oracle):
    """x = e_k gives y[n] = w_hat[n, k] exactly."""
    N, K = 9, 64
    codes, scales = wl.draw_matrix(N, K, 3, 51)
    W = oracle.dequant(codes, scales, N, K, 3)
    for k in (0, 2, 31, 32, 63):
        x = np.zeros((1, K), dtype=np.uint16)
        x[0, k] = 0x3C00
        assert np.array_equal(oracle.qmatmul(codes, scales, N, K, 3, x, "f16")[0], W[:, k])


# ---------------------------------------------------------------- accounting
def test_bytes_per_block_and_bits_per_weight(oracle):
    """Per block 4b code bytes + a 2-byte scale: 10 / 14 / 18 bytes, i.e. 2.5 / 3.5 / 4.5
    stored bits per weight; a 3-bit block has 12 code bytes."""
    for b, per_block, bpw in ((2, 10, Fraction(5, 2)), (3, 14, Fraction(7, 2)), (4, 18, Fraction(9, 2))):
        assert oracle.stored_bytes(1, 32, b) == per_block
        assert oracle.bits_per_weight(b) == bpw
        assert Fraction(oracle.stored_bytes(4096, 4096, b) * 8, 4096 * 4096) == bpw
    assert wl.draw_codes(1, 32, 3, 0).shape == (1, 1, 12)
    assert oracle.stored_bytes(4096, 4096, 2) == 5_242_880
    assert oracle.stored_bytes(4096, 4096, 3) == 7_340_032
    assert oracle.stored_bytes(4096, 4096, 4) == 9_437_184
    assert oracle.stored_bytes(11008, 4096, 4) == 25_362_432
    assert oracle.stored_bytes(4096, 11008, 2) == 14_090_240


def _table1():
    rows, ratios = [], []
    for line in open(os.path.join(GOLDEN, "table1_footprint.txt")):
        t = line.split()
        if not t or t[0].startswith("#"):
            continue
        if t[0] in ("consistent", "inconsistent"):
            rows.append((t[0], t[1], float(t[2]), t[3], float(t[4]), float(t[5]), float(t[6])))
        elif t[0] == "ratio":
            ratios.append((float(t[1]), float(t[2]), float(t[3])))
    return rows, ratios


def test_footprint_arithmetic_reproduces_table1(oracle):
    """Mem = fp16 size * (VLA bits per weight) / 16 reproduces the printed memory of
    Table 1's self-consistent rows to the printed digit, and the printed ratios
    (14.3 -> 2.7 GB = 5.3x; 6.7 -> 2.7 GB = 2.5x) follow from the printed sizes."""
    rows, ratios = _table1()
    assert sum(r[0] == "consistent" for r in rows) >= 6
    for kind, _model, fp16_gb, _method, _bb, vla_bpw, mem in rows:
        got = round(oracle.footprint_gb(fp16_gb, vla_bpw), 1)
        if kind == "consistent":
            assert got == mem
        else:
            assert got != mem      # documented: the table does not close on these rows
    for fp16_gb, q_gb, ratio in ratios:
        assert round(fp16_gb / q_gb, 1) == ratio
    # the headline 2.5-bit row: 16 / 3.0 stored bits = 5.33x, printed as 5.3x
    assert round(16 / 3.0, 1) == 5.3


def test_synthetic_stream_accounting(oracle):
    """Weight and byte counts of the backbone-shaped streams."""
    llama = wl.backbone_stream("llama2-7b", "floor")
    assert len(llama) == 224
    assert sum(m.weights for m in llama) == 6_476_005_376
    assert sum(oracle.stored_bytes(m.N, m.K, m.bits) for m in llama) == 2_023_751_680
    assert wl.stored_bits_per_weight(llama) == 2.5
    mixed = wl.backbone_stream("llama2-7b", "mixed")
    assert {m.bits for m in mixed} == {2, 3, 4}
    tot = sum(m.weights for m in mixed)
    code_bits = sum(m.weights * m.bits for m in mixed) / tot
    assert 2.49 < code_bits <= 2.5
    stored = sum(oracle.stored_bytes(m.N, m.K, m.bits) for m in mixed)
    assert stored <= 2_428_502_016 and stored > 2_420_000_000
    gemma = wl.backbone_stream("gemma-2b", "b3")
    assert len(gemma) == 126
    assert sum(m.weights for m in gemma) == 1_981_808_640
    assert sum(oracle.stored_bytes(m.N, m.K, m.bits) for m in gemma) == 867_041_280


def test_workload_generators_are_seeded():
    a = wl.draw_codes(8, 64, 3, 1, 2)
    assert np.array_equal(a, wl.draw_codes(8, 64, 3, 1, 2))
    assert not np.array_equal(a, wl.draw_codes(8, 64, 3, 1, 3))
    s = wl.draw_scales(64, 4096, 5).view(np.float16).astype(np.float64)
    assert s.min() >= 0 and abs(s.mean() - 0.02 * np.sqrt(2 / np.pi)) < 5e-4
    x = wl.draw_activations(300, 64, "bf16", 9, image_rows=256, image_gain=3.0)
    xf = (x.astype(np.uint32) << 16).view(np.float32)
    assert abs(xf[:256].std() - 3.0) < 0.1 and abs(xf[256:].std() - 1.0) < 0.1
    assert wl.seeded_allocation([(4, 4)] * 10, 2.5) == wl.seeded_allocation([(4, 4)] * 10, 2.5)


# ---------------------------------------------------------------- the acceptance measure and the row sampler
def test_rel_l2_on_hand_computed_pairs(oracle):
    """||Y - ref|| / ||ref|| on pairs worked by hand (Pythagorean triples, so every norm is an integer).
    ref = (3, 4), Y = ref + (5, 12): numerator 13, denominator 5.  A dropped square root gives 169 / 25
    or 13 / 25, the norms swapped 5 / 13, the norm of Y in the denominator 13 / sqrt(8^2 + 16^2)."""
    ref = np.array([3.0, 4.0])
    assert oracle.rel_l2(ref + np.array([5.0, 12.0]), ref) == pytest.approx(13.0 / 5.0, rel=1e-15)
    # not symmetric in its arguments: the reference's norm divides
    assert oracle.rel_l2(ref, ref + np.array([5.0, 12.0])) == pytest.approx(13.0 / np.sqrt(8.0 ** 2 + 16.0 ** 2), rel=1e-15)
    # a 2-D pair, taken over the whole array: ref norm sqrt(1+4+4+16) = 5, difference (0, 0, 0, 0.5)
    ref2 = np.array([[1.0, 2.0], [2.0, 4.0]])
    y2 = ref2.copy()
    y2[1, 1] += 0.5
    assert oracle.rel_l2(y2, ref2) == pytest.approx(0.1, rel=1e-15)
    assert oracle.rel_l2(ref2, ref2) == 0.0
    # scale invariance and the 1e-3 bar itself: a uniform relative perturbation of 1e-3 measures 1e-3
    big = np.arange(1.0, 101.0) * 1e6
    assert oracle.rel_l2(big * (1 + 1e-3), big) == pytest.approx(1e-3, rel=1e-9)
    # fp32 inputs are widened, not compared in fp32 (2^-30 survives next to 1)
    a = np.array([1.0, 1.0], dtype=np.float32)
    b = np.array([1.0, 1.0 + 2.0 ** -30], dtype=np.float64)
    assert oracle.rel_l2(a, b) == pytest.approx(2.0 ** -30 / np.sqrt(1 + (1 + 2.0 ** -30) ** 2), rel=1e-12)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_qmatmul_rows_equals_the_matching_columns_of_qmatmul(oracle, bits):
    """qmatmul_rows(rows) = the columns `rows` of the full product, in the order asked for, duplicates
    included, on a ragged matrix (N = 37, K = 96) and for a single row; and against exact rationals for one
    sampled row, so the sampler is pinned to the definition and not only to the function it wraps."""
    N, K, M = 37, 96, 3
    codes = wl.draw_codes(N, K, bits, 71, bits)
    scales = wl.draw_scales(N, K, 72)
    X = wl.draw_activations(M, K, "bf16", 73)
    full = oracle.qmatmul(codes, scales, N, K, bits, X, "bf16")
    rows = [36, 0, 5, 5, 17]
    got = oracle.qmatmul_rows(codes, scales, rows, K, bits, X, "bf16")
    assert got.shape == (M, len(rows))
    assert np.array_equal(got, full[:, rows])
    one = oracle.qmatmul_rows(codes, scales, [9], K, bits, X, "bf16")
    assert np.array_equal(one[:, 0], full[:, 9])
    # exact rationals for row 17, activation row 1
    q = oracle.unpack(codes, N, K, bits)
    d = scales.reshape(N, K // 32).view(np.float16)
    xf = (X[1].astype(np.uint32) << 16).view(np.float32)
    acc = Fraction(0)
    for k in range(K):
        acc += Fraction(float(xf[k])) * Fraction(float(d[17, k // 32])) * (int(q[17, k]) - (1 << (bits - 1)))
    assert abs(got[1, 4] - float(acc)) <= 1e-13 * max(1.0, abs(float(acc)))
