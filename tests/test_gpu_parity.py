"""Parity of the HIP path (through the C ABI) against the CPU oracle, element by element,
on the same seeded inputs.  Bars: codes and dequantised weights bit-exact; outputs
relative L2 <= 1e-3 against the fp64 oracle (fp32 accumulation), and exact on inputs
where every summation order gives the same fp32 bits."""
import numpy as np
import pytest

import aq_workloads as wl

pytestmark = pytest.mark.gpu

REL_L2_BAR = 1e-3        # the acceptance bar
REL_L2_EXPECTED = 2e-4   # fp32-accumulation error model: anything above this hints at a bug


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2605_24011_amd as aq
    assert torch.cuda.is_available(), "these tests need the GPU"
    aq.lib()
    return torch, aq


def _dev(torch, a, kind=None):
    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16) if a.dtype == np.uint16 else np.ascontiguousarray(a))
    t = t.cuda()
    if kind == "f16":
        t = t.view(torch.float16)
    elif kind == "bf16":
        t = t.view(torch.bfloat16)
    return t


def _pack(torch, aq, codes, scales, N, K, bits):
    return aq.aq_pack_weights(_dev(torch, codes), _dev(torch, scales), N, K, bits)


SHAPES = [  # several tiles, ragged N (not a multiple of 16 / 128), K not a multiple of 256
    (8, 32), (16, 256), (17, 96), (200, 1056), (128, 512), (300, 4096), (131, 2048),
]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", SHAPES)
def test_codes_and_dequant_bit_exact(gpu, oracle, bits, N, K):
    torch, aq = gpu
    codes, scales = wl.draw_matrix(N, K, bits, 1, N, K)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    q = aq.aq_unpack_codes(packed, N, K, bits).cpu().numpy()
    assert np.array_equal(q, oracle.unpack(codes, N, K, bits))
    W = aq.aq_dequant_f32(packed, N, K, bits).cpu().numpy()
    want = oracle.dequant(codes, scales, N, K, bits)
    assert np.array_equal(W.astype(np.float64), want)     # -0.0 == 0.0 compares equal


def test_subnormal_and_zero_scales_are_exact(gpu, oracle):
    torch, aq = gpu
    N, K, bits = 32, 256, 4
    codes = wl.draw_codes(N, K, bits, 2)
    scales = wl.draw_scales(N, K, 2)
    scales[0, :] = 0x0000                  # zero scale: all-zero block
    scales[1, :] = 0x0001                  # smallest subnormal
    scales[2, :] = 0x03FF                  # largest subnormal
    scales[3, :] = 0x0400                  # smallest normal
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    W = aq.aq_dequant_f32(packed, N, K, bits).cpu().numpy()
    assert np.array_equal(W.astype(np.float64), oracle.dequant(codes, scales, N, K, bits))
    x = wl.draw_activations(1, K, "f16", 2)
    y = aq.aq_qgemv(packed, N, K, bits, _dev(torch, x[0], "f16")).cpu().numpy()
    ref = oracle.qmatmul(codes, scales, N, K, bits, x, "f16")[0]
    assert oracle.rel_l2(y, ref) <= REL_L2_EXPECTED
    assert np.all(y[0] == 0.0)


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", SHAPES + [(4096, 4096), (256, 2048), (1000, 11008)])
def test_qgemv_matches_oracle(gpu, oracle, bits, N, K, dtype):
    torch, aq = gpu
    codes, scales = wl.draw_matrix(N, K, bits, 3, N, K)
    x = wl.draw_activations(1, K, dtype, 3, N, K)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    y = aq.aq_qgemv(packed, N, K, bits, _dev(torch, x[0], dtype)).cpu().numpy()
    ref = oracle.qmatmul(codes, scales, N, K, bits, x, dtype)[0]
    err = oracle.rel_l2(y, ref)
    assert err <= REL_L2_BAR
    assert err <= REL_L2_EXPECTED, err


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_qgemv_exact_on_integer_inputs(gpu, oracle, bits, dtype):
    """Integer activations in [-4, 4] and power-of-two scales: all partial sums are exact in
    fp32 whatever the order, so the GPU must equal the oracle bit for bit."""
    torch, aq = gpu
    N, K = 300, 11008
    codes = wl.draw_codes(N, K, bits, 4, bits)
    scales = wl.draw_pow2_scales(N, K, 4, bits)
    x = wl.draw_int_activations(1, K, dtype, 4, bits)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    y = aq.aq_qgemv(packed, N, K, bits, _dev(torch, x[0], dtype)).cpu().numpy()
    ref = oracle.qmatmul(codes, scales, N, K, bits, x, dtype)[0]
    assert np.array_equal(y.astype(np.float64), ref)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_qgemv_one_hot_reads_dequantised_weights(gpu, oracle, bits):
    """x = e_k: y[n] = w_hat[n, k] exactly, for k at every position class of a block."""
    torch, aq = gpu
    N, K = 48, 512
    codes, scales = wl.draw_matrix(N, K, bits, 5, bits)
    W = oracle.dequant(codes, scales, N, K, bits)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    for k in list(range(0, 64)) + [255, 256, 300, 511]:
        x = np.zeros(K, dtype=np.uint16)
        x[k] = 0x3C00
        y = aq.aq_qgemv(packed, N, K, bits, _dev(torch, x, "f16")).cpu().numpy()
        assert np.array_equal(y.astype(np.float64), W[:, k]), k


def test_qgemv_zero_activations_and_scaling(gpu, oracle):
    torch, aq = gpu
    N, K, bits = 64, 1024, 3
    codes, scales = wl.draw_matrix(N, K, bits, 6)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    y0 = aq.aq_qgemv(packed, N, K, bits, torch.zeros(K, dtype=torch.float16, device="cuda")).cpu().numpy()
    assert not y0.any()
    x = wl.draw_activations(1, K, "bf16", 6)
    # huge and tiny bf16 activations (outside fp16's range) keep the accuracy
    for shift in (-60, 0, 40):
        xs = (x[0].astype(np.int32) + (shift << 7)).astype(np.uint16)      # multiply by 2^shift
        y = aq.aq_qgemv(packed, N, K, bits, _dev(torch, xs, "bf16")).cpu().numpy()
        ref = oracle.qmatmul(codes, scales, N, K, bits, xs[None], "bf16")[0]
        assert oracle.rel_l2(y, ref) <= REL_L2_EXPECTED


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_qgemv_wide_dynamic_range_inside_one_vector(gpu, oracle, bits, dtype):
    """Activations whose magnitude differs by many binades from block to block of ONE vector (bf16: 2^-60 .. 2^40
    over the blocks, f16: 2^-12 .. 2^12) and by 2^-12 inside blocks: the staging keeps one exponent per block of
    32, so every block keeps 16 bits below its own largest element.  Lone call and batched launch."""
    torch, aq = gpu
    N, K = 272, 4096
    codes, scales = wl.draw_matrix(N, K, bits, 17, bits)
    rng = np.random.default_rng(171 + bits)
    x = rng.standard_normal(K).astype(np.float32)
    span = 100 if dtype == "bf16" else 24
    block_exp = rng.integers(0, span + 1, size=K // 32) - (60 if dtype == "bf16" else 12)
    x *= np.exp2(np.repeat(block_exp, 32)).astype(np.float32)
    small = rng.random(K) < 0.25                    # a quarter of the elements sit 2^-12 below their block
    x[small] *= np.float32(2.0 ** -12)
    xb = (wl.f32_to_bf16_bits(x[None]) if dtype == "bf16" else wl.f32_to_f16_bits(x[None]))
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    ref = oracle.qmatmul(codes, scales, N, K, bits, xb, dtype)[0]
    xd = _dev(torch, xb[0], dtype)
    y = aq.aq_qgemv(packed, N, K, bits, xd).cpu().numpy()
    assert np.isfinite(y).all()
    assert oracle.rel_l2(y, ref) <= REL_L2_EXPECTED
    yb = torch.empty(N, dtype=torch.float32, device="cuda")
    aq.GemvBatch([(packed, N, K, bits, xd, yb)]).run()
    assert oracle.rel_l2(yb.cpu().numpy(), ref) <= REL_L2_EXPECTED


def test_qgemv_batch_matches_single_calls(gpu, oracle):
    """A mixed-bit stream in one launch gives what the per-matrix calls give, and the oracle's."""
    torch, aq = gpu
    specs = [(256, 512, 2, "f16"), (130, 2048, 3, "bf16"), (512, 1056, 4, "f16"), (16, 32, 2, "f16"),
             (384, 11008, 3, "f16"), (1000, 4096, 4, "bf16")]
    items, refs, singles = [], [], []
    for i, (N, K, bits, dt) in enumerate(specs):
        codes, scales = wl.draw_matrix(N, K, bits, 7, i)
        x = wl.draw_activations(1, K, dt, 7, i)
        packed = _pack(torch, aq, codes, scales, N, K, bits)
        xd = _dev(torch, x[0], dt)
        y = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, xd, y))
        refs.append(oracle.qmatmul(codes, scales, N, K, bits, x, dt)[0])
        singles.append(aq.aq_qgemv(packed, N, K, bits, xd).cpu().numpy())
    batch = aq.GemvBatch(items)
    batch.run()
    batch.run()          # a plan can be replayed
    torch.cuda.synchronize()
    for (packed, N, K, bits, xd, y), ref, single in zip(items, refs, singles):
        got = y.cpu().numpy()
        assert oracle.rel_l2(got, ref) <= REL_L2_EXPECTED
        assert oracle.rel_l2(got, single) <= 1e-5


GEMM_CASES = [  # (N, K, M): M spans 1..3 m-tiles per wavefront, uneven tile deals and two workgroups along m
    (64, 256, 16), (17, 96, 1), (200, 1056, 7), (256, 2048, 64), (512, 512, 300), (130, 4096, 81),
    (128, 512, 129), (144, 288, 257), (96, 544, 385), (260, 256, 800),
]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K,M", GEMM_CASES)
def test_qgemm_matches_oracle(gpu, oracle, bits, N, K, M, dtype):
    torch, aq = gpu
    codes, scales = wl.draw_matrix(N, K, bits, 8, N, K)
    X = wl.draw_activations(M, K, dtype, 8, N, K, image_rows=min(256, M) if M >= 256 else 0, image_gain=3.0)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, dtype)).cpu().numpy()
    ref = oracle.qmatmul(codes, scales, N, K, bits, X, dtype)
    err = oracle.rel_l2(Y, ref)
    assert err <= REL_L2_BAR
    assert err <= REL_L2_EXPECTED, err
    # per-row too: a wrong row hides in the global norm when image rows are 3x larger
    for m in range(M):
        assert oracle.rel_l2(Y[m], ref[m]) <= REL_L2_BAR


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_qgemm_exact_on_integer_inputs_and_one_hot(gpu, oracle, bits):
    torch, aq = gpu
    N, K, M = 96, 1056, 40
    codes = wl.draw_codes(N, K, bits, 9, bits)
    scales = wl.draw_pow2_scales(N, K, 9, bits)
    X = wl.draw_int_activations(M, K, "bf16", 9, bits)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, "bf16")).cpu().numpy()
    assert np.array_equal(Y.astype(np.float64), oracle.qmatmul(codes, scales, N, K, bits, X, "bf16"))
    # one-hot rows read dequantised weights through the public entry point, with random scales
    codes, scales = wl.draw_matrix(N, K, bits, 10, bits)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    ks = [0, 1, 31, 32, 33, 255, 256, 700, K - 1]
    X = np.zeros((len(ks), K), dtype=np.uint16)
    for m, k in enumerate(ks):
        X[m, k] = 0x3F80          # bf16 1.0
    Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, "bf16")).cpu().numpy()
    W = oracle.dequant(codes, scales, N, K, bits)
    assert np.array_equal(Y.astype(np.float64), W[:, ks].T)


def test_qgemm_row_equals_qgemv_and_strides(gpu, oracle):
    torch, aq = gpu
    N, K, M, bits = 192, 2048, 5, 3
    codes, scales = wl.draw_matrix(N, K, bits, 11)
    X = wl.draw_activations(M, K, "bf16", 11)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    Xd = _dev(torch, X, "bf16")
    # padded leading dimensions on both sides
    Xp = torch.zeros((M, K + 64), dtype=torch.bfloat16, device="cuda")
    Xp[:, :K] = Xd
    Yp = torch.full((M, N + 8), -7.0, dtype=torch.float32, device="cuda")
    aq.aq_qgemm(packed, N, K, bits, Xp[:, :K], Y=Yp[:, :N])
    Y = Yp.cpu().numpy()
    assert np.all(Y[:, N:] == -7.0)
    ref = oracle.qmatmul(codes, scales, N, K, bits, X, "bf16")
    assert oracle.rel_l2(Y[:, :N], ref) <= REL_L2_EXPECTED
    for m in range(M):
        yv = aq.aq_qgemv(packed, N, K, bits, Xd[m].contiguous()).cpu().numpy()
        assert oracle.rel_l2(yv, Y[m, :N]) <= 1e-5


def test_errors_raise_through_the_binding(gpu):
    torch, aq = gpu
    x = torch.zeros(64, dtype=torch.float32, device="cuda")
    p = torch.zeros(4096, dtype=torch.uint8, device="cuda")
    with pytest.raises(aq.AqError):
        aq.aq_qgemv(p, 16, 64, 4, x)                       # fp32 activations
    with pytest.raises(aq.AqError):
        aq.aq_qgemv(p, 16, 64, 5, x.half())                # bad bit-width
    with pytest.raises(aq.AqError):
        aq.aq_qgemv(p, 16, 64, 4, x.half()[1:])            # misaligned pointer


# ---------------------------------------------------------------------------------------------
# full-size matrices in the launch configuration bench.py times (one batched launch over the
# seven LLaMA-2-7B-shaped matrices of a layer, mixed bit-widths), checked on sampled outputs
# ---------------------------------------------------------------------------------------------
def test_full_size_layer_batched_sampled_rows(gpu, oracle):
    torch, aq = gpu
    rng = np.random.default_rng(123)
    bits_of = {"q": 2, "k": 3, "v": 4, "o": 2, "gate": 3, "up": 2, "down": 4}
    items, host = [], []
    for i, (name, N, K) in enumerate(wl.LLAMA2_7B_LAYER):
        b = bits_of[name]
        codes, scales = wl.draw_matrix(N, K, b, 12, i)
        x = wl.draw_activations(1, K, "f16", 12, i)
        packed = _pack(torch, aq, codes, scales, N, K, b)
        y = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, b, _dev(torch, x[0], "f16"), y))
        host.append((codes, scales, x, N, K, b))
    aq.GemvBatch(items).run()
    torch.cuda.synchronize()
    for (packed, N, K, b, xd, y), (codes, scales, x, _, _, _) in zip(items, host):
        got = y.cpu().numpy()
        assert np.isfinite(got).all()
        rows = np.unique(np.concatenate([[0, 15, 16, 127, 128, N - 1], rng.integers(0, N, 250)]))
        ref = oracle.qmatmul_rows(codes, scales, rows, K, b, x, "f16")[0]
        assert oracle.rel_l2(got[rows], ref) <= REL_L2_EXPECTED
        # unpacked codes of the sampled rows are bit-exact at full size too
        q = aq.aq_unpack_codes(packed, N, K, b)[torch.from_numpy(rows).cuda()].cpu().numpy()
        assert np.array_equal(q, oracle.unpack(codes[rows], len(rows), K, b))


@pytest.mark.parametrize("name,N,K", [("q", 2048, 2048), ("k", 256, 2048), ("gate", 16384, 2048), ("down", 2048, 16384)])
def test_gemma_shapes_decode_and_prefill_sampled(gpu, oracle, name, N, K):
    """Gemma-2B-shaped matrices at 3 bits, bf16 activations, M in {1, 16, 64}; sampled columns."""
    torch, aq = gpu
    rng = np.random.default_rng(7)
    codes, scales = wl.draw_matrix(N, K, 3, 13, N, K)
    packed = _pack(torch, aq, codes, scales, N, K, 3)
    rows = np.unique(np.concatenate([[0, N - 1], rng.integers(0, N, 120)]))
    for M in (1, 16, 64):
        X = wl.draw_activations(M, K, "bf16", 13, N, K, M)
        ref = oracle.qmatmul_rows(codes, scales, rows, K, 3, X, "bf16")
        Y = aq.aq_qgemm(packed, N, K, 3, _dev(torch, X, "bf16")).cpu().numpy()
        assert oracle.rel_l2(Y[:, rows], ref) <= REL_L2_EXPECTED
        if M == 1:
            y = aq.aq_qgemv(packed, N, K, 3, _dev(torch, X[0], "bf16")).cpu().numpy()
            assert oracle.rel_l2(y[rows], ref[0]) <= REL_L2_EXPECTED


def test_full_size_prefill_m300_sampled(gpu, oracle):
    """One 4096 x 4096 matrix per bit-width at M = 300 (256 image rows x3, 44 text rows), sampled columns."""
    torch, aq = gpu
    rng = np.random.default_rng(9)
    N = K = 4096
    X = wl.draw_activations(300, K, "bf16", 14, image_rows=256, image_gain=3.0)
    Xd = _dev(torch, X, "bf16")
    for bits in (2, 3, 4):
        codes, scales = wl.draw_matrix(N, K, bits, 14, bits)
        packed = _pack(torch, aq, codes, scales, N, K, bits)
        Y = aq.aq_qgemm(packed, N, K, bits, Xd).cpu().numpy()
        rows = np.unique(np.concatenate([[0, 63, 64, N - 1], rng.integers(0, N, 60)]))
        ref = oracle.qmatmul_rows(codes, scales, rows, K, bits, X, "bf16")
        assert oracle.rel_l2(Y[:, rows], ref) <= REL_L2_EXPECTED
        for m in (0, 255, 256, 299):
            assert oracle.rel_l2(Y[m, rows], ref[m]) <= REL_L2_EXPECTED


def test_qgemm_batch_matches_single_calls(gpu, oracle):
    """Mixed-bit list of prefill products in one launch == the per-matrix calls == the oracle."""
    torch, aq = gpu
    specs = [(256, 512, 2, 37), (130, 2048, 3, 300), (512, 1056, 4, 64), (16, 32, 2, 1), (1000, 4096, 4, 200)]
    items, refs = [], []
    for i, (N, K, bits, M) in enumerate(specs):
        codes, scales = wl.draw_matrix(N, K, bits, 15, i)
        X = wl.draw_activations(M, K, "bf16", 15, i)
        packed = _pack(torch, aq, codes, scales, N, K, bits)
        Xd = _dev(torch, X, "bf16")
        Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, Xd, Y))
        refs.append(oracle.qmatmul(codes, scales, N, K, bits, X, "bf16"))
    batch = aq.GemmBatch(items)
    batch.run()
    batch.run()
    torch.cuda.synchronize()
    for (packed, N, K, bits, Xd, Y), ref in zip(items, refs):
        got = Y.cpu().numpy()
        assert np.isfinite(got).all()
        assert oracle.rel_l2(got, ref) <= REL_L2_EXPECTED
        single = aq.aq_qgemm(packed, N, K, bits, Xd).cpu().numpy()
        assert oracle.rel_l2(got, single) <= 1e-5


def test_qgemm_batch_shares_and_separates_activations(gpu, oracle):
    """Products that read the same X share one re-ordered copy; a view with another row stride gets its own."""
    torch, aq = gpu
    K, M = 1056, 300
    X = wl.draw_activations(M, K, "bf16", 16, 0, image_rows=256, image_gain=3.0)
    X2 = wl.draw_activations(M, K, "bf16", 16, 1)
    Xd = _dev(torch, X, "bf16")
    wide = torch.zeros((M, K + 24), dtype=torch.bfloat16, device="cuda")
    wide[:, :K] = _dev(torch, X2, "bf16")
    X2d = wide[:, :K]                                   # row stride K + 24
    items, refs = [], []
    for i, (N, bits, xd, x) in enumerate([(272, 2, Xd, X), (130, 3, Xd, X), (512, 4, X2d, X2), (64, 2, Xd, X)]):
        codes, scales = wl.draw_matrix(N, K, bits, 16, i)
        packed = _pack(torch, aq, codes, scales, N, K, bits)
        Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, xd, Y))
        refs.append(oracle.qmatmul(codes, scales, N, K, bits, x, "bf16"))
    batch = aq.GemmBatch(items)
    assert batch.workspace_bytes == 2 * (304 * K * 2 + 2048)     # two distinct activation matrices (+ row factors)
    batch.run()
    torch.cuda.synchronize()
    for (packed, N, K_, bits, xd, Y), ref in zip(items, refs):
        got = Y.cpu().numpy()
        assert np.isfinite(got).all()
        assert oracle.rel_l2(got, ref) <= REL_L2_EXPECTED


# ---- prefill, fp16-weight mode (AQ_GEMM_FAST) ---------------------------------------------------------
# d * (q - z) is formed in binary16: exact for 2 bits; for 3 and 4 bits the codes whose product needs more
# than 11 significant bits are rounded (relative error <= 2^-12 per weight), which shows as rel-L2 ~1e-4.
FAST_EXPECTED = {2: 2e-5, 3: 3e-4, 4: 3e-4}


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K,M", [(200, 1056, 7), (256, 2048, 64), (512, 512, 300), (130, 4096, 81), (96, 544, 385),
                                   (17, 96, 1), (144, 288, 16), (272, 1056, 17), (128, 2048, 33), (1000, 4096, 48)])
def test_qgemm_fast_matches_oracle(gpu, oracle, bits, N, K, M, dtype):
    torch, aq = gpu
    codes, scales = wl.draw_matrix(N, K, bits, 18, N, K)
    X = wl.draw_activations(M, K, dtype, 18, N, K, image_rows=min(256, M) if M >= 256 else 0, image_gain=3.0)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, dtype), fast=True).cpu().numpy()
    ref = oracle.qmatmul(codes, scales, N, K, bits, X, dtype)
    assert np.isfinite(Y).all()
    err = oracle.rel_l2(Y, ref)
    assert err <= REL_L2_BAR
    assert err <= FAST_EXPECTED[bits], err


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_qgemm_fast_is_exact_where_the_products_are(gpu, oracle, bits):
    """Power-of-two scales make every d * (q - z) a binary16 number: with integer activations the result is
    exact whatever the summation order; one-hot rows return the dequantised weights themselves."""
    torch, aq = gpu
    N, K, M = 96, 1056, 40
    codes = wl.draw_codes(N, K, bits, 19, bits)
    scales = wl.draw_pow2_scales(N, K, 19, bits)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    for dtype in ("bf16", "f16"):
        X = wl.draw_int_activations(M, K, dtype, 19, bits)
        Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, dtype), fast=True).cpu().numpy()
        assert np.array_equal(Y.astype(np.float64), oracle.qmatmul(codes, scales, N, K, bits, X, dtype))
    ks = [0, 1, 31, 32, 33, 255, 256, 700, K - 1]
    X = np.zeros((len(ks), K), dtype=np.uint16)
    for m, k in enumerate(ks):
        X[m, k] = 0x3F80          # bf16 1.0
    Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, "bf16"), fast=True).cpu().numpy()
    W = oracle.dequant(codes, scales, N, K, bits)
    assert np.array_equal(Y.astype(np.float64), W[:, ks].T)
    # two bits: q - z is 0 or a power of two, so random scales are exact as well
    if bits == 2:
        codes, scales = wl.draw_matrix(N, K, bits, 20, bits)
        packed = _pack(torch, aq, codes, scales, N, K, bits)
        Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, "bf16"), fast=True).cpu().numpy()
        assert np.array_equal(Y.astype(np.float64), oracle.dequant(codes, scales, N, K, bits)[:, ks].T)


def test_qgemm_fast_row_factors_and_large_scales(gpu, oracle):
    """bf16 rows 2^60 apart in magnitude (each row gets its own power-of-two factor), an all-zero row, and a
    matrix whose scales would overflow binary16 once multiplied by q - z (computed on the exact path)."""
    torch, aq = gpu
    N, K, M, bits = 144, 2048, 37, 4
    codes, scales = wl.draw_matrix(N, K, bits, 21, 0)
    Xf = wl.bf16_bits_to_f32(wl.draw_activations(M, K, "bf16", 21, 0))
    for m in range(M):
        Xf[m] = np.ldexp(Xf[m], (m % 7 - 3) * 10)       # 2^-30 .. 2^+30
    Xf[5] = 0.0
    X = wl.f32_to_bf16_bits(Xf)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, "bf16"), fast=True).cpu().numpy()
    ref = oracle.qmatmul(codes, scales, N, K, bits, X, "bf16")
    assert np.isfinite(Y).all() and not Y[5].any()
    for m in range(M):
        if m != 5:
            assert oracle.rel_l2(Y[m], ref[m]) <= FAST_EXPECTED[bits], m
    # scales around 2^14: 8 * d exceeds 65504
    big = wl.f32_to_f16_bits(np.ldexp(wl.f16_bits_to_f32(scales), 19))
    assert wl.f16_bits_to_f32(big).max() > 8192 and np.isfinite(wl.f16_bits_to_f32(big)).all()
    packed = _pack(torch, aq, codes, big, N, K, bits)
    # 64 < M with too few m-tiles for the producer / consumer kernel (M = 70: 5 tiles): the shared-role kernel, whose
    # workgroups take the exact path for such a matrix (no weight is rounded); the producer / consumer kernel (M = 100)
    # and the streaming kernel (M <= 64) scale every d by a power of two before the binary16 product instead
    for M2, bar in ((70, 2e-5), (100, FAST_EXPECTED[bits]), (M, FAST_EXPECTED[bits])):
        X = wl.draw_activations(M2, K, "bf16", 21, M2)
        Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, "bf16"), fast=True).cpu().numpy()
        ref = oracle.qmatmul(codes, big, N, K, bits, X, "bf16")
        assert np.isfinite(Y).all()
        assert oracle.rel_l2(Y, ref) <= bar, M2


def test_qgemm_fast_batch_full_size_sampled(gpu, oracle):
    """One LLaMA-shaped layer (7 matrices, mixed bit-widths) at M = 300 in the launch shape the bench times, fast
    mode: sampled output columns against the oracle."""
    torch, aq = gpu
    specs = wl.backbone_stream("llama2-7b", "mixed", layers=1)
    M = wl.PREFILL_M
    Xs = {K: wl.draw_activations(M, K, "bf16", 22, K, image_rows=wl.PREFILL_IMAGE_ROWS, image_gain=wl.PREFILL_IMAGE_GAIN)
          for K in sorted({m.K for m in specs})}
    Xd = {K: _dev(torch, x, "bf16") for K, x in Xs.items()}
    items, keep = [], []
    for m in specs:
        codes, scales = wl.draw_matrix(m.N, m.K, m.bits, 22, m.index)
        packed = _pack(torch, aq, codes, scales, m.N, m.K, m.bits)
        Y = torch.full((M, m.N), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, m.N, m.K, m.bits, Xd[m.K], Y))
        rows = np.unique(np.concatenate([[0, 127, 128, m.N - 1], np.random.default_rng(m.index).integers(0, m.N, 28)]))
        keep.append((codes.reshape(m.N, -1)[rows], scales[rows], rows))
    batch = aq.GemmBatch(items, fast=True)
    batch.run()
    torch.cuda.synchronize()
    for m, (packed, N, K, bits, xd, Y), (crow, srow, rows) in zip(specs, items, keep):
        got = Y.cpu().numpy()
        assert np.isfinite(got).all()
        ref = oracle.qmatmul(crow, srow, len(rows), K, bits, Xs[K], "bf16")
        assert oracle.rel_l2(got[:, rows], ref) <= FAST_EXPECTED[bits], (m.name, bits)


# ---- block-level scale optimisation (Section 4.2, Eq. 10-11) -------------------------------------------
def _check_scale_opt(torch, aq, oracle, W, F, bits, rounds):
    N, K = W.shape
    Wd = torch.from_numpy(W).cuda()
    Fd = None if F is None else torch.from_numpy(F).cuda()
    codes_d, scales_d = aq.aq_optimize_scales(Wd, Fd, bits, rounds)
    got_codes = codes_d.cpu().numpy()
    got_scales = scales_d.view(torch.int16).cpu().numpy().view(np.uint16)
    ref_q, ref_scales = oracle.scale_optimize(W, F, bits, rounds)
    ref_codes = oracle.pack(ref_q, bits)
    assert np.array_equal(got_scales, ref_scales)
    assert np.array_equal(got_codes, ref_codes)
    return codes_d, scales_d, ref_q, ref_scales


@pytest.mark.parametrize("rounds", [0, 1, 4, 9])
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_optimize_scales_matches_oracle(gpu, oracle, bits, rounds):
    """Codes and scales are decisions taken in fp64 on both sides: required bit-exact."""
    torch, aq = gpu
    for (N, K, with_F) in [(7, 96, True), (130, 1056, True), (64, 2048, False)]:
        W = wl.draw_weights(N, K, 30, bits, rounds, N)
        F = wl.draw_sensitivities(N, K, 30, bits, rounds, N) if with_F else None
        _check_scale_opt(torch, aq, oracle, W, F, bits, rounds)


def test_optimize_scales_degenerate_blocks(gpu, oracle):
    """All-zero blocks, one non-zero element, one sign only, magnitudes beyond the fp16 scale range at both ends,
    zero sensitivities, a block whose sensitivities single out one element, and a block of exact ties between
    neighbouring codes (half-integers at a scale of one)."""
    torch, aq = gpu
    rng = np.random.default_rng(31)
    W = (rng.standard_normal((12, 64)) * 0.02).astype(np.float32)
    F = rng.uniform(0.1, 2.0, size=W.shape).astype(np.float32)
    W[0, :32] = 0.0
    W[1, :] = 0.0
    W[1, 5] = 0.3
    W[2, :32] = np.abs(W[2, :32])
    W[3, :32] = -np.abs(W[3, :32])
    W[4, :32] *= np.float32(1e7)                 # max|w| / 8 far above 65504: the scale saturates
    W[5, :32] *= np.float32(1e-7)                # scales in fp16's subnormal range
    W[6, :32] *= np.float32(1e-12)               # below the smallest subnormal: d = 0
    F[7, :32] = 0.0                              # nothing to fit: the start scale is kept
    F[8, :32] = 1e-6
    F[8, 3] = 1e6
    for bits in (2, 3, 4):
        _check_scale_opt(torch, aq, oracle, W, F, bits, 4)
        _check_scale_opt(torch, aq, oracle, W, None, bits, 2)
        T = np.zeros((1, 32), dtype=np.float32)                              # max|w| = 2^(bits-1): start scale 1
        T[0, :8] = [-(1 << (bits - 1)), 0.5, -1.5, -0.5, 1.5, -0.25, 0.75, 1.0]
        _check_scale_opt(torch, aq, oracle, T, None, bits, 0)


def test_optimize_scales_feeds_the_matmul(gpu, oracle):
    """End to end: optimise, pack, multiply; equal to the oracle's chain, and closer to the fp32 weights' product
    than plain nearest-code quantisation at the absmax scale (rounds = 0) in the sensitivity-weighted error."""
    torch, aq = gpu
    N, K, bits = 256, 2048, 3
    W = wl.draw_weights(N, K, 32, 0)
    F = wl.draw_sensitivities(N, K, 32, 0)
    codes_d, scales_d, ref_q, ref_scales = _check_scale_opt(torch, aq, oracle, W, F, bits, 4)
    packed = aq.aq_pack_weights(codes_d, scales_d, N, K, bits)
    x = wl.draw_activations(1, K, "f16", 32, 1)
    y = aq.aq_qgemv(packed, N, K, bits, _dev(torch, x[0], "f16")).cpu().numpy()
    ref = oracle.qmatmul(oracle.pack(ref_q, bits), ref_scales, N, K, bits, x, "f16")[0]
    assert oracle.rel_l2(y, ref) <= REL_L2_EXPECTED
    z = 1 << (bits - 1)
    def weighted_error(q, scales):
        what = oracle.f16_to_f64(scales).repeat(32, axis=1) * (q.astype(np.float64) - z)
        w = W.astype(np.float64)
        sig = np.sqrt(np.repeat((w.reshape(N, -1, 32) ** 2).mean(axis=2), 32, axis=1) + w * w)
        return float(np.sum(F * sig * (w - what) ** 2))
    q0, s0 = oracle.scale_optimize(W, F, bits, 0)
    assert weighted_error(ref_q, ref_scales) < 0.8 * weighted_error(q0, s0)


def test_optimize_scales_full_size_sampled(gpu, oracle):
    """A 4096 x 4096 matrix in the launch shape the bench times; the oracle checks sampled rows."""
    torch, aq = gpu
    N, K, bits = 4096, 4096, 2
    g = torch.Generator(device="cuda").manual_seed(33)
    Wd = torch.randn((N, K), generator=g, device="cuda", dtype=torch.float32) * 0.02
    Fd = torch.rand((N, K), generator=g, device="cuda", dtype=torch.float32) + 0.05
    codes_d, scales_d = aq.aq_optimize_scales(Wd, Fd, bits, 4)
    rows = [0, 1, 127, 128, 2049, 4095]
    W, F = Wd[rows].cpu().numpy(), Fd[rows].cpu().numpy()
    ref_q, ref_scales = oracle.scale_optimize(W, F, bits, 4)
    assert np.array_equal(scales_d[rows].view(torch.int16).cpu().numpy().view(np.uint16), ref_scales)
    assert np.array_equal(codes_d[rows].cpu().numpy(), oracle.pack(ref_q, bits))


def test_optimize_scales_errors(gpu):
    torch, aq = gpu
    W = torch.zeros((4, 64), dtype=torch.float32, device="cuda")
    with pytest.raises(aq.AqError):
        aq.aq_optimize_scales(W, None, 5, 4)
    with pytest.raises(aq.AqError):
        aq.aq_optimize_scales(W, None, 4, 65)
    with pytest.raises(aq.AqError):
        aq.aq_optimize_scales(W, None, 4, -1)


def test_qgemm_fast_small_m_batch(gpu, oracle):
    """Mixed-bit list at M <= 64 (the streaming kernel), shared and separate activations, f16 and bf16."""
    torch, aq = gpu
    for dtype in ("bf16", "f16"):
        M = 40
        Xs = {K: wl.draw_activations(M, K, dtype, 23, K) for K in (1056, 2048)}
        Xd = {K: _dev(torch, x, dtype) for K, x in Xs.items()}
        items, refs = [], []
        for i, (N, K, bits) in enumerate([(272, 1056, 2), (130, 2048, 3), (512, 1056, 4), (64, 2048, 2), (1000, 2048, 4)]):
            codes, scales = wl.draw_matrix(N, K, bits, 23, i)
            packed = _pack(torch, aq, codes, scales, N, K, bits)
            Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
            items.append((packed, N, K, bits, Xd[K], Y))
            refs.append((oracle.qmatmul(codes, scales, N, K, bits, Xs[K], dtype), bits))
        batch = aq.GemmBatch(items, fast=True)
        batch.run()
        batch.run()
        torch.cuda.synchronize()
        for (packed, N, K, bits, xd, Y), (ref, b) in zip(items, refs):
            got = Y.cpu().numpy()
            assert np.isfinite(got).all()
            assert oracle.rel_l2(got, ref) <= FAST_EXPECTED[b]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K,M", [(200, 1056, 7), (272, 2048, 16), (130, 4096, 29), (128, 512, 32)])
def test_qgemm_exact_small_m_rounds_no_weight(gpu, oracle, bits, N, K, M, dtype):
    """Exact mode at M <= 32 runs the streaming kernel with every weight as the sum of two binary16 terms: the
    error must be that of fp32 summation (1e-7), far below what one rounded term per weight gives at 3 and 4 bits
    (1e-4), also with scales at both ends of binary16's range."""
    torch, aq = gpu
    codes, scales = wl.draw_matrix(N, K, bits, 51, N, K)
    X = wl.draw_activations(M, K, dtype, 51, N, K)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, dtype)).cpu().numpy()
    ref = oracle.qmatmul(codes, scales, N, K, bits, X, dtype)
    assert oracle.rel_l2(Y, ref) <= 2e-6
    # a matrix of tiny (subnormal) scales, and one of scales so large that d * (q - z) leaves binary16's range
    for value, bar in ((3.0e-6, 2e-6), (20000.0, 2e-6)):
        s2 = scales.copy()
        s2[0::2] = wl.f32_to_f16_bits(np.full(s2[0::2].shape, value, dtype=np.float32))
        if value < 1.0:
            s2[1::2] = wl.f32_to_f16_bits(np.full(s2[1::2].shape, value * 37.0, dtype=np.float32))
        packed = _pack(torch, aq, codes, s2, N, K, bits)
        Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, dtype)).cpu().numpy()
        ref = oracle.qmatmul(codes, s2, N, K, bits, X, dtype)
        for rows in (slice(0, None, 2), slice(1, None, 2)):
            assert oracle.rel_l2(Y[:, rows], ref[:, rows]) <= bar, (value, rows)


def test_qgemm_exact_small_m_batch(gpu, oracle):
    """A planned exact-mode batch with every M <= 32 (the streaming kernel, mixed bit-widths, shared activations)."""
    torch, aq = gpu
    shapes = [(256, 1024, 2), (384, 1024, 3), (128, 1024, 4), (200, 544, 3)]
    M = 24
    Xs = {K: wl.draw_activations(M, K, "bf16", 52, K) for K in (1024, 544)}
    Xd = {K: _dev(torch, v, "bf16") for K, v in Xs.items()}
    items, refs = [], []
    for i, (N, K, bits) in enumerate(shapes):
        codes, scales = wl.draw_matrix(N, K, bits, 52, i)
        packed = _pack(torch, aq, codes, scales, N, K, bits)
        Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, Xd[K], Y))
        refs.append(oracle.qmatmul(codes, scales, N, K, bits, Xs[K], "bf16"))
    aq.GemmBatch(items).run()
    torch.cuda.synchronize()
    for it, ref in zip(items, refs):
        assert oracle.rel_l2(it[5].cpu().numpy(), ref) <= 2e-6


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K,M", [(200, 1056, 257), (128, 512, 320), (260, 256, 800), (300, 2048, 300), (96, 544, 645)])
def test_qgemm_fast_producer_consumer_shapes(gpu, oracle, bits, N, K, M):
    """Fast mode at prefill-sized M runs the producer / consumer kernel when blocks of 320 rows are at least 4/5 full:
    17 and 20 m-tiles in one block, 50 in three (the last one half empty), ragged N, K not a multiple of 256."""
    torch, aq = gpu
    codes, scales = wl.draw_matrix(N, K, bits, 53, N, K)
    X = wl.draw_activations(M, K, "bf16", 53, N, K, image_rows=min(256, M), image_gain=3.0)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, "bf16"), fast=True).cpu().numpy()
    ref = oracle.qmatmul(codes, scales, N, K, bits, X, "bf16")
    assert oracle.rel_l2(Y, ref) <= FAST_EXPECTED[bits]
    for m in range(0, M, 7):
        assert oracle.rel_l2(Y[m], ref[m]) <= REL_L2_BAR
    # exact where the products are: power-of-two scales, integer activations
    scales2 = wl.draw_pow2_scales(N, K, 53, bits)
    Xi = wl.draw_int_activations(M, K, "f16", 53, bits)
    packed = _pack(torch, aq, codes, scales2, N, K, bits)
    Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, Xi, "f16"), fast=True).cpu().numpy()
    assert np.array_equal(Y.astype(np.float64), oracle.qmatmul(codes, scales2, N, K, bits, Xi, "f16"))
    # scales so large that d * (q - z) leaves binary16: every scale is halved a few times first
    big = wl.f32_to_f16_bits(np.ldexp(wl.f16_bits_to_f32(scales), 19))
    packed = _pack(torch, aq, codes, big, N, K, bits)
    Y = aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, "bf16"), fast=True).cpu().numpy()
    assert np.isfinite(Y).all()
    assert oracle.rel_l2(Y, oracle.qmatmul(codes, big, N, K, bits, X, "bf16")) <= FAST_EXPECTED[bits]


@pytest.mark.parametrize("fast", [False, True])
@pytest.mark.parametrize("N,K,M,bits", [(300, 2208, 300, 3), (136, 4096, 257, 4), (512, 2336, 130, 2)])
def test_qgemm_lone_call_that_splits_k(gpu, oracle, N, K, M, bits, fast):
    """A lone product with few 128-row groups and at least 8 chunks of K runs two workgroups per (group, m-block), each
    half of the chunks (9 chunks: 5 + 4), which add their sums into an output the re-tiling launch cleared: the output
    buffer starts as NaN, has a row stride beyond N whose extra columns must stay untouched, and a second call must give
    the same bits (two parts sum to the same fp32 number in either order)."""
    torch, aq = gpu
    codes, scales = wl.draw_matrix(N, K, bits, 58, N, K)
    X = wl.draw_activations(M, K, "bf16", 58, N, K, image_rows=min(256, M), image_gain=3.0)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    Xd = _dev(torch, X, "bf16")
    big = torch.full((M, N + 24), float("nan"), dtype=torch.float32, device="cuda")
    Y = big[:, :N]
    aq.aq_qgemm(packed, N, K, bits, Xd, Y=Y, fast=fast)
    first = Y.cpu().numpy().copy()
    assert torch.isnan(big[:, N:]).all()
    ref = oracle.qmatmul(codes, scales, N, K, bits, X, "bf16")
    assert oracle.rel_l2(first, ref) <= (FAST_EXPECTED[bits] if fast else 2e-6)
    for m in range(0, M, 11):
        assert oracle.rel_l2(first[m], ref[m]) <= REL_L2_BAR
    aq.aq_qgemm(packed, N, K, bits, Xd, Y=Y, fast=fast)
    assert np.array_equal(Y.cpu().numpy(), first)
    assert torch.isnan(big[:, N:]).all()
    # integer activations, power-of-two scales: every order of summation gives the same fp32 bits
    scales2 = wl.draw_pow2_scales(N, K, 58, bits)
    Xi = wl.draw_int_activations(M, K, "f16", 58, bits)
    packed = _pack(torch, aq, codes, scales2, N, K, bits)
    Yi = aq.aq_qgemm(packed, N, K, bits, _dev(torch, Xi, "f16"), fast=fast).cpu().numpy()
    assert np.array_equal(Yi.astype(np.float64), oracle.qmatmul(codes, scales2, N, K, bits, Xi, "f16"))


@pytest.mark.parametrize("K,bits", [(32768, 3), (32768 + 4096 + 32, 2), (65536, 4)])
def test_deep_k_codecs_and_prefill(gpu, oracle, K, bits):
    """K far beyond the layer shapes (no kernel's LDS or registers grow with K): codes and dequantised weights
    bit-exact, then prefill products of the streaming kernel (M = 20), the shared-role kernel (M = 130) and the producer
    / consumer kernels (M = 300, which also splits K for so few rows), both modes, against rows of one oracle product."""
    torch, aq = gpu
    N, M = 70, 300
    codes, scales = wl.draw_matrix(N, K, bits, 59, K)
    packed = _pack(torch, aq, codes, scales, N, K, bits)
    assert np.array_equal(aq.aq_unpack_codes(packed, N, K, bits).cpu().numpy(), oracle.unpack(codes, N, K, bits))
    W = aq.aq_dequant_f32(packed, N, K, bits).cpu().numpy().astype(np.float64)
    assert np.array_equal(W, oracle.dequant(codes, scales, N, K, bits))
    X = wl.draw_activations(M, K, "bf16", 59, K, image_rows=256, image_gain=3.0)
    ref = oracle.qmatmul(codes, scales, N, K, bits, X, "bf16")
    # exact products, fp32 sums: the rounding error of a sum grows with the square root of its length; 2e-6 is the bar of
    # the other exact-mode cases (K up to 16384)
    exact_bar = 2e-6 * max(1.0, (K / 16384) ** 0.5)
    for m in (20, 130, 300):
        Xd = _dev(torch, X[:m], "bf16")
        Y = aq.aq_qgemm(packed, N, K, bits, Xd).cpu().numpy()
        assert oracle.rel_l2(Y, ref[:m]) <= exact_bar, (m, "exact")
        Yf = aq.aq_qgemm(packed, N, K, bits, Xd, fast=True).cpu().numpy()
        assert oracle.rel_l2(Yf, ref[:m]) <= FAST_EXPECTED[bits], (m, "fast")
        for r in range(0, m, 13):
            assert oracle.rel_l2(Y[r], ref[r]) <= REL_L2_BAR and oracle.rel_l2(Yf[r], ref[r]) <= REL_L2_BAR


def test_qgemv_seeded_sweep_of_shapes_around_the_kernel_boundaries(gpu, oracle):
    """Shapes drawn around what the decode kernel's structure makes special: K at and next to multiples of a chunk
    (256), of a staged segment (4096) and of a lone call's four-way split of K; N at and next to multiples of a tile
    (16) and of a group (128); every bit-width and both activation types; lone calls and one listed launch of all."""
    torch, aq = gpu
    rng = np.random.default_rng(2024)
    ks = [32, 224, 256, 288, 1024 - 32, 1024 + 32, 4096 - 32, 4096, 4096 + 32, 8192, 8192 + 256 + 32, 12288 - 32, 16384,
          32768 - 32, 32768 + 256, 65536]
    ns = [1, 15, 16, 17, 127, 128, 129, 255, 300]
    cases = [(int(rng.choice(ns)), int(k), int(rng.integers(2, 5)), str(rng.choice(["f16", "bf16"]))) for k in ks for _ in range(2)]
    items, refs = [], []
    for i, (N, K, bits, dtype) in enumerate(cases):
        codes, scales = wl.draw_matrix(N, K, bits, 97, i)
        x = wl.draw_activations(1, K, dtype, 97, i)
        packed = _pack(torch, aq, codes, scales, N, K, bits)
        xd = _dev(torch, x[0], dtype)
        ref = oracle.qmatmul(codes, scales, N, K, bits, x, dtype)[0]
        y = aq.aq_qgemv(packed, N, K, bits, xd).cpu().numpy()
        assert oracle.rel_l2(y, ref) <= REL_L2_EXPECTED, (N, K, bits, dtype)
        yb = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, xd, yb))
        refs.append(ref)
    aq.GemvBatch(items).run()
    torch.cuda.synchronize()
    for it, ref, case in zip(items, refs, cases):
        assert oracle.rel_l2(it[5].cpu().numpy(), ref) <= REL_L2_EXPECTED, case


def test_qgemm_seeded_sweep_of_lone_call_shapes(gpu, oracle):
    """Lone prefill calls at shapes drawn around what the dispatch makes special: M at and next to the streaming
    kernel's limits (16, 32, 64), the producer / consumer kernels' m-blocks and a 300-row prefill; N at and next to tiles
    and groups; K at and next to chunks and the depth from which a lone call splits K; both modes, both activation
    types, an output whose row stride exceeds N (the extra columns must stay untouched)."""
    torch, aq = gpu
    rng = np.random.default_rng(2026)
    for case in range(36):
        N = int(rng.choice([1, 16, 17, 100, 128, 129, 300, 520, int(rng.integers(1, 600))]))
        K = 32 * int(rng.choice([1, 7, 8, 9, 33, 64, 65, 96, 128, 200, int(rng.integers(1, 256))]))
        M = int(rng.choice([1, 15, 16, 17, 33, 64, 65, 100, 129, 257, 300, 385, int(rng.integers(1, 400))]))
        bits, kind = int(rng.integers(2, 5)), str(rng.choice(["bf16", "f16"]))
        codes, scales = wl.draw_matrix(N, K, bits, 71, case)
        X = wl.draw_activations(M, K, kind, 71, case)
        packed = _pack(torch, aq, codes, scales, N, K, bits)
        ref = oracle.qmatmul(codes, scales, N, K, bits, X, kind)
        pad = int(rng.choice([0, 8, 24]))
        for fast in (False, True):
            big = torch.full((M, N + pad), float("nan"), dtype=torch.float32, device="cuda")
            Y = big[:, :N]
            aq.aq_qgemm(packed, N, K, bits, _dev(torch, X, kind), Y=Y, fast=fast)
            got = Y.cpu().numpy()
            assert np.isfinite(got).all(), (case, N, K, M, bits, kind, fast)
            assert pad == 0 or torch.isnan(big[:, N:]).all(), (case, N, K, M, bits, kind, fast)
            assert oracle.rel_l2(got, ref) <= (FAST_EXPECTED[bits] if fast else 3e-6), (case, N, K, M, bits, kind, fast)


def test_qgemm_seeded_sweep_of_lists_with_unlike_products(gpu, oracle):
    """Listed prefill launches whose products differ in N, K, M and bit-width (a list's kernel is chosen from all of its
    products: the streaming kernel only when every M fits it, the producer / consumer kernels only when every product
    fills their m-tile slots, else the shared-role kernel): ten seeded lists, both modes, every output against the
    oracle."""
    torch, aq = gpu
    rng = np.random.default_rng(2027)
    for lst in range(10):
        kind = str(rng.choice(["bf16", "f16"]))
        same_m = bool(rng.integers(0, 2))
        M0 = int(rng.choice([1, 16, 20, 64, 65, 130, 300, 385]))
        tasks = []
        for j in range(int(rng.integers(1, 7))):
            N = int(rng.choice([1, 17, 128, 129, 300, int(rng.integers(1, 500))]))
            K = 32 * int(rng.choice([1, 8, 9, 64, 65, 100, int(rng.integers(1, 160))]))
            M = M0 if same_m else int(rng.choice([1, 16, 33, 64, 65, 130, 300]))
            bits = int(rng.integers(2, 5))
            codes, scales = wl.draw_matrix(N, K, bits, 73, lst, j)
            X = wl.draw_activations(M, K, kind, 73, lst, j)
            tasks.append((N, K, M, bits, _pack(torch, aq, codes, scales, N, K, bits), _dev(torch, X, kind),
                          oracle.qmatmul(codes, scales, N, K, bits, X, kind)))
        for fast in (False, True):
            items = [(packed, N, K, bits, Xd, torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda"))
                     for (N, K, M, bits, packed, Xd, _ref) in tasks]
            aq.GemmBatch(items, fast=fast).run()
            torch.cuda.synchronize()
            for it, t in zip(items, tasks):
                got = it[5].cpu().numpy()
                assert np.isfinite(got).all(), (lst, t[:4], fast)
                assert oracle.rel_l2(got, t[6]) <= (FAST_EXPECTED[t[3]] if fast else 3e-6), (lst, t[:4], fast)


def test_entry_points_replayed_from_a_captured_graph(gpu, oracle):
    """The library launches kernels only (no memset nodes, no allocation, no synchronisation), so a caller may capture
    its calls in a HIP graph: a lone decode call, a listed decode launch, a lone prefill call that splits K (its
    pre-pass clears Y) in both modes, the entry point that allocates nothing and a listed prefill launch are recorded
    once and replayed three times with new activations copied in between (the program's own eager work between replays);
    every replay must match the oracle and the eager results bit for bit."""
    torch, aq = gpu
    N, K, M = 300, 2336, 130
    mats = []
    for bits in (2, 3, 4):
        codes, scales = wl.draw_matrix(N, K, bits, 63, bits)
        mats.append((bits, codes, scales, _pack(torch, aq, codes, scales, N, K, bits)))
    x = torch.empty(K, dtype=torch.float16, device="cuda")
    X = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    ys = [torch.empty(N, dtype=torch.float32, device="cuda") for _ in range(4)]
    Ys = [torch.empty((M, N), dtype=torch.float32, device="cuda") for _ in range(6)]
    ws = torch.empty(aq.aq_qgemm_workspace_size(M, N, K, 4), dtype=torch.uint8, device="cuda")
    gv = aq.GemvBatch([(m[3], N, K, m[0], x, ys[1 + i]) for i, m in enumerate(mats)])
    gm = aq.GemmBatch([(m[3], N, K, m[0], X, Ys[3 + i]) for i, m in enumerate(mats)], fast=True)

    def calls():
        aq.aq_qgemv(mats[2][3], N, K, 4, x, ys[0])
        gv.run()
        aq.aq_qgemm(mats[1][3], N, K, 3, X, Y=Ys[0], workspace=ws)
        aq.aq_qgemm(mats[1][3], N, K, 3, X, Y=Ys[1], workspace=ws, fast=True)
        aq.aq_qgemm_noalloc(mats[0][3], N, K, 2, X, Ys[2])
        gm.run()

    def fill(seed):
        xh = wl.draw_activations(1, K, "f16", 63, seed)
        Xh = wl.draw_activations(M, K, "bf16", 63, seed, image_rows=100, image_gain=3.0)
        x.copy_(_dev(torch, xh[0], "f16"))
        X.copy_(_dev(torch, Xh, "bf16"))
        return xh, Xh

    side = torch.cuda.Stream()
    fill(0)
    side.wait_stream(torch.cuda.current_stream())
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        calls()                                           # warm-up: per-kernel attributes are set outside the capture
        with torch.cuda.graph(graph, stream=side):
            calls()
    torch.cuda.current_stream().wait_stream(side)
    for seed in (1, 2, 3):
        xh, Xh = fill(seed)
        for t in ys + Ys:
            t.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got_y = [t.cpu().numpy().copy() for t in ys]
        got_Y = [t.cpu().numpy().copy() for t in Ys]
        refs = {m[0]: oracle.qmatmul(m[1], m[2], N, K, m[0], Xh, "bf16") for m in mats}
        assert oracle.rel_l2(got_y[0], oracle.qmatmul(mats[2][1], mats[2][2], N, K, 4, xh, "f16")[0]) <= REL_L2_EXPECTED
        for i, m in enumerate(mats):
            assert oracle.rel_l2(got_y[1 + i], oracle.qmatmul(m[1], m[2], N, K, m[0], xh, "f16")[0]) <= REL_L2_EXPECTED
            assert oracle.rel_l2(got_Y[3 + i], refs[m[0]]) <= FAST_EXPECTED[m[0]]
        assert oracle.rel_l2(got_Y[0], refs[3]) <= 2e-6
        assert oracle.rel_l2(got_Y[1], refs[3]) <= FAST_EXPECTED[3]
        assert oracle.rel_l2(got_Y[2], refs[2]) <= 2e-6
        for t in ys + Ys:
            t.fill_(float("nan"))
        calls()                                           # the same calls issued eagerly
        torch.cuda.synchronize()
        for t, g in zip(ys + Ys, got_y + got_Y):
            assert np.array_equal(t.cpu().numpy(), g)
