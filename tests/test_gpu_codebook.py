"""Parity of the non-uniform codebook variant (aqc_* entry points, through the C ABI) against its fp64 oracle on the
same seeded inputs.  Bars: codes bit-exact; dequantised weights equal to the oracle's value rounded once to fp32; decode
outputs relative L2 <= 1e-3 (the acceptance bar), expected <= 2e-4 (16-bit activation digits, fp32 sums of the planes'
terms, which cancel in part for tables far from linear); bit-exact on exact-arithmetic inputs."""
import numpy as np
import pytest

import aq_workloads as wl

pytestmark = pytest.mark.gpu

REL_L2_BAR = 1e-3
REL_L2_EXPECTED = 2e-4


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2605_24011_amd as aq
    assert torch.cuda.is_available(), "these tests need the GPU"
    aq.lib()
    return torch, aq


@pytest.fixture(scope="module")
def cb():
    from oracle import aq_codebook_oracle
    return aq_codebook_oracle


@pytest.fixture(scope="module")
def oracle():
    from oracle import aq_oracle
    return aq_oracle


def dev(torch, a, kind=None):
    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16) if a.dtype == np.uint16 else np.ascontiguousarray(a)).cuda()
    if kind == "f16":
        t = t.view(torch.float16)
    elif kind == "bf16":
        t = t.view(torch.bfloat16)
    return t


def tables(cb, bits):
    """(name, levels) the bit-width is tested with; the 4-bit list holds native tables as well."""
    out = [(k, wl.draw_levels(k, bits, 1)) for k in ("quantile", "random", "dyadic", "uniform", "signed_dyadic")]
    if bits == 4:
        e = cb.e2m1_levels().astype(np.float32)
        perm = np.random.default_rng(5).permutation(16)
        out += [("e2m1", e), ("e2m1_scaled_permuted", (e * np.float32(0.37))[perm])]
    return out


SHAPES = [(8, 32), (16, 256), (17, 96), (200, 1056), (128, 4096), (300, 11008), (1000, 544)]


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_pack_unpack_dequant(gpu, cb, oracle, bits):
    torch, aq = gpu
    for N, K in [(17, 96), (200, 1056), (130, 4096)]:
        codes, scales = wl.draw_matrix(N, K, bits, 81, N, K)
        for name, levels in tables(cb, bits):
            packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits)
            q = aq.aqc_unpack_codes(packed, N, K, bits, levels).cpu().numpy()
            assert np.array_equal(q, oracle.unpack(codes, N, K, bits)), name
            W = aq.aqc_dequant_f32(packed, N, K, bits, levels).cpu().numpy()
            assert np.array_equal(W, cb.dequant(codes, scales, levels, N, K, bits).astype(np.float32)), name


def test_native_tables_are_recognised_and_stored_as_fp4_patterns(gpu, cb, oracle):
    """The E2M1 table in its own order is stored unchanged (same blob as the base packer's); scaled and permuted, it is
    still native and the blob differs only by the re-numbering, which unpack undoes."""
    torch, aq = gpu
    N, K = 40, 512
    codes, scales = wl.draw_matrix(N, K, 4, 82)
    e = cb.e2m1_levels().astype(np.float32)
    assert aq.aqc_table_info(e, 4)[0] == aq.AQC_FORM_NATIVE and aq.aqc_table_info(e * 3.0, 4)[0] == aq.AQC_FORM_NATIVE
    assert aq.aqc_table_info(wl.draw_levels("quantile", 4, 1), 4)[0] == aq.AQC_FORM_SIGNED
    assert aq.aqc_table_info(np.where(np.arange(16) == 3, 1.6, e).astype(np.float32), 4)[0] == aq.AQC_FORM_PLANES   # one level off the grid
    base = aq.aq_pack_weights(dev(torch, codes), dev(torch, scales), N, K, 4)
    own = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), e, N, K, 4)
    assert torch.equal(base, own)
    perm = np.random.default_rng(6).permutation(16)
    other = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), e[perm], N, K, 4)
    assert not torch.equal(base, other)
    assert np.array_equal(aq.aqc_unpack_codes(other, N, K, 4, e[perm]).cpu().numpy(), oracle.unpack(codes, N, K, 4))


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", SHAPES)
def test_qgemv_matches_oracle(gpu, cb, oracle, bits, N, K, dtype):
    torch, aq = gpu
    codes, scales = wl.draw_matrix(N, K, bits, 83, N, K)
    x = wl.draw_activations(1, K, dtype, 83, N, K)
    for name, levels in tables(cb, bits):
        packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits)
        y = aq.aqc_qgemv(packed, N, K, bits, levels, dev(torch, x, dtype)[0]).cpu().numpy()
        ref = cb.qmatmul(codes, scales, levels, N, K, bits, x, dtype)[0]
        err = oracle.rel_l2(y, ref)
        assert err <= REL_L2_BAR, (name, err)
        assert err <= REL_L2_EXPECTED, (name, err)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_uniform_table_agrees_with_the_base_format(gpu, cb, oracle, bits):
    torch, aq = gpu
    N, K = 256, 2048
    codes, scales = wl.draw_matrix(N, K, bits, 84, bits)
    x = dev(torch, wl.draw_activations(1, K, "f16", 84, bits), "f16")[0]
    levels = wl.draw_levels("uniform", bits)
    y_base = aq.aq_qgemv(aq.aq_pack_weights(dev(torch, codes), dev(torch, scales), N, K, bits), N, K, bits, x)
    y_cb = aq.aqc_qgemv(aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits), N, K, bits, levels, x)
    assert oracle.rel_l2(y_cb.cpu().numpy(), y_base.cpu().numpy()) <= 1e-5


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_qgemv_bit_exact_on_exact_arithmetic_inputs(gpu, cb, oracle, bits):
    """Levels that are multiples of 1/8 (and the E2M1 grid times a power of two), power-of-two scales, small integer
    activations: every product and every partial sum is exact in fp32, so the output must equal the oracle's."""
    torch, aq = gpu
    N, K = 300, 4096
    codes = wl.draw_codes(N, K, bits, 85, bits)
    scales = wl.draw_pow2_scales(N, K, 85, bits)
    x = wl.draw_int_activations(1, K, "f16", 85, bits)
    tabs = [wl.draw_levels("dyadic", bits, 2), wl.draw_levels("signed_dyadic", bits, 2)]
    if bits == 4:
        tabs.append((cb.e2m1_levels() * 0.25).astype(np.float32))
    for levels in tabs:
        packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits)
        y = aq.aqc_qgemv(packed, N, K, bits, levels, dev(torch, x, "f16")[0]).cpu().numpy()
        assert np.array_equal(y.astype(np.float64), cb.qmatmul(codes, scales, levels, N, K, bits, x, "f16")[0])


def test_mixed_batch_matches_single_calls_and_oracle(gpu, cb, oracle):
    torch, aq = gpu
    e = cb.e2m1_levels().astype(np.float32)
    specs = [(256, 1024, 2, wl.draw_levels("quantile", 2, 1)), (384, 4096, 4, e), (130, 544, 3, wl.draw_levels("quantile", 3, 1)),
             (512, 11008, 4, (e * np.float32(1.7))[::-1].copy()), (128, 2048, 4, wl.draw_levels("quantile", 4, 1)),
             (640, 4096, 3, wl.draw_levels("random", 3, 2)), (256, 2048, 2, wl.draw_levels("random", 2, 2)),
             (384, 1024, 4, wl.draw_levels("random", 4, 2))]
    items, refs, singles = [], [], []
    for i, (N, K, bits, levels) in enumerate(specs):
        codes, scales = wl.draw_matrix(N, K, bits, 86, i)
        xh = wl.draw_activations(1, K, "bf16", 86, i)
        packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits)
        x = dev(torch, xh, "bf16")[0].contiguous()
        y = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, levels, x, y))
        refs.append(cb.qmatmul(codes, scales, levels, N, K, bits, xh, "bf16")[0])
        singles.append(aq.aqc_qgemv(packed, N, K, bits, levels, x))
    aq.CbGemvBatch(items).run()
    torch.cuda.synchronize()
    for it, ref, one in zip(items, refs, singles):
        assert oracle.rel_l2(it[6].cpu().numpy(), ref) <= REL_L2_EXPECTED
        assert oracle.rel_l2(it[6].cpu().numpy(), one.cpu().numpy()) <= 1e-5
    # uniform lists take the kernel built for their form: all native, all signed 3-bit planes, all general 3-bit planes
    for sel in ([1, 3], [2], [5]):
        sub = [items[i] for i in sel]
        for it in sub:
            it[6].fill_(float("nan"))
        aq.CbGemvBatch(sub).run()
        torch.cuda.synchronize()
        for i, it in zip(sel, sub):
            assert oracle.rel_l2(it[6].cpu().numpy(), refs[i]) <= REL_L2_EXPECTED


def test_full_size_layer_sampled_rows(gpu, cb, oracle):
    """One LLaMA-2-7B-shaped layer in the launch configuration the bench times (all seven matrices in one launch, native
    4-bit tables and 2- / 3-bit quantile tables), sampled rows against the oracle."""
    torch, aq = gpu
    rng = np.random.default_rng(87)
    e = cb.e2m1_levels().astype(np.float32)
    items, checks = [], []
    for j, (name, N, K) in enumerate(wl.LLAMA2_7B_LAYER):
        bits = 2 + j % 3
        levels = e if bits == 4 else wl.draw_levels("quantile", bits, 1)
        codes, scales = wl.draw_matrix(N, K, bits, 87, j)
        xh = wl.draw_activations(1, K, "f16", 87, j)
        packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits)
        y = torch.empty(N, dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, levels, dev(torch, xh, "f16")[0].contiguous(), y))
        rows = np.sort(rng.choice(N, size=64, replace=False))
        nb = K // 32
        checks.append((rows, cb.qmatmul(codes.reshape(N, nb, -1)[rows], scales[rows], levels, len(rows), K, bits, xh, "f16")[0]))
    aq.CbGemvBatch(items).run()
    torch.cuda.synchronize()
    for it, (rows, ref) in zip(items, checks):
        assert oracle.rel_l2(it[6].cpu().numpy()[rows], ref) <= REL_L2_EXPECTED


def test_qgemv_at_deep_k(gpu, cb, oracle):
    """The decode kernel stages x a segment at a time, so its LDS does not grow with K: 32768 columns, lone and listed."""
    torch, aq = gpu
    N, K, bits = 70, 32768, 4
    levels = cb.e2m1_levels().astype(np.float32)
    codes, scales = wl.draw_matrix(N, K, bits, 92)
    xh = wl.draw_activations(1, K, "bf16", 92)
    packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits)
    x = dev(torch, xh, "bf16")[0].contiguous()
    ref = cb.qmatmul(codes, scales, levels, N, K, bits, xh, "bf16")[0]
    assert oracle.rel_l2(aq.aqc_qgemv(packed, N, K, bits, levels, x).cpu().numpy(), ref) <= REL_L2_EXPECTED
    y = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
    aq.CbGemvBatch([(packed, N, K, bits, levels, x, y)]).run()
    torch.cuda.synchronize()
    assert oracle.rel_l2(y.cpu().numpy(), ref) <= REL_L2_EXPECTED


def test_errors(gpu, cb):
    torch, aq = gpu
    N, K = 16, 64
    codes, scales = wl.draw_matrix(N, K, 2, 88)
    levels = wl.draw_levels("quantile", 2, 1)
    packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, 2)
    x = torch.zeros(K, dtype=torch.float16, device="cuda")
    with pytest.raises(aq.AqError) as e:
        aq.aqc_qgemv(packed, N, K, 2, [0.0, 1.0, float("nan"), 2.0], x)
    assert e.value.status == aq.AQ_EINVAL
    with pytest.raises(aq.AqError) as e:
        aq.aqc_qgemv(packed, N, K + 1, 2, levels, x)
    assert e.value.status == aq.AQ_EINVAL
    with pytest.raises(aq.AqError) as e:
        aq.aqc_qgemv(packed, N, K, 2, levels, x.float())
    assert e.value.status == aq.AQ_EDTYPE


# ---- prefill over codebook blobs (aqc_qgemm: weights fp16(d * levels[q])) ----
GEMM_CASES = [(8, 32, 1), (17, 96, 7), (200, 1056, 65), (128, 512, 320), (300, 4096, 300), (131, 2048, 333)]


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K,M", GEMM_CASES)
def test_qgemm_matches_oracle(gpu, cb, oracle, bits, N, K, M, dtype):
    torch, aq = gpu
    codes, scales = wl.draw_matrix(N, K, bits, 89, N, K)
    X = wl.draw_activations(M, K, dtype, 89, N, K)
    for name, levels in tables(cb, bits):
        packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits)
        Y = aq.aqc_qgemm(packed, N, K, bits, levels, dev(torch, X, dtype)).cpu().numpy()
        err = oracle.rel_l2(Y, cb.qmatmul(codes, scales, levels, N, K, bits, X, dtype))
        assert err <= REL_L2_BAR, (name, err)


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_qgemm_is_exact_when_the_binary16_weights_are(gpu, cb, oracle, bits):
    """Levels that are multiples of 1/8, power-of-two scales, small integer activations: d * level is a binary16 number
    and every fp32 sum is exact."""
    torch, aq = gpu
    N, K, M = 144, 800, 70
    codes = wl.draw_codes(N, K, bits, 90, bits)
    scales = wl.draw_pow2_scales(N, K, 90, bits)
    X = wl.draw_int_activations(M, K, "f16", 90, bits)
    for levels in (wl.draw_levels("dyadic", bits, 3), wl.draw_levels("signed_dyadic", bits, 3)):
        packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits)
        Y = aq.aqc_qgemm(packed, N, K, bits, levels, dev(torch, X, "f16")).cpu().numpy()
        assert np.array_equal(Y.astype(np.float64), cb.qmatmul(codes, scales, levels, N, K, bits, X, "f16"))


def test_qgemm_agrees_with_qgemv_row_by_row(gpu, cb, oracle):
    torch, aq = gpu
    N, K, M, bits = 256, 2048, 5, 4
    codes, scales = wl.draw_matrix(N, K, bits, 91)
    levels = cb.e2m1_levels().astype(np.float32)[::-1].copy()
    X = wl.draw_activations(M, K, "f16", 91)
    packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits)
    Xd = dev(torch, X, "f16")
    Y = aq.aqc_qgemm(packed, N, K, bits, levels, Xd).cpu().numpy()
    for m in range(M):
        y = aq.aqc_qgemv(packed, N, K, bits, levels, Xd[m].contiguous()).cpu().numpy()
        assert oracle.rel_l2(Y[m], y) <= 5e-4


def test_qgemm_list_matches_single_calls(gpu, cb, oracle):
    torch, aq = gpu
    e = cb.e2m1_levels().astype(np.float32)
    shapes = [(256, 1024, 2, wl.draw_levels("quantile", 2, 1), 300), (384, 2048, 4, e, 300),
              (130, 544, 3, wl.draw_levels("random", 3, 2), 20), (512, 1024, 4, wl.draw_levels("quantile", 4, 1), 300)]
    items, singles, Xs = [], [], {}
    for i, (N, K, bits, levels, M) in enumerate(shapes):
        codes, scales = wl.draw_matrix(N, K, bits, 93, i)
        if (M, K) not in Xs:
            Xs[(M, K)] = dev(torch, wl.draw_activations(M, K, "bf16", 93, M, K), "bf16")
        packed = aq.aqc_pack_weights(dev(torch, codes), dev(torch, scales), levels, N, K, bits)
        Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, levels, Xs[(M, K)], Y))
        singles.append(aq.aqc_qgemm(packed, N, K, bits, levels, Xs[(M, K)]))
    aq.CbGemmBatch(items).run()
    torch.cuda.synchronize()
    for it, one in zip(items, singles):
        assert torch.equal(it[6], one)
