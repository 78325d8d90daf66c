"""Parity of the two-level format variant (aq2_* entry points, through the C ABI) against its fp64 oracle on the
same seeded inputs.  Bars: codes bit-exact; dequantised weights equal to the oracle's value rounded once to fp32;
decode outputs relative L2 <= 1e-3 (expected ~1e-6: exact integer products on the matrix cores, fp32 sums); prefill
outputs relative L2 <= 1e-3, expected <= 2e-5 for aq2_qgemm (exact products, fp32 sums of the scale and the offset
term, which cancel in part) and a few 1e-4 for aq2_qgemm_fast (weights formed in binary16 with three roundings)."""
import numpy as np
import pytest

import aq_workloads as wl

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def gpu():
    import torch
    import paper_2605_24011_amd as aq
    assert torch.cuda.is_available(), "these tests need the GPU"
    aq.lib()
    return torch, aq


@pytest.fixture(scope="module")
def af():
    from oracle import aq_affine_oracle
    return aq_affine_oracle


def dev(torch, a, kind=None):
    t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16) if a.dtype == np.uint16 else np.ascontiguousarray(a)).cuda()
    if kind == "f16":
        t = t.view(torch.float16)
    elif kind == "bf16":
        t = t.view(torch.bfloat16)
    return t


def pack(torch, aq, codes, sub, sup, N, K, bits):
    return aq.aq2_pack_weights(dev(torch, codes), dev(torch, sub), dev(torch, sup), N, K, bits)


SHAPES = [(8, 32), (16, 256), (17, 96), (200, 1056), (128, 512), (300, 4096), (131, 2048)]


@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", SHAPES)
def test_codes_and_dequant(gpu, oracle, af, bits, N, K):
    torch, aq = gpu
    codes = wl.draw_codes(N, K, bits, 71, N, K)
    sub, sup = wl.draw_affine_params(N, K, bits, 71, N, K)
    packed = pack(torch, aq, codes, sub, sup, N, K, bits)
    assert packed.numel() == aq.aq2_packed_size(N, K, bits)
    assert np.array_equal(aq.aq2_unpack_codes(packed, N, K, bits).cpu().numpy(), oracle.unpack(codes, N, K, bits))
    W = aq.aq2_dequant_f32(packed, N, K, bits).cpu().numpy()
    want = af.dequant(codes, sub, sup, N, K, bits)
    assert np.array_equal(W, want.astype(np.float32))            # D a q and M c are exact; their difference rounds once


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K", SHAPES + [(4096, 4096), (512, 11008)])
def test_qgemv_matches_oracle(gpu, oracle, af, bits, N, K, dtype):
    torch, aq = gpu
    codes = wl.draw_codes(N, K, bits, 72, N, K)
    sub, sup = wl.draw_affine_params(N, K, bits, 72, N, K)
    x = wl.draw_activations(1, K, dtype, 72, N, K)[0]
    packed = pack(torch, aq, codes, sub, sup, N, K, bits)
    y = aq.aq2_qgemv(packed, N, K, bits, dev(torch, x, dtype)).cpu().numpy()
    ref = af.qmatvec(codes, sub, sup, N, K, bits, x, dtype)
    err = oracle.rel_l2(y, ref)
    assert err <= 1e-3
    assert err <= 2e-5, err


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_reduces_to_the_base_kernel_and_reads_weights(gpu, oracle, af, bits):
    torch, aq = gpu
    N, K = 144, 800
    codes = wl.draw_codes(N, K, bits, 73, bits)
    # one-hot x reads single dequantised weights
    sub, sup = wl.draw_affine_params(N, K, bits, 73, bits)
    packed = pack(torch, aq, codes, sub, sup, N, K, bits)
    W = af.dequant(codes, sub, sup, N, K, bits)
    for k in (0, 31, 32, 255, 256, 500, K - 1):
        x = np.zeros(K, dtype=np.uint16); x[k] = 0x3C00         # binary16 1.0
        y = aq.aq2_qgemv(packed, N, K, bits, dev(torch, x, "f16")).cpu().numpy()
        assert np.allclose(y, W[:, k], rtol=1e-6, atol=1e-6 * np.abs(W).max()), k   # (D a)(q - z) and z D a - M c may cancel
    # c = a, M = D 2^(bits-1): the base format with d = D a; integer x and power-of-two D make every sum exact
    rng = np.random.default_rng(bits)
    a = rng.integers(0, 16, size=(N, K // 32)).astype(np.uint8)
    D = (2.0 ** rng.integers(-8, -2, size=(N, (K + 255) // 256))).astype(np.float32)
    sup = np.stack([wl.f32_to_f16_bits(D), wl.f32_to_f16_bits(D * (1 << (bits - 1)))], axis=2)
    sub = (a | (a << 4)).astype(np.uint8)
    x = wl.draw_int_activations(1, K, "f16", 73, bits)[0]
    packed = pack(torch, aq, codes, sub, sup, N, K, bits)
    y = aq.aq2_qgemv(packed, N, K, bits, dev(torch, x, "f16")).cpu().numpy()
    d = D[:, np.arange(K // 32) // 8] * a
    base = oracle.qmatmul(codes, wl.f32_to_f16_bits(d), N, K, bits, x.reshape(1, K), "f16")[0]
    assert np.array_equal(y.astype(np.float64), base)


def test_batch_plan_matches_single_calls_and_rejects_nothing_valid(gpu, oracle, af):
    torch, aq = gpu
    shapes = [(256, 1024, 2), (384, 2048, 3), (130, 544, 4), (512, 1024, 3)]
    items, refs = [], []
    for i, (N, K, bits) in enumerate(shapes):
        codes = wl.draw_codes(N, K, bits, 74, i)
        sub, sup = wl.draw_affine_params(N, K, bits, 74, i)
        x = wl.draw_activations(1, K, "bf16", 74, i)[0]
        packed = pack(torch, aq, codes, sub, sup, N, K, bits)
        y = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, dev(torch, x, "bf16"), y))
        refs.append(af.qmatvec(codes, sub, sup, N, K, bits, x, "bf16"))
    aq.GemvBatch(items, two_level=True).run()
    torch.cuda.synchronize()
    for it, ref in zip(items, refs):
        assert oracle.rel_l2(it[5].cpu().numpy(), ref) <= 2e-5
    uniform = [it for it in items if it[3] == 3]
    for it in uniform:
        it[5].fill_(float("nan"))
    aq.GemvBatch(uniform, two_level=True).run()
    torch.cuda.synchronize()
    for it, ref in zip(uniform, [r for r, s in zip(refs, shapes) if s[2] == 3]):
        assert oracle.rel_l2(it[5].cpu().numpy(), ref) <= 2e-5


def test_full_size_sampled_rows(gpu, oracle, af):
    """A LLaMA-shaped layer in one batched launch, the configuration the bench times; sampled rows against the oracle."""
    torch, aq = gpu
    rng = np.random.default_rng(75)
    items, checks = [], []
    for j, (name, N, K) in enumerate(wl.LLAMA2_7B_LAYER):
        bits = 2 + j % 3
        codes = wl.draw_codes(N, K, bits, 75, j)
        sub, sup = wl.draw_affine_params(N, K, bits, 75, j)
        x = wl.draw_activations(1, K, "bf16", 75, j)[0]
        packed = pack(torch, aq, codes, sub, sup, N, K, bits)
        y = torch.empty(N, dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, dev(torch, x, "bf16"), y))
        rows = np.sort(rng.choice(N, size=48, replace=False))
        nb = K // 32
        checks.append((rows, af.qmatvec(codes.reshape(N, nb, -1)[rows], sub[rows], sup[rows], len(rows), K, bits, x, "bf16")))
    aq.GemvBatch(items, two_level=True).run()
    torch.cuda.synchronize()
    for it, (rows, ref) in zip(items, checks):
        assert oracle.rel_l2(it[5].cpu().numpy()[rows], ref) <= 2e-5


# ---- prefill over two-level blobs (aq2_qgemm / the two-level GemmBatch) ----

def matmul_ref(oracle, af, codes, sub, sup, N, K, bits, X, dtype):
    return oracle.activations_to_f64(X, dtype) @ af.dequant(codes, sub, sup, N, K, bits).T


GEMM_CASES = [(8, 32, 1), (16, 256, 16), (17, 96, 7), (200, 1056, 65), (128, 512, 320), (300, 4096, 300),
              (131, 2048, 333), (1024, 1024, 641)]


@pytest.mark.parametrize("fast", [False, True])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("bits", [2, 3, 4])
@pytest.mark.parametrize("N,K,M", GEMM_CASES)
def test_qgemm_matches_oracle(gpu, oracle, af, bits, N, K, M, dtype, fast):
    torch, aq = gpu
    codes = wl.draw_codes(N, K, bits, 76, N, K)
    sub, sup = wl.draw_affine_params(N, K, bits, 76, N, K)
    X = wl.draw_activations(M, K, dtype, 76, N, K)
    packed = pack(torch, aq, codes, sub, sup, N, K, bits)
    Y = aq.aq2_qgemm(packed, N, K, bits, dev(torch, X, dtype), fast=fast).cpu().numpy()
    err = oracle.rel_l2(Y, matmul_ref(oracle, af, codes, sub, sup, N, K, bits, X, dtype))
    assert err <= (1e-3 if fast else 2e-5), err


@pytest.mark.parametrize("bits", [2, 3, 4])
def test_exact_qgemm_stays_finite_where_binary16_weights_overflow(gpu, oracle, af, bits):
    """Super-block scales near the top of binary16: D a q reaches 60000 * 15 * 15, far outside binary16, which the
    fp16-weight mode documents as its limit; the exact mode scales block sums in fp32 and must match the oracle."""
    torch, aq = gpu
    N, K, M = 130, 544, 70
    codes = wl.draw_codes(N, K, bits, 80, bits)
    sub, sup = wl.draw_affine_params(N, K, bits, 80, bits)
    rng = np.random.default_rng(80 + bits)
    big = rng.uniform(20000.0, 60000.0, size=sup.shape[:2]).astype(np.float32)
    sup = np.stack([wl.f32_to_f16_bits(big), wl.f32_to_f16_bits(big * np.float32(0.9))], axis=2)
    X = wl.draw_activations(M, K, "bf16", 80, bits)
    packed = pack(torch, aq, codes, sub, sup, N, K, bits)
    Y = aq.aq2_qgemm(packed, N, K, bits, dev(torch, X, "bf16")).cpu().numpy()
    assert np.isfinite(Y).all()
    assert oracle.rel_l2(Y, matmul_ref(oracle, af, codes, sub, sup, N, K, bits, X, "bf16")) <= 2e-5


@pytest.mark.parametrize("fast", [False, True])
@pytest.mark.parametrize("bits", [2, 3, 4])
def test_qgemm_is_exact_when_the_binary16_weights_are(gpu, oracle, af, bits, fast):
    """Power-of-two D and M, integer activations: q a D and c M are short integers times a power of two, so the
    binary16 weight is the true one and every fp32 sum is exact."""
    torch, aq = gpu
    N, K, M = 144, 800, 70
    codes = wl.draw_codes(N, K, bits, 77, bits)
    rng = np.random.default_rng(100 + bits)
    a = rng.integers(0, 16, size=(N, K // 32)).astype(np.uint8)
    c = rng.integers(0, 16, size=(N, K // 32)).astype(np.uint8)
    e = rng.integers(-8, -2, size=(N, (K + 255) // 256))
    sup = np.stack([wl.f32_to_f16_bits((2.0 ** e).astype(np.float32)),
                    wl.f32_to_f16_bits((2.0 ** (e + rng.integers(0, 3, size=e.shape))).astype(np.float32))], axis=2)
    sub = (a | (c << 4)).astype(np.uint8)
    X = wl.draw_int_activations(M, K, "f16", 77, bits)
    packed = pack(torch, aq, codes, sub, sup, N, K, bits)
    Y = aq.aq2_qgemm(packed, N, K, bits, dev(torch, X, "f16"), fast=fast).cpu().numpy()
    assert np.array_equal(Y.astype(np.float64), matmul_ref(oracle, af, codes, sub, sup, N, K, bits, X, "f16"))


@pytest.mark.parametrize("fast", [False, True])
def test_qgemm_batch_matches_single_calls(gpu, oracle, af, fast):
    torch, aq = gpu
    shapes = [(256, 1024, 2, 300), (384, 2048, 3, 300), (130, 544, 4, 20), (512, 1024, 3, 300)]
    items, singles = [], []
    Xs = {}
    for i, (N, K, bits, M) in enumerate(shapes):
        codes = wl.draw_codes(N, K, bits, 78, i)
        sub, sup = wl.draw_affine_params(N, K, bits, 78, i)
        if (M, K) not in Xs:                                   # products of equal shape read the same activations
            Xs[(M, K)] = dev(torch, wl.draw_activations(M, K, "bf16", 78, M, K), "bf16")
        packed = pack(torch, aq, codes, sub, sup, N, K, bits)
        Y = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, Xs[(M, K)], Y))
        singles.append(aq.aq2_qgemm(packed, N, K, bits, Xs[(M, K)], fast=fast))
    aq.GemmBatch(items, two_level=True, fast=fast).run()
    torch.cuda.synchronize()
    for it, one in zip(items, singles):
        assert torch.equal(it[5], one)


@pytest.mark.parametrize("fast", [False, True])
def test_qgemm_full_size_sampled_columns(gpu, oracle, af, fast):
    """A LLaMA-shaped layer at the bench's M = 300 in one batched launch; sampled rows of W against the oracle."""
    torch, aq = gpu
    rng = np.random.default_rng(79)
    M = 300
    items, checks = [], []
    Xs = {}
    for j, (name, N, K) in enumerate(wl.LLAMA2_7B_LAYER):
        bits = 2 + j % 3
        codes = wl.draw_codes(N, K, bits, 79, j)
        sub, sup = wl.draw_affine_params(N, K, bits, 79, j)
        if K not in Xs:
            Xh = wl.draw_activations(M, K, "bf16", 79, K)
            Xs[K] = (Xh, dev(torch, Xh, "bf16"))
        packed = pack(torch, aq, codes, sub, sup, N, K, bits)
        Y = torch.empty((M, N), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, Xs[K][1], Y))
        rows = np.sort(rng.choice(N, size=48, replace=False))
        nb = K // 32
        checks.append((rows, matmul_ref(oracle, af, codes.reshape(N, nb, -1)[rows], sub[rows], sup[rows], len(rows), K,
                                        bits, Xs[K][0], "bf16")))
    aq.GemmBatch(items, two_level=True, fast=fast).run()
    torch.cuda.synchronize()
    for it, (rows, ref) in zip(items, checks):
        assert oracle.rel_l2(it[5].cpu().numpy()[:, rows], ref) <= (1e-3 if fast else 2e-5)


def test_qgemv_seeded_sweep_of_shapes_around_the_kernel_boundaries(gpu, oracle, af):
    """As in the base format's sweep: K around chunk, segment and K-split boundaries, N around tile and group
    boundaries, lone calls and one listed launch."""
    torch, aq = gpu
    rng = np.random.default_rng(2025)
    ks = [32, 224, 256, 288, 1024 + 32, 4096 - 32, 4096, 4096 + 32, 8192 + 256 + 32, 16384, 32768 + 256 + 32]
    ns = [1, 15, 16, 17, 127, 128, 129, 300]
    cases = [(int(rng.choice(ns)), int(k), int(rng.integers(2, 5)), str(rng.choice(["f16", "bf16"]))) for k in ks for _ in range(2)]
    items, refs = [], []
    for i, (N, K, bits, dtype) in enumerate(cases):
        codes = wl.draw_codes(N, K, bits, 98, i)
        sub, sup = wl.draw_affine_params(N, K, bits, 98, i)
        x = wl.draw_activations(1, K, dtype, 98, i)
        packed = pack(torch, aq, codes, sub, sup, N, K, bits)
        xd = dev(torch, x, dtype)[0].contiguous()
        ref = af.qmatvec(codes, sub, sup, N, K, bits, x[0], dtype)
        y = aq.aq2_qgemv(packed, N, K, bits, xd).cpu().numpy()
        assert oracle.rel_l2(y, ref) <= 2e-4, (N, K, bits, dtype)
        yb = torch.full((N,), float("nan"), dtype=torch.float32, device="cuda")
        items.append((packed, N, K, bits, xd, yb))
        refs.append(ref)
    aq.GemvBatch(items, two_level=True).run()
    torch.cuda.synchronize()
    for it, ref, case in zip(items, refs, cases):
        assert oracle.rel_l2(it[5].cpu().numpy(), ref) <= 2e-4, case
