"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol
include/aq.h declares, and rejects bad arguments before touching the device.

The device pointers below are made-up numbers.  Every call that takes them must FAIL validation (or only build a
plan on the host): these tests also run on machines with a GPU, where a call that passed validation would launch a
kernel on those addresses."""
import ctypes
import os
import re

import pytest

import paper_2605_24011_amd as aq

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def L():
    if not os.path.exists(aq.LIB_PATH):
        from paper_2605_24011_amd import build
        build.build()
    return aq.lib()


def test_every_declared_symbol_is_exported(L):
    header = open(os.path.join(ROOT, "include", "aq.h")).read()
    names = set(re.findall(r"\b(aq[2c]?_[a-z0-9_]+)\s*\(", header))
    assert {"aq_pack_weights", "aq_qgemv", "aq_qgemm", "aq_packed_size", "aq_qgemv_batch", "aq2_qgemm", "aq2_qgemm_fast",
            "aqc_qgemv", "aqc_table_info", "aqc_qgemv_batch"} <= names
    for n in names:
        assert hasattr(L, n), n


def test_packed_size_is_canonical_bytes_on_aligned_shapes(L):
    # bits/8 + 1/16 bytes per weight when N % 128 == 0 and K % 256 == 0, plus a 256-byte trailer
    T = 256
    for b, want in ((2, 5_242_880), (3, 7_340_032), (4, 9_437_184)):
        assert aq.aq_packed_size(4096, 4096, b) == want + T
    assert aq.aq_packed_size(11008, 4096, 4) == 25_362_432 + T
    assert aq.aq_packed_size(4096, 11008, 2) == 14_090_240 + T
    assert aq.aq_packed_size(16384, 2048, 3) == 14_680_064 + T
    # padded shapes are never smaller than the canonical form
    assert aq.aq_packed_size(17, 96, 3) >= 17 * 96 * 3 // 8 + 17 * 3 * 2
    # invalid arguments give 0
    for bad in ((0, 32, 4, 32), (4, 33, 4, 32), (4, 32, 5, 32), (4, 32, 4, 64), (4, 65536 + 32, 4, 32)):
        assert aq.aq_packed_size(*bad) == 0


def test_argument_validation_without_a_gpu(L):
    A = 4096   # any 16-byte aligned non-null fake address: validation must fail before it is used
    assert L.aq_pack_weights(A, A, 16, 64, 7, 32, A, 1 << 20, None) == aq.AQ_EINVAL
    assert L.aq_pack_weights(A, A, 16, 48, 4, 32, A, 1 << 20, None) == aq.AQ_EINVAL
    assert L.aq_pack_weights(None, A, 16, 64, 4, 32, A, 1 << 20, None) == aq.AQ_ENULL
    assert L.aq_pack_weights(A + 4, A, 16, 64, 4, 32, A, 1 << 20, None) == aq.AQ_EALIGN
    assert L.aq_pack_weights(A, A, 16, 64, 4, 32, A, 100, None) == aq.AQ_ESIZE
    assert L.aq_qgemv(A, 16, 64, 4, 32, A, 7, A, None) == aq.AQ_EDTYPE
    assert L.aq_qgemv(A, 16, 64, 4, 32, None, aq.AQ_F16, A, None) == aq.AQ_ENULL
    assert L.aq_qgemv(A, 16, 64, 4, 32, A, aq.AQ_F16, A + 8, None) == aq.AQ_EALIGN
    assert L.aq_qgemv(A, 0, 64, 4, 32, A, aq.AQ_F16, A, None) == aq.AQ_EINVAL
    assert L.aq_qgemm(A, 16, 64, 4, 32, A, 0, 64, aq.AQ_BF16, A, 16, None, 0, None) == aq.AQ_EINVAL
    assert L.aq_qgemm(A, 16, 64, 4, 32, A, 4, 32, aq.AQ_BF16, A, 16, None, 0, None) == aq.AQ_EINVAL   # ldx < K
    assert L.aq_qgemm(A, 16, 64, 4, 32, A, 4, 64, aq.AQ_BF16, A, 8, None, 0, None) == aq.AQ_EINVAL    # ldy < N
    assert L.aq_qgemm(A, 16, 64, 4, 32, A, 4, 64, 9, A, 16, None, 0, None) == aq.AQ_EDTYPE
    assert L.aq_unpack_codes(None, 16, 64, 4, 32, A, None) == aq.AQ_ENULL
    assert L.aq_dequant_f32(A, 16, 64, 3, 32, A + 2, None) == aq.AQ_EALIGN
    for s in (0, -1, -2, -3, -4, -5, -6, -99):
        assert aq.status_string(s)


def test_batch_plan_validation(L):
    A = 4096
    n = 3
    descs = (aq.aq_gemv_desc * n)()
    for i, d in enumerate(descs):
        d.packed, d.x, d.y, d.N, d.K, d.bits, d.x_dtype = A, A, A, 256 * (i + 1), 512, 2 + i, aq.AQ_F16
    size = L.aq_qgemv_batch_plan_size(descs, n, 32)
    assert size >= n * 80
    assert L.aq_qgemv_batch_plan_size(descs, 0, 32) == 0 and L.aq_qgemv_batch_plan_size(None, n, 32) == 0
    buf = ctypes.create_string_buffer(size)
    assert L.aq_qgemv_batch_plan(descs, n, 32, buf, size) == aq.AQ_OK
    assert L.aq_qgemv_batch_plan(descs, n, 32, buf, size - 1) == aq.AQ_ESIZE
    assert L.aq_qgemv_batch_plan(descs, 0, 32, buf, size) == aq.AQ_EINVAL
    descs[1].bits = 5
    assert L.aq_qgemv_batch_plan(descs, n, 32, buf, size) == aq.AQ_EINVAL
    descs[1].bits = 3
    descs[2].x = None
    assert L.aq_qgemv_batch_plan(descs, n, 32, buf, size) == aq.AQ_ENULL
    bad = ctypes.create_string_buffer(size)
    assert L.aq_qgemv_batch(bad, A, None) == aq.AQ_EINVAL     # not a plan image
    assert L.aq_qgemv_batch(buf, None, None) == aq.AQ_ENULL
    assert L.aq_qgemv_batch(buf, A + 8, None) == aq.AQ_EALIGN


def test_gemm_batch_plan_validation_and_workspace(L):
    """Host-side planning of a prefill list: sizes, shared activations, every error path (no GPU work)."""
    A = 4096
    n = 4
    descs = (aq.aq_gemm_desc * n)()
    shapes = [(4096, 4096), (1024, 4096), (512, 2048), (4096, 4096)]
    for i, (d, (N, K)) in enumerate(zip(descs, shapes)):
        d.packed, d.Y, d.N, d.K, d.M, d.ldx, d.ldy = A, A, N, K, 300, K, N
        d.bits, d.x_dtype = 2 + i % 3, aq.AQ_BF16
    # products 0, 1 and 3 read the same activations; product 2 its own
    descs[0].X = descs[1].X = descs[3].X = A
    descs[2].X = 2 * A
    size = L.aq_qgemm_batch_plan_size(n)
    assert size >= n * 96
    buf = ctypes.create_string_buffer(size)
    assert L.aq_qgemm_batch_plan(descs, n, 32, 0, buf, size) == aq.AQ_OK
    # one re-ordered copy per distinct X: rows rounded up to 16, 2 bytes per element
    assert L.aq_qgemm_batch_workspace_size(buf) == (304 * 4096 * 2 + 2048) + (304 * 2048 * 2 + 2048)
    assert L.aq_qgemm_workspace_size(300, 4096, 4096, 2) == 304 * 4096 * 2 + 2048
    # M <= 64: room for the streaming kernel's layout as well (k padded to 256, 16 rows: 8 KiB per chunk, + 1 KiB)
    assert L.aq_qgemm_workspace_size(1, 16, 32, 4) == 8 * 1024 + 1024
    assert L.aq_qgemm_workspace_size(64, 16, 2048, 4) == 8 * 8 * 4 * 1024 + 1024
    # same pointer but another row stride is another copy
    descs[1].ldx = 4096 + 8
    assert L.aq_qgemm_batch_plan(descs, n, 32, 0, buf, size) == aq.AQ_OK
    assert L.aq_qgemm_batch_workspace_size(buf) == 2 * (304 * 4096 * 2 + 2048) + (304 * 2048 * 2 + 2048)
    descs[1].ldx = 4096
    assert L.aq_qgemm_batch_plan(descs, n, 32, 0, buf, size - 1) == aq.AQ_ESIZE
    assert L.aq_qgemm_batch_plan(descs, 0, 32, 0, buf, size) == aq.AQ_EINVAL
    assert L.aq_qgemm_batch_plan(descs, n, 64, 0, buf, size) == aq.AQ_EINVAL
    descs[2].x_dtype = aq.AQ_F16
    assert L.aq_qgemm_batch_plan(descs, n, 32, 0, buf, size) == aq.AQ_EDTYPE     # one dtype per plan
    descs[2].x_dtype = aq.AQ_BF16
    descs[2].ldx = 2048 + 4
    assert L.aq_qgemm_batch_plan(descs, n, 32, 0, buf, size) == aq.AQ_EINVAL     # rows of X lose 16-byte alignment
    descs[2].ldx = 2048
    descs[3].Y = None
    assert L.aq_qgemm_batch_plan(descs, n, 32, 0, buf, size) == aq.AQ_ENULL
    descs[3].Y = A
    descs[3].X = A + 2
    assert L.aq_qgemm_batch_plan(descs, n, 32, 0, buf, size) == aq.AQ_EALIGN
    descs[3].X = A
    assert L.aq_qgemm_batch_plan(descs, n, 32, 0, buf, size) == aq.AQ_OK
    ws = L.aq_qgemm_batch_workspace_size(buf)
    assert ws == (304 * 4096 * 2 + 2048) + (304 * 2048 * 2 + 2048)
    bad = ctypes.create_string_buffer(size)
    assert L.aq_qgemm_batch_workspace_size(bad) == 0
    assert L.aq_qgemm_batch(bad, A, A, ws, None) == aq.AQ_EINVAL              # not a plan image
    assert L.aq_qgemm_batch(buf, None, A, ws, None) == aq.AQ_ENULL
    assert L.aq_qgemm_batch(buf, A, None, ws, None) == aq.AQ_ENULL
    assert L.aq_qgemm_batch(buf, A, A + 4, ws, None) == aq.AQ_EALIGN
    assert L.aq_qgemm_batch(buf, A, A, ws - 1, None) == aq.AQ_ESIZE
    # single call: the workspace is required and checked before anything is launched
    assert L.aq_qgemm(A, 4096, 4096, 2, 32, A, 300, 4096, aq.AQ_BF16, A, 4096, None, 0, None) == aq.AQ_ENULL
    assert L.aq_qgemm_fast(A, 4096, 4096, 2, 32, A, 300, 4096, aq.AQ_BF16, A, 4096, A, 1024, None) == aq.AQ_ESIZE
    assert L.aq_qgemm_fast(A, 4096, 4096, 2, 32, A, 0, 4096, aq.AQ_BF16, A, 4096, A, 1 << 24, None) == aq.AQ_EINVAL
    assert L.aq_qgemm_batch_plan(descs, n, 32, 7, buf, size) == aq.AQ_EINVAL          # unknown flags


def test_optimize_scales_validation_without_a_gpu(L):
    A = 4096
    assert L.aq_optimize_scales(A, A, 16, 64, 7, 32, 4, A, A, None) == aq.AQ_EINVAL
    assert L.aq_optimize_scales(A, A, 16, 48, 4, 32, 4, A, A, None) == aq.AQ_EINVAL
    assert L.aq_optimize_scales(A, A, 16, 64, 4, 64, 4, A, A, None) == aq.AQ_EINVAL
    assert L.aq_optimize_scales(A, A, 16, 64, 4, 32, 65, A, A, None) == aq.AQ_EINVAL
    assert L.aq_optimize_scales(A, A, 16, 64, 4, 32, -1, A, A, None) == aq.AQ_EINVAL
    assert L.aq_optimize_scales(None, A, 16, 64, 4, 32, 4, A, A, None) == aq.AQ_ENULL
    assert L.aq_optimize_scales(A, None, 16, 64, 4, 32, 4, A, None, None) == aq.AQ_ENULL
    assert L.aq_optimize_scales(A, A + 4, 16, 64, 4, 32, 4, A, A, None) == aq.AQ_EALIGN
    assert L.aq_optimize_scales(A, None, 16, 64, 4, 32, 4, A + 8, A, None) == aq.AQ_EALIGN


def _decode_plan(L, shape, blocks, layers, x=4096, qkv=8192, ws=16384, ws_bytes=None, plan_bytes=None, block=32):
    sh = aq.aq_block_shape(*shape)
    need_ws = L.aq_decode_workspace_size(ctypes.byref(sh))
    size = L.aq_decode_plan_size(max(layers, 1))
    buf = (ctypes.c_uint8 * max(size, 16))()
    rc = L.aq_decode_plan(ctypes.byref(sh), blocks, layers, block, x, qkv, ws,
                          need_ws if ws_bytes is None else ws_bytes, buf, size if plan_bytes is None else plan_bytes)
    return rc, buf, size


def test_decode_plan_validation_and_stage_split(L):
    A = 1 << 20
    blocks = (aq.aq_block_desc * 2)()
    for b in blocks:
        for j in range(7):
            b.w[j] = A + 4096 * j
            b.bits[j] = 2 + j % 3
        b.norm_attn, b.norm_mlp = A, A
    good = (4096, 32, 32, 128, 11008, aq.AQ_ACT_SILU, 1e-5)
    rc, buf, size = _decode_plan(L, good, blocks, 2)
    assert rc == aq.AQ_OK
    assert size == 48 + 2 * (4 * 16 + 7 * 96)
    assert L.aq_decode_workspace_size(ctypes.byref(aq.aq_block_shape(*good))) == 2 * 11008 * 4
    # the plan: 4 stages per layer; every stage fits one round of 768 workgroups and covers all of K
    import numpy as np
    raw = np.frombuffer(bytes(buf), dtype=np.uint8)
    head = raw[:16].view(np.int32)
    assert head[1] == 2 and head[2] == 8
    stages = raw[48:48 + 8 * 16].view(np.int32).reshape(8, 4)
    tasks = raw[48 + 8 * 16:48 + 8 * 16 + 14 * 96].view(np.int32).reshape(14, 24)
    assert stages[:, 1].tolist() == [3, 1, 2, 1] * 2 and stages[:, 3].tolist() == [0, 1, 0, 0] * 2
    assert (stages[:, 2] <= 768).all() and (stages[:, 2] >= 256).all()
    for st in stages:
        total = 0
        for t in tasks[st[0]:st[0] + st[1]]:
            N, K, nchunks, part, parts, wg_begin, wg_count = t[8], t[9], t[11], t[12], t[13], t[14], t[15]
            assert nchunks == (K + 255) // 256 and 1 <= part <= 8 and parts == (nchunks + part - 1) // part
            assert wg_begin == total and wg_count == ((N + 127) // 128) * parts
            total += wg_count
        assert total == st[2]
    # rejected before anything touches a device
    assert _decode_plan(L, (4090, 32, 32, 128, 11008, 0, 1e-5), blocks, 2)[0] == aq.AQ_EINVAL     # d_model % 32
    assert _decode_plan(L, (4096, 32, 5, 128, 11008, 0, 1e-5), blocks, 2)[0] == aq.AQ_EINVAL      # heads % kv heads
    assert _decode_plan(L, (4096, 32, 32, 124, 11008, 0, 1e-5), blocks, 2)[0] == aq.AQ_EINVAL     # head_dim % 8
    assert _decode_plan(L, (4096, 32, 32, 128, 11008, 7, 1e-5), blocks, 2)[0] == aq.AQ_EINVAL     # activation
    assert _decode_plan(L, (4096, 32, 32, 128, 11008, 0, -1.0), blocks, 2)[0] == aq.AQ_EINVAL     # eps
    assert _decode_plan(L, good, blocks, 0)[0] == aq.AQ_EINVAL
    assert _decode_plan(L, good, blocks, 2, block=64)[0] == aq.AQ_EINVAL
    assert _decode_plan(L, good, blocks, 2, x=None)[0] == aq.AQ_ENULL
    assert _decode_plan(L, good, blocks, 2, x=4100)[0] == aq.AQ_EALIGN
    assert _decode_plan(L, good, blocks, 2, ws_bytes=100)[0] == aq.AQ_ESIZE
    assert _decode_plan(L, good, blocks, 2, plan_bytes=size - 1)[0] == aq.AQ_ESIZE
    blocks[1].bits[3] = 5
    assert _decode_plan(L, good, blocks, 2)[0] == aq.AQ_EINVAL
    blocks[1].bits[3] = 3
    blocks[1].norm_mlp = None
    assert _decode_plan(L, good, blocks, 2)[0] == aq.AQ_ENULL
    # a step needs a plan
    assert L.aq_decode_step(None, None) == aq.AQ_ENULL
    junk = (ctypes.c_uint8 * 4096)()
    assert L.aq_decode_step(junk, None) == aq.AQ_EINVAL


def test_two_level_variant_validation_without_a_gpu(L):
    A = 1 << 20
    L.aq2_packed_size.restype = ctypes.c_size_t
    # same tiling as the base format, 192 bytes of parameters per unit instead of 256 bytes of scales, no trailer
    assert L.aq2_packed_size(128, 256, 2, 32) == 8 * (512 * 2 + 192)
    assert L.aq2_packed_size(129, 257 - 1 + 32, 3, 32) == 2 * 2 * 8 * (512 * 3 + 192)
    assert L.aq2_packed_size(128, 256, 5, 32) == 0 and L.aq2_packed_size(128, 250, 2, 32) == 0
    size = L.aq2_packed_size(64, 512, 4, 32)
    assert L.aq2_pack_weights(A, A, A, 64, 512, 4, 32, A, size - 1, None) == aq.AQ_ESIZE
    assert L.aq2_pack_weights(A, None, A, 64, 512, 4, 32, A, size, None) == aq.AQ_ENULL
    assert L.aq2_pack_weights(A, A, A + 2, 64, 512, 4, 32, A, size, None) == aq.AQ_EALIGN
    assert L.aq2_pack_weights(A, A, A, 64, 500, 4, 32, A, size, None) == aq.AQ_EINVAL
    assert L.aq2_qgemv(A, 64, 512, 4, 32, A, 7, A, None) == aq.AQ_EDTYPE
    assert L.aq2_qgemv(A, 64, 512, 6, 32, A, aq.AQ_F16, A, None) == aq.AQ_EINVAL
    assert L.aq2_qgemv(A, 64, 512, 4, 32, None, aq.AQ_F16, A, None) == aq.AQ_ENULL
    assert L.aq2_qgemv(A, 64, 512, 4, 32, A + 8, aq.AQ_F16, A, None) == aq.AQ_EALIGN
    assert L.aq2_dequant_f32(A, 64, 512, 4, 32, None, None) == aq.AQ_ENULL
    assert L.aq2_unpack_codes(A, 64, 512, 1, 32, A, None) == aq.AQ_EINVAL
    # a plan of two-level products is marked as such and launched through the common entry point
    descs = (aq.aq_gemv_desc * 2)()
    for d, (N, K, b) in zip(descs, [(256, 1024, 2), (128, 512, 3)]):
        d.packed, d.x, d.y, d.N, d.K, d.bits, d.x_dtype = A, A, A, N, K, b, aq.AQ_BF16
    size = L.aq_qgemv_batch_plan_size(descs, 2, 32)
    buf = (ctypes.c_uint8 * size)()
    assert L.aq2_qgemv_batch_plan(descs, 2, 32, buf, size) == aq.AQ_OK
    import numpy as np
    head = np.frombuffer(bytes(buf[:64]), dtype=np.int32)
    assert head[1] == 2 and head[4] == 0 and head[6] == 1          # count, mixed bit-widths, format
    assert L.aq_qgemv_batch_plan(descs, 2, 32, buf, size) == aq.AQ_OK
    assert np.frombuffer(bytes(buf[:64]), dtype=np.int32)[6] == 0
    descs[1].bits = 9
    assert L.aq2_qgemv_batch_plan(descs, 2, 32, buf, size) == aq.AQ_EINVAL
    # prefill over two-level blobs: every call below is rejected before anything is launched
    L.aq_qgemm_workspace_size.restype = ctypes.c_size_t
    ws = L.aq_qgemm_workspace_size(40, 64, 512, 4)
    assert L.aq2_qgemm(A, 64, 512, 4, 32, A, 40, 512, aq.AQ_F16, A, 64, A, ws - 1, None) == aq.AQ_ESIZE
    assert L.aq2_qgemm(A, 64, 512, 4, 32, A, 40, 512, aq.AQ_F16, A, 64, None, ws, None) == aq.AQ_ENULL
    assert L.aq2_qgemm(A, 64, 512, 4, 32, A, 40, 512, 5, A, 64, A, ws, None) == aq.AQ_EDTYPE
    assert L.aq2_qgemm(A, 64, 512, 4, 32, A, 0, 512, aq.AQ_F16, A, 64, A, ws, None) == aq.AQ_EINVAL
    assert L.aq2_qgemm(A, 64, 512, 4, 32, A, 40, 500, aq.AQ_F16, A, 64, A, ws, None) == aq.AQ_EINVAL     # ldx < K
    assert L.aq2_qgemm(A + 4, 64, 512, 4, 32, A, 40, 512, aq.AQ_F16, A, 64, A, ws, None) == aq.AQ_EALIGN
    assert L.aq2_qgemm_fast(A, 64, 512, 4, 32, A, 40, 512, aq.AQ_F16, A, 64, A, ws - 1, None) == aq.AQ_ESIZE
    assert L.aq2_qgemm_fast(A, 64, 512, 7, 32, A, 40, 512, aq.AQ_F16, A, 64, A, ws, None) == aq.AQ_EINVAL
    # planning launches nothing; the plan is marked two-level; its fp16-weight mode takes the producer / consumer
    # kernel at any M, its exact mode the 8-wavefront kernel
    gd = (aq.aq_gemm_desc * 2)()
    for d, (N, K, b, M) in zip(gd, [(256, 1024, 2, 5), (128, 512, 3, 300)]):
        d.packed, d.X, d.Y, d.N, d.K, d.M, d.ldx, d.ldy, d.bits, d.x_dtype = A, A, A, N, K, M, K, N, b, aq.AQ_BF16
    size = L.aq_qgemm_batch_plan_size(2)
    buf = (ctypes.c_uint8 * size)()
    assert L.aq2_qgemm_batch_plan(gd, 2, 32, aq.AQ_GEMM_FAST, buf, size) == aq.AQ_OK
    head = np.frombuffer(bytes(buf[:64]), dtype=np.int32)
    assert head[1] == 2 and head[2] == 0 and head[11] == 1 and head[12] == 0 and head[13] == 1 and head[14] == 1
    assert L.aq2_qgemm_batch_plan(gd, 2, 32, aq.AQ_GEMM_EXACT, buf, size) == aq.AQ_OK
    head = np.frombuffer(bytes(buf[:64]), dtype=np.int32)
    assert head[11] == 0 and head[12] == 0 and head[13] == 0 and head[14] == 1       # exact, not small, not pc, two-level
    assert L.aq_qgemm_batch_workspace_size(buf) > 0
    assert L.aq2_qgemm_batch_plan(gd, 2, 32, 5, buf, size) == aq.AQ_EINVAL
    assert L.aq_qgemm_batch_workspace_size(buf) > 0
    assert L.aq_qgemm_batch_plan(gd, 2, 32, aq.AQ_GEMM_FAST, buf, size) == aq.AQ_OK
    assert np.frombuffer(bytes(buf[:64]), dtype=np.int32)[14] == 0
    assert L.aq2_qgemm_batch_plan(gd, 2, 32, aq.AQ_GEMM_FAST, buf, size - 1) == aq.AQ_ESIZE
    gd[0].M = 0
    assert L.aq2_qgemm_batch_plan(gd, 2, 32, aq.AQ_GEMM_EXACT, buf, size) == aq.AQ_EINVAL


def test_codebook_variant_table_analysis_and_validation_without_a_gpu(L):
    """The table analysis is host arithmetic: the multilinear coefficients must reproduce the table (sum of coef[S] over
    the subsets S of a code's set bits), the E2M1 grid is recognised in any order and at any factor, and every
    launching call below is rejected before anything is launched."""
    import numpy as np
    rng = np.random.default_rng(3)
    for bits in (2, 3, 4):
        n = 1 << bits
        for T in (rng.normal(size=n), np.arange(n) - n / 2, rng.integers(-40, 41, size=n) / 8.0):
            form, coef = aq.aqc_table_info(T.astype(np.float32), bits)
            assert form == aq.AQC_FORM_PLANES
            rec = np.array([sum(coef[S] for S in range(n) if (S & q) == S) for q in range(n)])
            assert np.abs(rec - T.astype(np.float32)).max() <= 1e-6 * max(1.0, np.abs(T).max())
            if bits == 2:                       # closed form: a_0 = L0, a_1 = L1 - L0, a_2 = L2 - L0, a_3 = L3 - L2 - L1 + L0
                Tf = T.astype(np.float32).astype(np.float64)
                assert np.allclose(coef[:4], [Tf[0], Tf[1] - Tf[0], Tf[2] - Tf[0], Tf[3] - Tf[2] - Tf[1] + Tf[0]], atol=1e-6)
    e2m1 = np.array([0, .5, 1, 1.5, 2, 3, 4, 6, -0., -.5, -1, -1.5, -2, -3, -4, -6], dtype=np.float32)
    for alpha in (1.0, 0.37, 1e-3, 4096.0):
        form, coef = aq.aqc_table_info((e2m1 * np.float32(alpha))[rng.permutation(16)], 4)
        assert form == aq.AQC_FORM_NATIVE and abs(coef[0] - np.float32(alpha)) <= 1e-6 * alpha
    assert aq.aqc_table_info(np.abs(e2m1), 4)[0] == aq.AQC_FORM_PLANES   # every magnitude twice: no permutation, no pairs
    assert aq.aqc_table_info(np.zeros(16, dtype=np.float32), 4)[0] == aq.AQC_FORM_SIGNED
    # pairs +v, -v in any order: the coefficients expand the ascending magnitudes over the index bits
    for bits in (2, 3, 4):
        half = 1 << (bits - 1)
        mags = np.sort(np.abs(rng.normal(size=half))).astype(np.float32)
        T = np.concatenate([mags, -mags])[rng.permutation(2 * half)]
        form, coef = aq.aqc_table_info(T, bits)
        assert form == aq.AQC_FORM_SIGNED
        rec = np.array([sum(coef[S] for S in range(half) if (S & m) == S) for m in range(half)])
        assert np.abs(rec - mags).max() <= 1e-6
    off = np.array([-1.5, -0.5, 0.5, 1.25], dtype=np.float32)            # one magnitude without its partner
    assert aq.aqc_table_info(off, 2)[0] == aq.AQC_FORM_PLANES
    A = 1 << 20
    lv = (ctypes.c_float * 4)(-1.5, -0.25, 0.25, 1.5)
    bad = (ctypes.c_float * 4)(0.0, float("inf"), 1.0, 2.0)
    assert L.aqc_table_info(lv, 5, None, None) == aq.AQ_EINVAL
    assert L.aqc_table_info(None, 2, None, None) == aq.AQ_ENULL
    assert L.aqc_table_info(bad, 2, None, None) == aq.AQ_EINVAL
    assert L.aqc_pack_weights(A, A, lv, 16, 64, 2, 32, A, 10, None) == aq.AQ_ESIZE
    assert L.aqc_pack_weights(A, A, None, 16, 64, 2, 32, A, 1 << 20, None) == aq.AQ_ENULL
    assert L.aqc_pack_weights(A, A, bad, 16, 64, 2, 32, A, 1 << 20, None) == aq.AQ_EINVAL
    assert L.aqc_qgemv(A, 16, 64, 2, 32, lv, A, 7, A, None) == aq.AQ_EDTYPE
    assert L.aqc_qgemv(A, 16, 65, 2, 32, lv, A, aq.AQ_F16, A, None) == aq.AQ_EINVAL
    assert L.aqc_qgemv(A + 8, 16, 64, 2, 32, lv, A, aq.AQ_F16, A, None) == aq.AQ_EALIGN
    assert L.aqc_qgemv(A, 16, 64, 2, 32, lv, None, aq.AQ_F16, A, None) == aq.AQ_ENULL
    assert L.aqc_unpack_codes(A, 16, 64, 2, 32, lv, None, None) == aq.AQ_ENULL
    L.aqc_qgemm_workspace_size.restype = ctypes.c_size_t
    L.aq_qgemm_workspace_size.restype = ctypes.c_size_t
    wsz = L.aqc_qgemm_workspace_size(40, 64, 512, 2)
    assert wsz == L.aq_qgemm_workspace_size(40, 64, 512, 2) + 64 and L.aqc_qgemm_workspace_size(40, 64, 500, 2) == 0
    assert L.aqc_qgemm(A, 64, 512, 2, 32, lv, A, 40, 512, aq.AQ_F16, A, 64, A, wsz - 1, None) == aq.AQ_ESIZE
    assert L.aqc_qgemm(A, 64, 512, 2, 32, None, A, 40, 512, aq.AQ_F16, A, 64, A, wsz, None) == aq.AQ_ENULL
    assert L.aqc_qgemm(A, 64, 512, 2, 32, bad, A, 40, 512, aq.AQ_F16, A, 64, A, wsz, None) == aq.AQ_EINVAL
    assert L.aqc_qgemm(A, 64, 512, 2, 32, lv, A, 40, 500, aq.AQ_F16, A, 64, A, wsz, None) == aq.AQ_EINVAL      # ldx < K
    assert L.aqc_qgemm(A, 64, 512, 2, 32, lv, A, 40, 512, 3, A, 64, A, wsz, None) == aq.AQ_EDTYPE
    assert L.aqc_dequant_f32(A, 16, 64, 6, 32, lv, A, None) == aq.AQ_EINVAL
    # prefill list plans: the base plan image, then one table per task in plan order (longest K first)
    gd = (aq.aqc_gemm_desc * 2)()
    lv4q = (ctypes.c_float * 16)(*[float(v) for v in range(-8, 8)])
    for d, (N, K, b, tab) in zip(gd, [(256, 512, 2, lv), (128, 1024, 4, lv4q)]):
        p = d.product
        p.packed, p.X, p.Y, p.N, p.K, p.M, p.ldx, p.ldy, p.bits, p.x_dtype = A, A, A, N, K, 300, K, N, b, aq.AQ_BF16
        d.levels = ctypes.cast(tab, ctypes.c_void_p)
    L.aqc_qgemm_batch_plan_size.restype = ctypes.c_size_t
    L.aq_qgemm_batch_plan_size.restype = ctypes.c_size_t
    psz = L.aqc_qgemm_batch_plan_size(2)
    assert psz == L.aq_qgemm_batch_plan_size(2) + 128
    pbuf = (ctypes.c_uint8 * psz)()
    assert L.aqc_qgemm_batch_plan(gd, 2, 32, pbuf, psz) == aq.AQ_OK
    head = np.frombuffer(bytes(pbuf[:64]), dtype=np.int32)
    assert head[1] == 2 and head[2] == 0 and head[11] == 1 and head[13] == 1 and head[14] == 2      # mixed, fast, pc, codebook
    tabs = np.frombuffer(bytes(pbuf[psz - 128:]), dtype=np.float32).reshape(2, 16)
    assert tabs[0].tolist() == [float(v) for v in range(-8, 8)]        # K = 1024 first; planes: stored = canonical codes
    assert sorted(tabs[1, :4].tolist()) == [-1.5, -0.25, 0.25, 1.5] and not tabs[1, 4:].any()
    assert L.aq_qgemm_batch_workspace_size(pbuf) > 0
    assert L.aqc_qgemm_batch_plan(gd, 2, 32, pbuf, psz - 1) == aq.AQ_ESIZE
    gd[1].levels = None
    assert L.aqc_qgemm_batch_plan(gd, 2, 32, pbuf, psz) == aq.AQ_ENULL
    # list plans: made on the host, nothing launched
    descs = (aq.aqc_gemv_desc * 2)()
    lv4 = (ctypes.c_float * 16)(*[float(v) for v in e2m1])
    for d, (N, K, b, tab) in zip(descs, [(256, 1024, 2, lv), (300, 11008, 4, lv4)]):
        d.product.packed, d.product.x, d.product.y = A, A, A
        d.product.N, d.product.K, d.product.bits, d.product.x_dtype = N, K, b, aq.AQ_BF16
        d.levels = ctypes.cast(tab, ctypes.c_void_p)
    size = L.aqc_qgemv_batch_plan_size(descs, 2, 32)
    assert size == 64 + 2 * 192 + 16 * ((4 * (2 + 3) + 15) // 16)
    buf = (ctypes.c_uint8 * size)()
    assert L.aqc_qgemv_batch_plan(descs, 2, 32, buf, size) == aq.AQ_OK
    head = np.frombuffer(bytes(buf[:64]), dtype=np.int32)
    assert head[1] == 2 and head[2] == 11008 and head[3] == 5 and head[4] == 1          # count, max K, workgroups, light mixed
    heavy = (ctypes.c_float * 16)(*[float(v) for v in np.random.default_rng(4).normal(size=16)])     # 15 planes
    descs[1].levels = ctypes.cast(heavy, ctypes.c_void_p)
    assert L.aqc_qgemv_batch_plan(descs, 2, 32, buf, size) == aq.AQ_OK
    assert np.frombuffer(bytes(buf[:64]), dtype=np.int32)[4] == 0
    descs[0].levels = ctypes.cast(heavy, ctypes.c_void_p); descs[0].product.bits = 4
    assert L.aqc_qgemv_batch_plan(descs, 2, 32, buf, size) == aq.AQ_OK
    assert np.frombuffer(bytes(buf[:64]), dtype=np.int32)[4] == 4                       # uniform: planes at 4 bits
    descs[0].levels = ctypes.cast(lv, ctypes.c_void_p); descs[0].product.bits = 2
    descs[1].levels = ctypes.cast(lv4, ctypes.c_void_p)
    assert L.aqc_qgemv_batch_plan(descs, 2, 32, buf, size - 1) == aq.AQ_ESIZE
    assert L.aqc_qgemv_batch(buf, None, None) == aq.AQ_ENULL
    assert L.aqc_qgemv_batch(buf, A + 4, None) == aq.AQ_EALIGN
    descs[1].levels = None
    assert L.aqc_qgemv_batch_plan(descs, 2, 32, buf, size) == aq.AQ_ENULL
    zero = (ctypes.c_uint8 * size)()
    assert L.aqc_qgemv_batch(zero, A, None) == aq.AQ_EINVAL


def test_hsic_validation_without_a_gpu(L):
    A = 1 << 20
    L.aq_hsic_workspace_size.restype = ctypes.c_size_t
    K = 100
    floats = 3 * K * K + 3 * K
    assert L.aq_hsic_workspace_size(K) == ((floats * 4 + 15) // 16) * 16 + (3 * K + 8) * 8
    assert L.aq_hsic_workspace_size(1) == 0 and L.aq_hsic_workspace_size(1 << 17) == 0
    f, dbl = ctypes.c_float, ctypes.c_double
    sens = lambda *a: L.aq_hsic_sensitivity(*a)
    ws = L.aq_hsic_workspace_size(K)
    good = [A, 8, 8, f(1.0), A, 8, 8, f(1.0), A, 4, 4, f(1.0), K, dbl(1.0), dbl(1.0), A, A, ws, None]
    def with_(i, v):
        a = list(good); a[i] = v; return a
    assert sens(*with_(12, 1)) == aq.AQ_EINVAL                    # K < 2
    assert sens(*with_(3, f(0.0))) == aq.AQ_EINVAL                # gamma must be positive
    assert sens(*with_(2, 4)) == aq.AQ_EINVAL                     # row stride below the row length
    assert sens(*with_(13, dbl(-1.0))) == aq.AQ_EINVAL            # alpha in R+
    assert sens(*with_(4, None)) == aq.AQ_ENULL
    assert sens(*with_(15, A + 8)) == aq.AQ_EALIGN
    assert sens(*with_(17, ws - 1)) == aq.AQ_ESIZE
    assert L.aq_rbf_gram(A, K, 8, 8, f(-1.0), A, A, 4 * K, None) == aq.AQ_EINVAL
    assert L.aq_rbf_gram(A, K, 8, 8, f(1.0), None, A, 4 * K, None) == aq.AQ_ENULL
    assert L.aq_rbf_gram(A, K, 8, 8, f(1.0), A, A, 4 * K - 1, None) == aq.AQ_ESIZE
