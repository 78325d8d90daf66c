"""Host-only checks of the C ABI: the library loads without a GPU, exports every symbol
include/aq.h declares, and rejects bad arguments before touching the device."""
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
    names = set(re.findall(r"\b(aq_[a-z0-9_]+)\s*\(", header))
    assert {"aq_pack_weights", "aq_qgemv", "aq_qgemm", "aq_packed_size", "aq_qgemv_batch"} <= names
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
    for bad in ((0, 32, 4, 32), (4, 33, 4, 32), (4, 32, 5, 32), (4, 32, 4, 64), (4, 32768, 4, 32)):
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
    assert L.aq_qgemm(A, 16, 64, 4, 32, A, 0, 64, aq.AQ_BF16, A, 16, 0, None, 0, None) == aq.AQ_EINVAL
    assert L.aq_qgemm(A, 16, 64, 4, 32, A, 4, 32, aq.AQ_BF16, A, 16, 0, None, 0, None) == aq.AQ_EINVAL   # ldx < K
    assert L.aq_qgemm(A, 16, 64, 4, 32, A, 4, 64, aq.AQ_BF16, A, 8, 0, None, 0, None) == aq.AQ_EINVAL    # ldy < N
    assert L.aq_qgemm(A, 16, 64, 4, 32, A, 4, 64, 9, A, 16, 0, None, 0, None) == aq.AQ_EDTYPE
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
    size = L.aq_qgemv_batch_plan_size(n)
    assert size >= n * 64
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
    assert L.aq_qgemm(A, 4096, 4096, 2, 32, A, 300, 4096, aq.AQ_BF16, A, 4096, 0, None, 0, None) == aq.AQ_ENULL
    assert L.aq_qgemm(A, 4096, 4096, 2, 32, A, 300, 4096, aq.AQ_BF16, A, 4096, 1, A, 1024, None) == aq.AQ_ESIZE
    assert L.aq_qgemm(A, 4096, 4096, 2, 32, A, 300, 4096, aq.AQ_BF16, A, 4096, 2, A, 1 << 24, None) == aq.AQ_EINVAL
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
