"""The allocation-free prefill entry point (aq_qgemm_noalloc) against aq_qgemm, through the C ABI: two calls in a row,
the second with a smaller input, so that stale contents of the library's fixed scratch array would show."""
import ctypes

import numpy as np
import pytest

import aq_workloads as wl

pytestmark = pytest.mark.gpu


def test_noalloc_qgemm_equals_qgemm_on_two_calls_in_a_row(oracle):
    import torch
    import paper_2605_24011_amd as aq
    L = aq.lib()
    torch.cuda.set_device(0)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)

    def dev(a, kind):
        t = torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).cuda()
        return t.view(torch.bfloat16 if kind == "bf16" else torch.float16)

    for call, (N, K, M, bits, dt) in enumerate([(300, 2048, 300, 3, "bf16"), (130, 544, 23, 4, "f16")]):
        codes, scales = wl.draw_matrix(N, K, bits, 61, call)
        X = wl.draw_activations(M, K, dt, 62, call)
        packed = aq.aq_pack_weights(torch.from_numpy(codes).cuda(), torch.from_numpy(scales.view(np.int16)).cuda(), N, K, bits)
        Xd = dev(X, dt)
        want = aq.aq_qgemm(packed, N, K, bits, Xd)
        got = torch.full((M, N), float("nan"), dtype=torch.float32, device="cuda")
        rc = L.aq_qgemm_noalloc(ctypes.c_void_p(packed.data_ptr()), N, K, bits, 32, ctypes.c_void_p(Xd.data_ptr()), M,
                                Xd.stride(0), aq.AQ_BF16 if dt == "bf16" else aq.AQ_F16,
                                ctypes.c_void_p(got.data_ptr()), got.stride(0), stream)
        assert rc == aq.AQ_OK
        torch.cuda.synchronize()
        assert torch.equal(got, want)                 # the same kernels on the same inputs: bit for bit
        ref = oracle.qmatmul(codes, scales, N, K, bits, X, dt)
        assert oracle.rel_l2(got.cpu().numpy(), ref) <= 1e-3
    # sizes beyond the fixed array are refused before anything is launched
    A = ctypes.c_void_p(4096)
    assert L.aq_qgemm_noalloc(A, 4096, 16384, 4, 32, A, 1024, 16384, aq.AQ_BF16, A, 4096, None) == aq.AQ_ESIZE
    assert L.aq_qgemm_noalloc(A, 4096, 4096, 4, 32, None, 300, 4096, aq.AQ_BF16, A, 4096, None) == aq.AQ_ENULL
