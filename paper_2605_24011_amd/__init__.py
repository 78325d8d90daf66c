"""Python binding of libaq.so -- block-quantised matmul kernels for MI355X (gfx950).

Argument marshalling only: every function below forwards torch tensors' device pointers
to the C entry point of the same name (see include/aq.h); nothing is computed in Python
and there is no CPU fallback.  If libaq.so has not been built (paper_2605_24011_amd/build.py)
importing a function raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import Sequence

AQ_OK = 0
AQ_EINVAL, AQ_ENULL, AQ_EALIGN, AQ_ESIZE, AQ_EDTYPE, AQ_ELAUNCH = -1, -2, -3, -4, -5, -6
AQ_F16, AQ_BF16 = 1, 2
AQ_GEMM_EXACT, AQ_GEMM_FAST = 0, 1
AQ_ACT_SILU, AQ_ACT_GELU_TANH = 0, 1
BLOCK_MATRICES = ("q", "k", "v", "o", "gate", "up", "down")
BLOCK = 32

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("AQ_LIB_PATH") or os.path.join(_HERE, "libaq.so")   # AQ_LIB_PATH: another build of the same library
_lib = None

_i64, _int, _p, _sz = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_size_t


class AqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class aq_gemv_desc(ctypes.Structure):
    _fields_ = [("packed", _p), ("x", _p), ("y", _p), ("N", _i64), ("K", _i64),
                ("bits", ctypes.c_int32), ("x_dtype", ctypes.c_int32)]


class aqc_gemv_desc(ctypes.Structure):
    _fields_ = [("product", aq_gemv_desc), ("levels", _p)]


class aq_block_shape(ctypes.Structure):
    _fields_ = [("d_model", ctypes.c_int32), ("n_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("d_ff", ctypes.c_int32), ("act", ctypes.c_int32), ("eps", ctypes.c_float)]


class aq_block_desc(ctypes.Structure):
    _fields_ = [("w", _p * 7), ("bits", ctypes.c_int32 * 7), ("norm_attn", _p), ("norm_mlp", _p)]


class aq_gemm_desc(ctypes.Structure):
    _fields_ = [("packed", _p), ("X", _p), ("Y", _p), ("N", _i64), ("K", _i64), ("M", _i64), ("ldx", _i64),
                ("ldy", _i64), ("bits", ctypes.c_int32), ("x_dtype", ctypes.c_int32)]


class aqc_gemm_desc(ctypes.Structure):
    _fields_ = [("product", aq_gemm_desc), ("levels", _p)]


def lib() -> ctypes.CDLL:
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2605_24011_amd.build` "
                              "(there is no fallback path)")
        # PyTorch ships its own copy of the HIP runtime.  The library's kernels must register with the runtime
        # that owns torch's devices and streams, so torch's copy has to be in the process before libaq.so is
        # loaded (its libamdhip64 dependency then resolves to it); loaded the other way round, every launch
        # from this library fails.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(LIB_PATH)
        L.aq_status_string.restype = ctypes.c_char_p
        L.aq_status_string.argtypes = [_int]
        L.aq_packed_size.restype = _sz
        L.aq_packed_size.argtypes = [_i64, _i64, _int, _int]
        L.aq_pack_weights.argtypes = [_p, _p, _i64, _i64, _int, _int, _p, _sz, _p]
        L.aq_qgemv.argtypes = [_p, _i64, _i64, _int, _int, _p, _int, _p, _p]
        L.aq_qgemv_batch_plan_size.restype = _sz
        L.aq_qgemv_batch_plan_size.argtypes = [ctypes.POINTER(aq_gemv_desc), _int, _int]
        L.aq_qgemv_batch_plan.argtypes = [ctypes.POINTER(aq_gemv_desc), _int, _int, _p, _sz]
        L.aq_qgemv_batch.argtypes = [_p, _p, _p]
        L.aq_qgemm_workspace_size.restype = _sz
        L.aq_qgemm_workspace_size.argtypes = [_i64, _i64, _i64, _int]
        L.aq_qgemm.argtypes = [_p, _i64, _i64, _int, _int, _p, _i64, _i64, _int, _p, _i64, _p, _sz, _p]
        L.aq_qgemm_fast.argtypes = [_p, _i64, _i64, _int, _int, _p, _i64, _i64, _int, _p, _i64, _p, _sz, _p]
        L.aq_qgemm_noalloc.argtypes = [_p, _i64, _i64, _int, _int, _p, _i64, _i64, _int, _p, _i64, _p]
        L.aq_qgemm_batch_plan_size.restype = _sz
        L.aq_qgemm_batch_plan_size.argtypes = [_int]
        L.aq_qgemm_batch_plan.argtypes = [ctypes.POINTER(aq_gemm_desc), _int, _int, _int, _p, _sz]
        L.aq_qgemm_batch_workspace_size.restype = _sz
        L.aq_qgemm_batch_workspace_size.argtypes = [_p]
        L.aq_qgemm_batch.argtypes = [_p, _p, _p, _sz, _p]
        L.aq_optimize_scales.argtypes = [_p, _p, _i64, _i64, _int, _int, _int, _p, _p, _p]
        L.aq_allocate_bits.argtypes = [_p, _p, _int, _int, _p, _int, ctypes.c_double, _p]
        L.aq2_packed_size.restype = _sz
        L.aq2_packed_size.argtypes = [_i64, _i64, _int, _int]
        L.aq2_pack_weights.argtypes = [_p, _p, _p, _i64, _i64, _int, _int, _p, _sz, _p]
        L.aq2_qgemv.argtypes = [_p, _i64, _i64, _int, _int, _p, _int, _p, _p]
        L.aq2_qgemv_batch_plan.argtypes = [ctypes.POINTER(aq_gemv_desc), _int, _int, _p, _sz]
        L.aq2_qgemm.argtypes = [_p, _i64, _i64, _int, _int, _p, _i64, _i64, _int, _p, _i64, _p, _sz, _p]
        L.aq2_qgemm_fast.argtypes = L.aq2_qgemm.argtypes
        L.aq2_qgemm_batch_plan.argtypes = [ctypes.POINTER(aq_gemm_desc), _int, _int, _int, _p, _sz]
        L.aq2_unpack_codes.argtypes = [_p, _i64, _i64, _int, _int, _p, _p]
        L.aq2_dequant_f32.argtypes = [_p, _i64, _i64, _int, _int, _p, _p]
        _pf = ctypes.POINTER(ctypes.c_float)
        L.aqc_table_info.argtypes = [_pf, _int, ctypes.POINTER(ctypes.c_int), _pf]
        L.aqc_pack_weights.argtypes = [_p, _p, _pf, _i64, _i64, _int, _int, _p, _sz, _p]
        L.aqc_qgemv.argtypes = [_p, _i64, _i64, _int, _int, _pf, _p, _int, _p, _p]
        L.aqc_qgemv_batch_plan_size.restype = _sz
        L.aqc_qgemv_batch_plan_size.argtypes = [ctypes.POINTER(aqc_gemv_desc), _int, _int]
        L.aqc_qgemv_batch_plan.argtypes = [ctypes.POINTER(aqc_gemv_desc), _int, _int, _p, _sz]
        L.aqc_qgemv_batch.argtypes = [_p, _p, _p]
        L.aqc_qgemm_batch_plan_size.restype = _sz
        L.aqc_qgemm_batch_plan_size.argtypes = [_int]
        L.aqc_qgemm_batch_plan.argtypes = [ctypes.POINTER(aqc_gemm_desc), _int, _int, _p, _sz]
        L.aqc_qgemm_workspace_size.restype = _sz
        L.aqc_qgemm_workspace_size.argtypes = [_i64, _i64, _i64, _int]
        L.aqc_qgemm.argtypes = [_p, _i64, _i64, _int, _int, _pf, _p, _i64, _i64, _int, _p, _i64, _p, _sz, _p]
        L.aqc_unpack_codes.argtypes = [_p, _i64, _i64, _int, _int, _pf, _p, _p]
        L.aqc_dequant_f32.argtypes = [_p, _i64, _i64, _int, _int, _pf, _p, _p]
        L.aq_hsic_workspace_size.restype = _sz
        L.aq_hsic_workspace_size.argtypes = [_i64]
        L.aq_rbf_gram.argtypes = [_p, _i64, _i64, _i64, ctypes.c_float, _p, _p, _sz, _p]
        L.aq_hsic_sensitivity.argtypes = [_p, _i64, _i64, ctypes.c_float, _p, _i64, _i64, ctypes.c_float,
                                          _p, _i64, _i64, ctypes.c_float, _i64, ctypes.c_double, ctypes.c_double,
                                          _p, _p, _sz, _p]
        L.aq_decode_plan_size.restype = _sz
        L.aq_decode_plan_size.argtypes = [_int]
        L.aq_decode_workspace_size.restype = _sz
        L.aq_decode_workspace_size.argtypes = [ctypes.POINTER(aq_block_shape)]
        L.aq_decode_plan.argtypes = [ctypes.POINTER(aq_block_shape), ctypes.POINTER(aq_block_desc), _int, _int,
                                     _p, _p, _p, _sz, _p, _sz]
        L.aq_decode_step.argtypes = [_p, _p]
        L.aq_unpack_codes.argtypes = [_p, _i64, _i64, _int, _int, _p, _p]
        L.aq_dequant_f32.argtypes = [_p, _i64, _i64, _int, _int, _p, _p]
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().aq_status_string(int(status)).decode()


def _check(status: int, where: str) -> None:
    if status != AQ_OK:
        raise AqError(status, where)


def _stream(stream=None) -> int:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float16:
        return AQ_F16
    if t.dtype == torch.bfloat16:
        return AQ_BF16
    raise AqError(AQ_EDTYPE, "activation dtype")


def aq_packed_size(N: int, K: int, bits: int, block: int = BLOCK) -> int:
    return int(lib().aq_packed_size(N, K, bits, block))


def aq_pack_weights(codes, scales, N: int, K: int, bits: int, block: int = BLOCK, stream=None):
    """codes: cuda uint8 [N, K/32, 4*bits]; scales: cuda int16/uint16/float16 [N, K/32] -> uint8 blob."""
    import torch
    size = aq_packed_size(N, K, bits, block)
    if size == 0:
        raise AqError(AQ_EINVAL, "aq_packed_size")
    packed = torch.empty(size, dtype=torch.uint8, device=codes.device)
    _check(lib().aq_pack_weights(codes.data_ptr(), scales.data_ptr(), N, K, bits, block,
                                 packed.data_ptr(), size, _stream(stream)), "aq_pack_weights")
    return packed


def aq_qgemv(packed, N: int, K: int, bits: int, x, y=None, block: int = BLOCK, stream=None):
    """x: cuda float16/bfloat16 [K] -> y: cuda float32 [N]."""
    import torch
    if y is None:
        y = torch.empty(N, dtype=torch.float32, device=x.device)
    _check(lib().aq_qgemv(packed.data_ptr(), N, K, bits, block, x.data_ptr(), _dtype_code(x),
                          y.data_ptr(), _stream(stream)), "aq_qgemv")
    return y


class GemvBatch:
    """A planned stream of decode products (one launch).  Holds references to every tensor."""

    def __init__(self, items: Sequence[tuple], block: int = BLOCK, two_level: bool = False):
        """items: (packed, N, K, bits, x, y) per matrix; two_level: every blob is in the two-level format variant
        (aq2_pack_weights) and the list is planned with aq2_qgemv_batch_plan."""
        import torch
        n = len(items)
        descs = (aq_gemv_desc * n)()
        for d, (packed, N, K, bits, x, y) in zip(descs, items):
            d.packed, d.x, d.y = packed.data_ptr(), x.data_ptr(), y.data_ptr()
            d.N, d.K, d.bits, d.x_dtype = N, K, bits, _dtype_code(x)
        size = int(lib().aq_qgemv_batch_plan_size(descs, n, block))      # 0: an invalid descriptor; the planner names it
        self.plan_host = torch.empty(max(size, 64), dtype=torch.uint8)
        plan = lib().aq2_qgemv_batch_plan if two_level else lib().aq_qgemv_batch_plan
        _check(plan(descs, n, block, self.plan_host.data_ptr(), size), "aq_qgemv_batch_plan")
        self.plan_dev = self.plan_host.to(items[0][0].device)
        self.items = list(items)

    def run(self, stream=None) -> None:
        _check(lib().aq_qgemv_batch(self.plan_host.data_ptr(), self.plan_dev.data_ptr(), _stream(stream)),
               "aq_qgemv_batch")


def aq_qgemm_workspace_size(M: int, N: int, K: int, bits: int) -> int:
    return int(lib().aq_qgemm_workspace_size(M, N, K, bits))


def aq_qgemm(packed, N: int, K: int, bits: int, X, Y=None, workspace=None, block: int = BLOCK, stream=None,
             fast: bool = False):
    """X: cuda bfloat16/float16 [M, K] (row stride = X.stride(0)) -> Y: cuda float32 [M, N].
    fast=True forwards to the C entry point aq_qgemm_fast (weights formed in binary16) instead of aq_qgemm."""
    import torch
    M = X.shape[0]
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.float32, device=X.device)
    need = aq_qgemm_workspace_size(M, N, K, bits)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    fn = lib().aq_qgemm_fast if fast else lib().aq_qgemm
    _check(fn(packed.data_ptr(), N, K, bits, block, X.data_ptr(), M, X.stride(0), _dtype_code(X),
              Y.data_ptr(), Y.stride(0), ws_ptr, ws_bytes, _stream(stream)), "aq_qgemm_fast" if fast else "aq_qgemm")
    return Y


def aq_qgemm_noalloc(packed, N: int, K: int, bits: int, X, Y, block: int = BLOCK, stream=None):
    """The C entry point aq_qgemm_noalloc: aq_qgemm with the library's own fixed scratch array as workspace.  Y is the
    caller's (this wrapper allocates nothing either)."""
    _check(lib().aq_qgemm_noalloc(packed.data_ptr(), N, K, bits, block, X.data_ptr(), X.shape[0], X.stride(0), _dtype_code(X),
                                  Y.data_ptr(), Y.stride(0), _stream(stream)), "aq_qgemm_noalloc")
    return Y


def aq_qgemm_fast(packed, N: int, K: int, bits: int, X, Y=None, workspace=None, block: int = BLOCK, stream=None):
    """The C entry point aq_qgemm_fast: as aq_qgemm with the weights formed in binary16."""
    return aq_qgemm(packed, N, K, bits, X, Y, workspace, block, stream, fast=True)


class GemmBatch:
    """A planned list of prefill products (one launch).  Holds references to every tensor."""

    def __init__(self, items: Sequence[tuple], block: int = BLOCK, fast: bool = False, two_level: bool = False):
        """items: (packed, N, K, bits, X, Y) per matrix; X [M, K] half/bfloat16, Y [M, N] float32.
        two_level: every blob is in the two-level variant of the format (aq2_qgemm_batch_plan)."""
        import torch
        n = len(items)
        descs = (aq_gemm_desc * n)()
        for d, (packed, N, K, bits, X, Y) in zip(descs, items):
            d.packed, d.X, d.Y = packed.data_ptr(), X.data_ptr(), Y.data_ptr()
            d.N, d.K, d.M, d.ldx, d.ldy = N, K, X.shape[0], X.stride(0), Y.stride(0)
            d.bits, d.x_dtype = bits, _dtype_code(X)
        size = int(lib().aq_qgemm_batch_plan_size(n))
        self.plan_host = torch.empty(size, dtype=torch.uint8)
        if two_level:
            _check(lib().aq2_qgemm_batch_plan(descs, n, block, AQ_GEMM_FAST if fast else AQ_GEMM_EXACT,
                                              self.plan_host.data_ptr(), size), "aq2_qgemm_batch_plan")
        else:
            _check(lib().aq_qgemm_batch_plan(descs, n, block, AQ_GEMM_FAST if fast else AQ_GEMM_EXACT,
                                             self.plan_host.data_ptr(), size), "aq_qgemm_batch_plan")
        self.plan_dev = self.plan_host.to(items[0][0].device)
        self.workspace_bytes = int(lib().aq_qgemm_batch_workspace_size(self.plan_host.data_ptr()))
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=items[0][0].device)
        self.items = list(items)

    def run(self, stream=None) -> None:
        _check(lib().aq_qgemm_batch(self.plan_host.data_ptr(), self.plan_dev.data_ptr(), self.workspace.data_ptr(),
                                    self.workspace_bytes, _stream(stream)), "aq_qgemm_batch")


def aq_optimize_scales(W, F, bits: int, rounds: int = 4, block: int = BLOCK, stream=None):
    """W (and F, or None) cuda float32 [N, K] -> (codes uint8 [N, K/32, 4*bits], scales int16 view of fp16 bits
    [N, K/32]): the canonical form aq_pack_weights takes."""
    import torch
    N, K = W.shape
    assert W.dtype == torch.float32 and W.is_contiguous() and (F is None or (F.dtype == torch.float32 and F.is_contiguous()
                                                                              and F.shape == W.shape))
    codes = torch.empty((N, K // block, 4 * bits), dtype=torch.uint8, device=W.device)
    scales = torch.empty((N, K // block), dtype=torch.float16, device=W.device)
    _check(lib().aq_optimize_scales(W.data_ptr(), None if F is None else F.data_ptr(), N, K, bits, block, rounds,
                                    codes.data_ptr(), scales.data_ptr(), _stream(stream)), "aq_optimize_scales")
    return codes, scales


def aq_allocate_bits(S, sizes, choices=(2, 3, 4), avg_bits_budget: float = 2.5):
    """Host-only greedy layer-balanced allocation.  S, sizes: [L][J] nested sequences -> bits [L][J] (lists)."""
    L, J = len(S), len(S[0])
    Sa = (ctypes.c_double * (L * J))(*[float(v) for row in S for v in row])
    na = (ctypes.c_int64 * (L * J))(*[int(v) for row in sizes for v in row])
    ca = (ctypes.c_int * len(choices))(*[int(c) for c in choices])
    out = (ctypes.c_int * (L * J))()
    _check(lib().aq_allocate_bits(Sa, na, L, J, ca, len(choices), float(avg_bits_budget), out), "aq_allocate_bits")
    return [[int(out[l * J + j]) for j in range(J)] for l in range(L)]


class DecodeStep:
    """A planned decode step through a stack of transformer blocks (aq_decode_plan / aq_decode_step).

    layers[l] = {"q": (packed, bits), ..., "down": (packed, bits), "norm_attn": float32 tensor, "norm_mlp": ...};
    x: float32 [d_model] residual stream (advanced in place by run()); qkv: float32
    [layers, n_heads*head_dim + 2*n_kv_heads*head_dim], overwritten by run().  Holds references to every tensor."""

    def __init__(self, d_model: int, n_heads: int, n_kv_heads: int, head_dim: int, d_ff: int, act: str, eps: float,
                 layers: Sequence[dict], x, qkv, block: int = BLOCK):
        import torch
        acts = {"silu": AQ_ACT_SILU, "gelu_tanh": AQ_ACT_GELU_TANH}
        if act not in acts:
            raise AqError(AQ_EINVAL, "DecodeStep")
        self.shape = aq_block_shape(d_model, n_heads, n_kv_heads, head_dim, d_ff, acts[act], eps)
        n = len(layers)
        descs = (aq_block_desc * max(n, 1))()
        for d, layer in zip(descs, layers):
            for j, name in enumerate(BLOCK_MATRICES):
                packed, bits = layer[name]
                d.w[j] = packed.data_ptr()
                d.bits[j] = bits
            d.norm_attn, d.norm_mlp = layer["norm_attn"].data_ptr(), layer["norm_mlp"].data_ptr()
        ws = int(lib().aq_decode_workspace_size(ctypes.byref(self.shape)))
        self.workspace = torch.empty(max(ws, 16), dtype=torch.uint8, device=x.device)
        size = int(lib().aq_decode_plan_size(n))
        self.plan_host = torch.empty(max(size, 16), dtype=torch.uint8)
        _check(lib().aq_decode_plan(ctypes.byref(self.shape), descs, n, block, x.data_ptr(), qkv.data_ptr(),
                                    self.workspace.data_ptr(), ws, self.plan_host.data_ptr(), size), "aq_decode_plan")
        self.layers, self.x, self.qkv = list(layers), x, qkv

    def run(self, stream=None) -> None:
        _check(lib().aq_decode_step(self.plan_host.data_ptr(), _stream(stream)),
               "aq_decode_step")


def aq_unpack_codes(packed, N: int, K: int, bits: int, block: int = BLOCK, stream=None):
    import torch
    out = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    _check(lib().aq_unpack_codes(packed.data_ptr(), N, K, bits, block, out.data_ptr(), _stream(stream)),
           "aq_unpack_codes")
    return out


def aq_dequant_f32(packed, N: int, K: int, bits: int, block: int = BLOCK, stream=None):
    import torch
    out = torch.empty((N, K), dtype=torch.float32, device=packed.device)
    _check(lib().aq_dequant_f32(packed.data_ptr(), N, K, bits, block, out.data_ptr(), _stream(stream)),
           "aq_dequant_f32")
    return out


# ---- two-level variant of the format (include/aq.h, aq2_*) ----
def aq2_packed_size(N: int, K: int, bits: int, block: int = BLOCK) -> int:
    return int(lib().aq2_packed_size(N, K, bits, block))


def aq2_pack_weights(codes, sub, sup, N: int, K: int, bits: int, block: int = BLOCK, stream=None):
    """codes: cuda uint8 [N, K/32, 4*bits]; sub: cuda uint8 [N, K/32]; sup: cuda int16/uint16/float16
    [N, ceil(K/256), 2] -> uint8 blob."""
    import torch
    size = aq2_packed_size(N, K, bits, block)
    if size == 0:
        raise AqError(AQ_EINVAL, "aq2_packed_size")
    packed = torch.empty(size, dtype=torch.uint8, device=codes.device)
    _check(lib().aq2_pack_weights(codes.data_ptr(), sub.data_ptr(), sup.data_ptr(), N, K, bits, block,
                                  packed.data_ptr(), size, _stream(stream)), "aq2_pack_weights")
    return packed


def aq2_qgemv(packed, N: int, K: int, bits: int, x, y=None, block: int = BLOCK, stream=None):
    import torch
    if y is None:
        y = torch.empty(N, dtype=torch.float32, device=x.device)
    _check(lib().aq2_qgemv(packed.data_ptr(), N, K, bits, block, x.data_ptr(), _dtype_code(x),
                           y.data_ptr(), _stream(stream)), "aq2_qgemv")
    return y


def aq2_qgemm(packed, N: int, K: int, bits: int, X, Y=None, workspace=None, block: int = BLOCK, stream=None,
              fast: bool = False):
    """X: cuda bfloat16/float16 [M, K] -> Y: cuda float32 [M, N], the blob in the two-level variant of the format.
    Exact products; fast=True calls aq2_qgemm_fast (fp16 weights)."""
    import torch
    M = X.shape[0]
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.float32, device=X.device)
    need = aq_qgemm_workspace_size(M, N, K, bits)
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    fn = lib().aq2_qgemm_fast if fast else lib().aq2_qgemm
    _check(fn(packed.data_ptr(), N, K, bits, block, X.data_ptr(), M, X.stride(0), _dtype_code(X),
              Y.data_ptr(), Y.stride(0), ws_ptr, ws_bytes, _stream(stream)), "aq2_qgemm_fast" if fast else "aq2_qgemm")
    return Y


def aq2_qgemm_fast(packed, N: int, K: int, bits: int, X, Y=None, workspace=None, block: int = BLOCK, stream=None):
    return aq2_qgemm(packed, N, K, bits, X, Y, workspace, block, stream, fast=True)


def aq2_unpack_codes(packed, N: int, K: int, bits: int, block: int = BLOCK, stream=None):
    import torch
    out = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    _check(lib().aq2_unpack_codes(packed.data_ptr(), N, K, bits, block, out.data_ptr(), _stream(stream)),
           "aq2_unpack_codes")
    return out


def aq2_dequant_f32(packed, N: int, K: int, bits: int, block: int = BLOCK, stream=None):
    import torch
    out = torch.empty((N, K), dtype=torch.float32, device=packed.device)
    _check(lib().aq2_dequant_f32(packed.data_ptr(), N, K, bits, block, out.data_ptr(), _stream(stream)),
           "aq2_dequant_f32")
    return out


# ---- non-uniform codebook variant of the format ----
def _levels(levels, bits: int):
    vals = [float(v) for v in levels]
    if len(vals) != (1 << bits):
        raise AqError(AQ_EINVAL, "levels")
    return (ctypes.c_float * len(vals))(*vals)


AQC_FORM_PLANES, AQC_FORM_NATIVE, AQC_FORM_SIGNED = 0, 1, 2


def aqc_table_info(levels, bits: int):
    """-> (form: AQC_FORM_*, coef: list of 16 floats); see aq.h."""
    form = ctypes.c_int(0)
    coef = (ctypes.c_float * 16)()
    _check(lib().aqc_table_info(_levels(levels, bits), bits, ctypes.byref(form), coef), "aqc_table_info")
    return int(form.value), list(coef)


def aqc_pack_weights(codes, scales, levels, N: int, K: int, bits: int, block: int = BLOCK, stream=None):
    import torch
    size = aq_packed_size(N, K, bits, block)
    if size == 0:
        raise AqError(AQ_EINVAL, "aq_packed_size")
    packed = torch.empty(size, dtype=torch.uint8, device=codes.device)
    _check(lib().aqc_pack_weights(codes.data_ptr(), scales.data_ptr(), _levels(levels, bits), N, K, bits, block,
                                  packed.data_ptr(), size, _stream(stream)), "aqc_pack_weights")
    return packed


def aqc_qgemv(packed, N: int, K: int, bits: int, levels, x, y=None, block: int = BLOCK, stream=None):
    """x: cuda float16/bfloat16 [K] -> y: cuda float32 [N], the blob packed with aqc_pack_weights and the same levels."""
    import torch
    if y is None:
        y = torch.empty(N, dtype=torch.float32, device=x.device)
    _check(lib().aqc_qgemv(packed.data_ptr(), N, K, bits, block, _levels(levels, bits), x.data_ptr(), _dtype_code(x),
                           y.data_ptr(), _stream(stream)), "aqc_qgemv")
    return y


class CbGemvBatch:
    """A planned stream of decode products over codebook blobs (one launch).  Holds references to every tensor."""

    def __init__(self, items: Sequence[tuple], block: int = BLOCK):
        """items: (packed, N, K, bits, levels, x, y) per matrix."""
        import torch
        n = len(items)
        descs = (aqc_gemv_desc * n)()
        self._tables = []
        for d, (packed, N, K, bits, levels, x, y) in zip(descs, items):
            d.product.packed, d.product.x, d.product.y = packed.data_ptr(), x.data_ptr(), y.data_ptr()
            d.product.N, d.product.K, d.product.bits, d.product.x_dtype = N, K, bits, _dtype_code(x)
            tab = _levels(levels, bits)
            self._tables.append(tab)
            d.levels = ctypes.cast(tab, _p)
        size = int(lib().aqc_qgemv_batch_plan_size(descs, n, block))
        self.plan_host = torch.empty(max(size, 64), dtype=torch.uint8)
        _check(lib().aqc_qgemv_batch_plan(descs, n, block, self.plan_host.data_ptr(), size), "aqc_qgemv_batch_plan")
        self.plan_dev = self.plan_host.to(items[0][0].device)
        self.items = list(items)

    def run(self, stream=None) -> None:
        _check(lib().aqc_qgemv_batch(self.plan_host.data_ptr(), self.plan_dev.data_ptr(), _stream(stream)),
               "aqc_qgemv_batch")


def aqc_qgemm(packed, N: int, K: int, bits: int, levels, X, Y=None, workspace=None, block: int = BLOCK, stream=None):
    """X: cuda bfloat16/float16 [M, K] -> Y: cuda float32 [M, N], weights fp16(d * levels[q]) (see aq.h)."""
    import torch
    M = X.shape[0]
    if Y is None:
        Y = torch.empty((M, N), dtype=torch.float32, device=X.device)
    need = int(lib().aqc_qgemm_workspace_size(M, N, K, bits))
    if workspace is None and need:
        workspace = torch.empty(need, dtype=torch.uint8, device=X.device)
    ws_ptr = workspace.data_ptr() if workspace is not None else None
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    _check(lib().aqc_qgemm(packed.data_ptr(), N, K, bits, block, _levels(levels, bits), X.data_ptr(), M, X.stride(0),
                           _dtype_code(X), Y.data_ptr(), Y.stride(0), ws_ptr, ws_bytes, _stream(stream)), "aqc_qgemm")
    return Y


class CbGemmBatch:
    """A planned list of prefill products over codebook blobs (two launches).  Holds references to every tensor."""

    def __init__(self, items: Sequence[tuple], block: int = BLOCK):
        """items: (packed, N, K, bits, levels, X, Y) per matrix; X [M, K] half/bfloat16, Y [M, N] float32."""
        import torch
        n = len(items)
        descs = (aqc_gemm_desc * n)()
        self._tables = []
        for d, (packed, N, K, bits, levels, X, Y) in zip(descs, items):
            p = d.product
            p.packed, p.X, p.Y = packed.data_ptr(), X.data_ptr(), Y.data_ptr()
            p.N, p.K, p.M, p.ldx, p.ldy = N, K, X.shape[0], X.stride(0), Y.stride(0)
            p.bits, p.x_dtype = bits, _dtype_code(X)
            tab = _levels(levels, bits)
            self._tables.append(tab)
            d.levels = ctypes.cast(tab, _p)
        size = int(lib().aqc_qgemm_batch_plan_size(n))
        self.plan_host = torch.empty(size, dtype=torch.uint8)
        _check(lib().aqc_qgemm_batch_plan(descs, n, block, self.plan_host.data_ptr(), size), "aqc_qgemm_batch_plan")
        self.plan_dev = self.plan_host.to(items[0][0].device)
        self.workspace_bytes = int(lib().aq_qgemm_batch_workspace_size(self.plan_host.data_ptr()))
        self.workspace = torch.empty(self.workspace_bytes, dtype=torch.uint8, device=items[0][0].device)
        self.items = list(items)

    def run(self, stream=None) -> None:
        _check(lib().aq_qgemm_batch(self.plan_host.data_ptr(), self.plan_dev.data_ptr(), self.workspace.data_ptr(),
                                    self.workspace_bytes, _stream(stream)), "aq_qgemm_batch")


def aqc_unpack_codes(packed, N: int, K: int, bits: int, levels, block: int = BLOCK, stream=None):
    import torch
    out = torch.empty((N, K), dtype=torch.uint8, device=packed.device)
    _check(lib().aqc_unpack_codes(packed.data_ptr(), N, K, bits, block, _levels(levels, bits), out.data_ptr(),
                                  _stream(stream)), "aqc_unpack_codes")
    return out


def aqc_dequant_f32(packed, N: int, K: int, bits: int, levels, block: int = BLOCK, stream=None):
    import torch
    out = torch.empty((N, K), dtype=torch.float32, device=packed.device)
    _check(lib().aqc_dequant_f32(packed.data_ptr(), N, K, bits, block, _levels(levels, bits), out.data_ptr(),
                                 _stream(stream)), "aqc_dequant_f32")
    return out


# ---- HSIC sensitivity ----
def aq_rbf_gram(A, gamma: float, stream=None):
    """A: cuda float32 [K, d] -> the RBF kernel matrix, cuda float32 [K, K]."""
    import torch
    K, d = A.shape
    G = torch.empty((K, K), dtype=torch.float32, device=A.device)
    ws = torch.empty(max(K, 4), dtype=torch.float32, device=A.device)
    _check(lib().aq_rbf_gram(A.data_ptr(), K, d, A.stride(0), gamma, G.data_ptr(), ws.data_ptr(), ws.numel() * 4,
                             _stream(stream)), "aq_rbf_gram")
    return G


def aq_hsic_sensitivity(X, gamma_x: float, Z, gamma_z: float, Y, gamma_y: float, alpha: float, beta: float,
                        workspace=None, stream=None):
    """X, Z, Y: cuda float32 [K, d*] -> cuda float64 [3]: HSIC(X, Z), HSIC(Z, Y), -alpha HSIC(X, Z) + beta HSIC(Z, Y)."""
    import torch
    K = X.shape[0]
    size = int(lib().aq_hsic_workspace_size(K))
    if workspace is None:
        workspace = torch.empty(max(size, 16), dtype=torch.uint8, device=X.device)
    out = torch.empty(3, dtype=torch.float64, device=X.device)
    _check(lib().aq_hsic_sensitivity(X.data_ptr(), X.shape[1], X.stride(0), gamma_x, Z.data_ptr(), Z.shape[1], Z.stride(0),
                                     gamma_z, Y.data_ptr(), Y.shape[1], Y.stride(0), gamma_y, K, alpha, beta,
                                     out.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream(stream)),
           "aq_hsic_sensitivity")
    return out
