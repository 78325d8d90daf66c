"""numpy front end of the CPU oracle (TEST INFRASTRUCTURE, not product code).

Loads oracle/liboracle.so (plain C, fp64; built by `build()` below with gcc) and
exposes its functions on numpy arrays.  Only tests, the smoke check and the
bench's cpu_baseline leg may import this.  It imports nothing from the GPU
package and the GPU package imports nothing from here.

Every function names the passage it follows; see aq_oracle.c for the readings.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from fractions import Fraction

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "aq_oracle.c")
_SRC_SCALE = os.path.join(_HERE, "aq_scale_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")
_lib = None

_i64 = ctypes.c_int64
_int = ctypes.c_int
_p = ctypes.c_void_p


def build(force: bool = False) -> str:
    """Compile the C oracle with gcc (OpenMP on the plain loops, nothing else)."""
    newest = max(os.path.getmtime(_SRC), os.path.getmtime(_SRC_SCALE))
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < newest:
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, _SRC_SCALE, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        lib.aqo_f16_to_f64.restype = ctypes.c_double
        lib.aqo_f16_to_f64.argtypes = [ctypes.c_uint16]
        lib.aqo_bf16_to_f64.restype = ctypes.c_double
        lib.aqo_bf16_to_f64.argtypes = [ctypes.c_uint16]
        lib.aqo_f16_array_to_f64.argtypes = [_p, _i64, _p]
        lib.aqo_bf16_array_to_f64.argtypes = [_p, _i64, _p]
        lib.aqo_unpack.argtypes = [_p, _i64, _i64, _int, _int, _p]
        lib.aqo_pack.argtypes = [_p, _i64, _i64, _int, _int, _p]
        lib.aqo_dequant.argtypes = [_p, _p, _i64, _i64, _int, _int, _p]
        lib.aqo_rtn_codes.argtypes = [_p, _i64, ctypes.c_double, ctypes.c_double, _int, _p]
        lib.aqo_matmul_nt.argtypes = [_p, _p, _i64, _i64, _i64, _p]
        lib.aqo_qmatmul.argtypes = [_p, _p, _i64, _i64, _int, _int, _p, _i64, _int, _p, _p, _p]
        lib.aqo_stored_bytes.restype = _i64
        lib.aqo_stored_bytes.argtypes = [_i64, _i64, _int, _int]
        lib.aqo_num_threads.restype = _int
        lib.aqs_f64_to_f16.restype = ctypes.c_uint16
        lib.aqs_f64_to_f16.argtypes = [ctypes.c_double]
        lib.aqs_optimize.argtypes = [_p, _p, _i64, _i64, _int, _int, _int, _p, _p, _p]
        _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(_p)


def _c(a, dtype) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=dtype)


def num_threads() -> int:
    return int(_load().aqo_num_threads())


# ---- conversions -----------------------------------------------------------
def f16_to_f64(bits: np.ndarray) -> np.ndarray:
    """IEEE binary16 bit patterns -> float64 (exact)."""
    b = _c(bits, np.uint16)
    out = np.empty(b.shape, dtype=np.float64)
    _load().aqo_f16_array_to_f64(_ptr(b), b.size, _ptr(out))
    return out


def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns -> float64 (exact)."""
    b = _c(bits, np.uint16)
    out = np.empty(b.shape, dtype=np.float64)
    _load().aqo_bf16_array_to_f64(_ptr(b), b.size, _ptr(out))
    return out


def activations_to_f64(bits: np.ndarray, dtype: str) -> np.ndarray:
    return f16_to_f64(bits) if dtype == "f16" else bf16_to_f64(bits)


# ---- Eq. 1 -----------------------------------------------------------------
def unpack(stream: np.ndarray, N: int, K: int, bits: int, block: int = 32) -> np.ndarray:
    """Canonical bitstream uint8[N, K/block, block*bits/8] -> codes uint8[N, K]."""
    s = _c(stream, np.uint8)
    assert s.size == N * (K // block) * (block * bits // 8)
    q = np.empty((N, K), dtype=np.uint8)
    _load().aqo_unpack(_ptr(s), N, K, bits, block, _ptr(q))
    return q


def pack(q: np.ndarray, bits: int, block: int = 32) -> np.ndarray:
    """Codes uint8[N, K] -> canonical bitstream (inverse of `unpack`)."""
    q = _c(q, np.uint8)
    N, K = q.shape
    s = np.empty((N, K // block, block * bits // 8), dtype=np.uint8)
    _load().aqo_pack(_ptr(q), N, K, bits, block, _ptr(s))
    return s


def dequant(stream: np.ndarray, scales: np.ndarray, N: int, K: int, bits: int,
            block: int = 32) -> np.ndarray:
    """w_hat = d (q - 2^(bits-1)) in float64, shape [N, K] (Eq. 1, left part)."""
    s = _c(stream, np.uint8)
    d = _c(scales, np.uint16)
    assert d.size == N * (K // block)
    W = np.empty((N, K), dtype=np.float64)
    _load().aqo_dequant(_ptr(s), _ptr(d), N, K, bits, block, _ptr(W))
    return W


def rtn_codes(w: np.ndarray, s: float, z: float, bits: int) -> np.ndarray:
    """q_i = argmin_q |w_i - s (q - z)| over {0..2^bits-1} (Eq. 1, right part)."""
    w = _c(w, np.float64).ravel()
    q = np.empty(w.size, dtype=np.uint8)
    _load().aqo_rtn_codes(_ptr(w), w.size, float(s), float(z), bits, _ptr(q))
    return q


def matmul_nt(X: np.ndarray, W: np.ndarray) -> np.ndarray:
    """Y[M, N] = X[M, K] W[N, K]^T in float64, ascending-k sums."""
    X = _c(X, np.float64)
    W = _c(W, np.float64)
    M, K = X.shape
    N, K2 = W.shape
    assert K == K2
    Y = np.empty((M, N), dtype=np.float64)
    _load().aqo_matmul_nt(_ptr(X), _ptr(W), M, N, K, _ptr(Y))
    return Y


def qmatmul(stream: np.ndarray, scales: np.ndarray, N: int, K: int, bits: int,
            X_bits: np.ndarray, x_dtype: str, block: int = 32) -> np.ndarray:
    """The whole path: unpack -> dequantise (fp64) -> matmul.  X_bits uint16[M, K]."""
    s = _c(stream, np.uint8)
    d = _c(scales, np.uint16)
    X = _c(X_bits, np.uint16)
    if X.ndim == 1:
        X = X[None, :]
    M = X.shape[0]
    assert X.shape[1] == K
    sw = np.empty(N * K, dtype=np.float64)
    sx = np.empty(M * K, dtype=np.float64)
    Y = np.empty((M, N), dtype=np.float64)
    _load().aqo_qmatmul(_ptr(s), _ptr(d), N, K, bits, block, _ptr(X), M,
                        1 if x_dtype == "bf16" else 0, _ptr(sw), _ptr(sx), _ptr(Y))
    return Y


def qmatmul_rows(stream: np.ndarray, scales: np.ndarray, rows, K: int, bits: int,
                 X_bits: np.ndarray, x_dtype: str, block: int = 32) -> np.ndarray:
    """Columns `rows` of Y only (row n of W depends on codes[n], scales[n] alone):
    lets full-size matrices be checked on a sample of outputs."""
    rows = np.asarray(rows, dtype=np.int64)
    nb = K // block
    s = _c(stream, np.uint8).reshape(-1, nb, block * bits // 8)[rows]
    d = _c(scales, np.uint16).reshape(-1, nb)[rows]
    return qmatmul(s, d, len(rows), K, bits, X_bits, x_dtype, block)


def rel_l2(Y, Y_ref) -> float:
    """||Y - Y_ref||_2 / ||Y_ref||_2 in float64 (the acceptance measure)."""
    a = np.asarray(Y, dtype=np.float64).ravel()
    b = np.asarray(Y_ref, dtype=np.float64).ravel()
    den = float(np.sqrt(np.sum(b * b)))
    num = float(np.sqrt(np.sum((a - b) ** 2)))
    return num / den if den > 0 else num


# ---- storage accounting ------------------------------------------------------
def stored_bytes(N: int, K: int, bits: int, block: int = 32) -> int:
    """Bytes of the canonical form: codes plus one fp16 scale per block."""
    return int(_load().aqo_stored_bytes(N, K, bits, block))


def bits_per_weight(bits: int, block: int = 32, scale_bits: int = 16) -> Fraction:
    """Stored bits per weight of one matrix: the code bits plus the block's scale
    spread over its elements."""
    return Fraction(bits) + Fraction(scale_bits, block)


def footprint_gb(fp16_gb: float, avg_bpw: float) -> float:
    """Footprint of a model whose fp16 size is `fp16_gb` when it is stored at
    `avg_bpw` bits per weight on average (Table 1's Mem. column against its
    'VLA BPW' column)."""
    return fp16_gb * avg_bpw / 16.0


# ---- block-level scale optimisation (Section 4.2, Eq. 10-11; see aq_scale_oracle.c) -------------
def f64_to_f16_bits(x: float) -> int:
    """binary16 bit pattern of a double, round to nearest even."""
    return int(_load().aqs_f64_to_f16(float(x)))


def scale_optimize(W: np.ndarray, F, bits: int, rounds: int, block: int = 32, trace: bool = False):
    """Alternating code assignment / closed-form scale of Eq. 11 on every block of W[N, K].

    W float32 [N, K]; F float32 [N, K] (the diagonal sensitivities of Eq. 10) or None for all ones.
    Returns (codes uint8 [N, K] in {0..2^bits-1}, scales uint16 [N, K/block] binary16 bits[, trace])."""
    W = _c(W, np.float32)
    N, K = W.shape
    assert K % block == 0
    Fc = None if F is None else _c(F, np.float32)
    codes = np.empty((N, K), dtype=np.uint8)
    scales = np.empty((N, K // block), dtype=np.uint16)
    tr = np.zeros((N * (K // block), 2 * rounds + 3), dtype=np.float64) if trace else None
    _load().aqs_optimize(_ptr(W), None if Fc is None else _ptr(Fc), N, K, bits, block, rounds,
                         _ptr(codes), _ptr(scales), None if tr is None else _ptr(tr))
    return (codes, scales, tr) if trace else (codes, scales)
