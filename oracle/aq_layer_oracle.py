"""CPU oracle for one decode step through a stack of transformer blocks whose seven projection matrices
are block-quantised (TEST INFRASTRUCTURE, not product code; parity pinned by tests/test_layer_oracle_pins.py).

Plain numpy in float64, one operation after the other, nothing fused or reordered.  Shares nothing with the
library: the weights come from this package's own unpack + dequantise (Eq. 1).

What it follows: Section 3 ("Vision-Language-Action models") names the matrices of a block: the attention
projections W_Q, W_K, W_V, W_O and the MLP matrices W_gate, W_up, W_down.  The paper's backbone is LLaMA-2-7B (and a
Gemma-2B-sized one for the second model); what sits between the matrices is those published architectures':

    h   = rmsnorm(x; g_attn)           rmsnorm(x; g)_i = x_i / sqrt(mean_j x_j^2 + eps) * g_i
    q, k, v = W_Q h, W_K h, W_V h
    a   = attention(q, k, v)           softmax(q_h . k_h' / sqrt(head_dim)) over the keys seen so far, times v
    x   = x + W_O a
    h2  = rmsnorm(x; g_mlp)
    x   = x + W_down (act(W_gate h2) * W_up h2)       act = SiLU (LLaMA) or tanh-GELU (Gemma)

Readings (the paper gives no equations for the block):
  - the step is the FIRST token of a sequence: the only key a query sees is its own, so attention is written out
    over that one key (the softmax weight is exp(0)/exp(0) = 1).  Query head h reads key/value head
    h // (n_heads / n_kv_heads).  Rotary position embedding turns q and k of one position by the same angle and
    leaves their product unchanged; q, k, v are returned as the plain projections (what a key/value cache keeps,
    before any rotation).
  - g is the multiplier itself (a Gemma checkpoint stores g - 1).
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import List, Sequence, Tuple

import numpy as np

from . import aq_oracle as ao

MATRICES = ("q", "k", "v", "o", "gate", "up", "down")


@dataclass(frozen=True)
class Shape:
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    act: str = "silu"        # "silu" or "gelu_tanh"
    eps: float = 1e-5

    def matrix_shape(self, name: str) -> Tuple[int, int]:
        dq, dkv = self.n_heads * self.head_dim, self.n_kv_heads * self.head_dim
        return {"q": (dq, self.d_model), "k": (dkv, self.d_model), "v": (dkv, self.d_model),
                "o": (self.d_model, dq), "gate": (self.d_ff, self.d_model), "up": (self.d_ff, self.d_model),
                "down": (self.d_model, self.d_ff)}[name]


def rmsnorm(x: np.ndarray, g: np.ndarray, eps: float) -> np.ndarray:
    x = np.asarray(x, dtype=np.float64)
    mean_sq = float(np.sum(x * x)) / x.size
    return x / math.sqrt(mean_sq + eps) * np.asarray(g, dtype=np.float64)


def silu(a: np.ndarray) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64)
    return a / (1.0 + np.exp(-a))


def gelu_tanh(a: np.ndarray) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64)
    return 0.5 * a * (1.0 + np.tanh(math.sqrt(2.0 / math.pi) * (a + 0.044715 * a ** 3)))


def activation(name: str, a: np.ndarray) -> np.ndarray:
    if name == "silu":
        return silu(a)
    if name == "gelu_tanh":
        return gelu_tanh(a)
    raise ValueError(name)


def attention_first_token(q: np.ndarray, k: np.ndarray, v: np.ndarray, shape: Shape) -> np.ndarray:
    """Attention of one query position over the single key/value position it can see (its own)."""
    hd = shape.head_dim
    rep = shape.n_heads // shape.n_kv_heads
    out = np.empty(shape.n_heads * hd, dtype=np.float64)
    for h in range(shape.n_heads):
        kv = h // rep
        qh = q[h * hd:(h + 1) * hd]
        kh = k[kv * hd:(kv + 1) * hd]
        vh = v[kv * hd:(kv + 1) * hd]
        scores = np.array([float(qh @ kh) / math.sqrt(hd)])      # one key
        wts = np.exp(scores - scores.max())
        wts = wts / wts.sum()
        out[h * hd:(h + 1) * hd] = wts[0] * vh
    return out


def dequantised(layer: dict, name: str, shape: Shape) -> np.ndarray:
    """float64 W[N, K] of one matrix of a layer: layer[name] = (code bitstream, fp16 scale bits, bits)."""
    stream, scales, bits = layer[name]
    N, K = shape.matrix_shape(name)
    return ao.dequant(stream, scales, N, K, bits).reshape(N, K)


def decode_step(x: np.ndarray, layers: Sequence[dict], shape: Shape):
    """x float64[d_model] through every layer in turn.

    layers[l] = {"q": (stream, scales, bits), ..., "down": (...), "norm_attn": g, "norm_mlp": g}.
    Returns (x_out, qkv) with qkv[l] = (q, k, v) of layer l."""
    x = np.asarray(x, dtype=np.float64).copy()
    qkv: List[Tuple[np.ndarray, np.ndarray, np.ndarray]] = []
    for layer in layers:
        h = rmsnorm(x, layer["norm_attn"], shape.eps)
        q = dequantised(layer, "q", shape) @ h
        k = dequantised(layer, "k", shape) @ h
        v = dequantised(layer, "v", shape) @ h
        a = attention_first_token(q, k, v, shape)
        x = x + dequantised(layer, "o", shape) @ a
        h2 = rmsnorm(x, layer["norm_mlp"], shape.eps)
        gate = dequantised(layer, "gate", shape) @ h2
        up = dequantised(layer, "up", shape) @ h2
        x = x + dequantised(layer, "down", shape) @ (activation(shape.act, gate) * up)
        qkv.append((q, k, v))
    return x, qkv
