"""Pins of the layer-step oracle (oracle/aq_layer_oracle.py) against things other than itself: a hand-worked
block, torch's own rms_norm / silu / gelu / scaled_dot_product_attention / linear in float64, closed forms and
invariants.  No GPU."""
import math
import os

import numpy as np
import pytest
import torch

import aq_workloads as wl
from oracle import aq_layer_oracle as lo
from oracle import aq_oracle as ao

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "layer_step_example.txt")


def quantised(W: np.ndarray, d: float, bits: int = 2):
    """(stream, scales, bits) whose dequantised matrix is W, for W / d integer in the code range."""
    z = 1 << (bits - 1)
    q = np.rint(W / d).astype(np.int64) + z
    assert q.min() >= 0 and q.max() < (1 << bits)
    N, K = W.shape
    scales = np.full((N, K // 32), wl.f32_to_f16_bits(np.array([d], dtype=np.float32))[0], dtype=np.uint16)
    return ao.pack(q.astype(np.uint8), bits), scales, bits


def hand_block():
    n = 32
    shift = np.zeros((n, n)); shift[np.arange(n), (np.arange(n) + 1) % n] = 1.0
    eye = np.eye(n)
    layer = {"q": quantised(shift, 1.0), "k": quantised(shift, 1.0), "v": quantised(shift, 1.0),
             "o": quantised(0.5 * eye, 0.5), "gate": quantised(eye, 1.0), "up": quantised(-2.0 * eye, 1.0),
             "down": quantised(eye, 1.0), "norm_attn": np.ones(n), "norm_mlp": np.ones(n)}
    return layer, lo.Shape(32, 1, 1, 32, 32, "silu", 0.0)


def test_hand_worked_block():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    table = {int(r[0]): [float(v) for v in r[1:]] for r in rows}
    layer, shape = hand_block()
    x = np.array([table[i % 4][0] for i in range(32)])
    x2, qkv = lo.decode_step(x, [layer], shape)
    q, k, v = qkv[0]
    for i in range(32):
        _, v_exp, x1_exp, x2_exp = table[i % 4]
        assert v[i] == v_exp and q[i] == v_exp and k[i] == v_exp
        assert abs(x2[i] - x2_exp) < 5e-10
    # the intermediate column: the block with W_down = 0 stops after the attention half
    layer0 = dict(layer); layer0["down"] = quantised(np.zeros((32, 32)), 1.0)
    x1, _ = lo.decode_step(x, [layer0], shape)
    assert np.array_equal(x1, np.array([table[i % 4][2] for i in range(32)]))


def test_elementwise_pieces_against_torch():
    g = np.random.default_rng(1)
    x = g.standard_normal(96) * 3.0
    w = 1.0 + 0.2 * g.standard_normal(96)
    tx, tw = torch.tensor(x), torch.tensor(w)
    ref = torch.nn.functional.rms_norm(tx, (96,), tw, eps=1e-5).numpy()
    assert np.allclose(lo.rmsnorm(x, w, 1e-5), ref, rtol=1e-13, atol=0)
    assert np.allclose(lo.silu(x), torch.nn.functional.silu(tx).numpy(), rtol=1e-13, atol=1e-300)
    assert np.allclose(lo.gelu_tanh(x), torch.nn.functional.gelu(tx, approximate="tanh").numpy(), rtol=1e-12, atol=1e-15)


def test_closed_forms():
    assert lo.silu(np.array([0.0]))[0] == 0.0
    assert abs(lo.silu(np.array([math.log(3.0)]))[0] - 0.75 * math.log(3.0)) < 1e-15      # sigmoid(ln 3) = 3/4
    assert abs(lo.silu(np.array([-math.log(3.0)]))[0] + 0.25 * math.log(3.0)) < 1e-15
    assert lo.gelu_tanh(np.array([0.0]))[0] == 0.0
    big = lo.gelu_tanh(np.array([10.0, -10.0]))
    assert abs(big[0] - 10.0) < 1e-12 and abs(big[1]) < 1e-12
    # constant vector: rms = |c|, so the norm returns sign(c) * g
    g = np.linspace(0.5, 1.5, 64)
    assert np.allclose(lo.rmsnorm(np.full(64, -3.0), g, 0.0), -g, rtol=1e-15)
    # eps enters under the root, next to the MEAN of squares
    assert abs(lo.rmsnorm(np.array([3.0, 4.0]), np.ones(2), 3.5)[0] - 3.0 / 4.0) < 1e-15   # mean sq 12.5 + 3.5 = 16


def torch_block(x, Ws, g1, g2, shape):
    """The same block from torch's own building blocks, float64, sequence length one."""
    F = torch.nn.functional
    x = torch.tensor(x)
    W = {n: torch.tensor(w) for n, w in Ws.items()}
    h = F.rms_norm(x, (shape.d_model,), torch.tensor(g1), eps=shape.eps)
    q, k, v = F.linear(h, W["q"]), F.linear(h, W["k"]), F.linear(h, W["v"])
    hd, rep = shape.head_dim, shape.n_heads // shape.n_kv_heads
    q4 = q.view(1, shape.n_heads, 1, hd)
    k4 = k.view(1, shape.n_kv_heads, 1, hd).repeat_interleave(rep, dim=1)
    v4 = v.view(1, shape.n_kv_heads, 1, hd).repeat_interleave(rep, dim=1)
    a = F.scaled_dot_product_attention(q4, k4, v4).reshape(-1)
    x = x + F.linear(a, W["o"])
    h2 = F.rms_norm(x, (shape.d_model,), torch.tensor(g2), eps=shape.eps)
    gate, up = F.linear(h2, W["gate"]), F.linear(h2, W["up"])
    act = F.silu(gate) if shape.act == "silu" else F.gelu(gate, approximate="tanh")
    x = x + F.linear(act * up, W["down"])
    return x.numpy(), q.numpy(), k.numpy(), v.numpy()


@pytest.mark.parametrize("act,heads,kv", [("silu", 4, 4), ("silu", 4, 2), ("gelu_tanh", 4, 1)])
def test_stack_against_torch_building_blocks(act, heads, kv):
    shape = lo.Shape(128, heads, kv, 32, 160, act, 1e-5)
    wshape = wl.BlockShape(128, heads, kv, 32, 160, act, 1e-5)
    layers = wl.draw_block_stack(wshape, [[2, 3, 4, 3, 4, 2, 3], [4, 2, 3, 2, 3, 4, 2]], 77, heads, kv)
    x0 = wl.draw_residual(128, 77).astype(np.float64)
    x_or, qkv = lo.decode_step(x0, layers, shape)
    x = x0
    for l, layer in enumerate(layers):
        Ws = {}
        for name in lo.MATRICES:
            stream, scales, bits = layer[name]
            N, K = shape.matrix_shape(name)
            codes = ao.unpack(stream, N, K, bits).astype(np.float64)          # Eq. 1 retyped with numpy
            d = wl.f16_bits_to_f32(scales).astype(np.float64)
            Ws[name] = np.repeat(d, 32, axis=1) * (codes - (1 << (bits - 1)))
        x, q, k, v = torch_block(x, Ws, layer["norm_attn"].astype(np.float64), layer["norm_mlp"].astype(np.float64), shape)
        for got, ref in zip(qkv[l], (q, k, v)):
            assert ao.rel_l2(got, ref) < 1e-13
    assert ao.rel_l2(x_or, x) < 1e-13


def test_grouped_heads_read_their_own_value_head():
    # 4 query heads over 2 key/value heads: heads 0,1 read value head 0; heads 2,3 read value head 1
    shape = lo.Shape(64, 4, 2, 16, 64)
    v = np.arange(32, dtype=np.float64)
    q = np.ones(64); k = np.ones(32)
    a = lo.attention_first_token(q, k, v, shape)
    assert np.array_equal(a, np.concatenate([v[:16], v[:16], v[16:], v[16:]]))


def test_invariants():
    wshape = wl.BlockShape(64, 2, 1, 32, 96, "silu", 0.0)
    shape = lo.Shape(64, 2, 1, 32, 96, "silu", 0.0)
    layers = wl.draw_block_stack(wshape, [[3, 3, 3, 3, 3, 3, 3]], 5)
    x0 = wl.draw_residual(64, 5).astype(np.float64)
    # eps = 0: the first norm removes the scale of x, so q, k, v and what the attention half ADDS do not depend
    # on it (the MLP half then sees 8 x + delta, not 8 (x + delta): only the first half is invariant)
    N, K = shape.matrix_shape("down")
    half = dict(layers[0]); half["down"] = quantised(np.zeros((N, K)), 1.0, 3)
    x1, qkv1 = lo.decode_step(x0, [half], shape)
    x2, qkv2 = lo.decode_step(8.0 * x0, [half], shape)
    assert ao.rel_l2(x2 - 8.0 * x0, x1 - x0) < 1e-12
    for a, b in zip(qkv2[0], qkv1[0]):
        assert ao.rel_l2(a, b) < 1e-13
    # zero output projections: the residual stream passes through untouched
    mute = dict(layers[0])
    for name in ("o", "down"):
        N, K = shape.matrix_shape(name)
        mute[name] = quantised(np.zeros((N, K)), 1.0, 3)
    x3, _ = lo.decode_step(x0, [mute], shape)
    assert np.array_equal(x3, x0)
    # layers compose: two layers = one after the other
    two = wl.draw_block_stack(wshape, [[2] * 7, [4] * 7], 6)
    xa, _ = lo.decode_step(x0, two[:1], shape)
    xb, _ = lo.decode_step(xa, two[1:], shape)
    xc, _ = lo.decode_step(x0, two, shape)
    assert np.array_equal(xb, xc)
