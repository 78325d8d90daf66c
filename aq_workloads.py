"""Seeded synthetic inputs for the block-quantised matmul workloads.

This module only draws random numbers and lists shapes.  It holds none of the
method's arithmetic (no unpacking, no dequantisation, no matmul): the CPU
oracle and the HIP library both receive exactly the arrays produced here and
each does its own work on them.

Interchange ("canonical") form of one quantised matrix W[N, K] with bit-width
b and blocks of 32 along K (the block format of Eq. 1, Section 3):

  codes  : uint8 [N, K/32, 4*b]  -- per block a little-endian bitstream of
           32 b-bit codes.  Codes are iid uniform on {0..2^b-1}, so the
           bitstream is simply iid uniform bytes and is drawn as such.
  scales : uint16 [N, K/32]      -- fp16 bit patterns of d = fp16(|g| * 0.02),
           g ~ N(0, 1) drawn in fp32.

Activations are N(0, 1) drawn in fp32 and rounded (nearest-even) to fp16 or
bf16; they are carried as uint16 bit patterns so numpy needs no bf16 type.

The shapes stand in for the LLaMA-2-7B backbone of OpenVLA-OFT and for a
Gemma-2B-shaped backbone; no real checkpoint or benchmark item is used.
"""
from __future__ import annotations

import dataclasses
from typing import Iterator, List, Sequence, Tuple

import numpy as np

BLOCK = 32
BASE_SEED = 0

# (name, N, K) of the seven matrices of one transformer layer, in layer order.
LLAMA2_7B_LAYER: Tuple[Tuple[str, int, int], ...] = (
    ("q", 4096, 4096),
    ("k", 4096, 4096),
    ("v", 4096, 4096),
    ("o", 4096, 4096),
    ("gate", 11008, 4096),
    ("up", 11008, 4096),
    ("down", 4096, 11008),
)
LLAMA2_7B_LAYERS = 32

GEMMA_2B_LAYER: Tuple[Tuple[str, int, int], ...] = (
    ("q", 2048, 2048),
    ("k", 256, 2048),
    ("v", 256, 2048),
    ("o", 2048, 2048),
    ("gate", 16384, 2048),
    ("up", 16384, 2048),
    ("down", 2048, 16384),
)
GEMMA_2B_LAYERS = 18

PREFILL_M = 300          # 256 image-patch rows followed by 44 text rows
PREFILL_IMAGE_ROWS = 256
PREFILL_IMAGE_GAIN = 3.0


@dataclasses.dataclass(frozen=True)
class MatrixSpec:
    """One matrix of a backbone-shaped stream."""
    index: int      # position in the stream
    layer: int
    name: str
    N: int
    K: int
    bits: int

    @property
    def weights(self) -> int:
        return self.N * self.K


def _rng(*key: int) -> np.random.Generator:
    """Counter-based generator keyed by a tuple of small integers."""
    ss = np.random.SeedSequence([int(k) & 0xFFFFFFFF for k in key])
    return np.random.Generator(np.random.Philox(ss))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to bf16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32).astype(np.uint64)
    u = (u + 0x7FFF + ((u >> 16) & 1)) >> 16
    return u.astype(np.uint16)


def f32_to_f16_bits(a: np.ndarray) -> np.ndarray:
    """Round fp32 values to fp16 (nearest-even, numpy's cast); returns uint16 bit patterns."""
    return np.ascontiguousarray(a, dtype=np.float32).astype(np.float16).view(np.uint16)


def draw_weights(N: int, K: int, *key: int, sigma: float = 0.02, outlier_rate: float = 0.01) -> np.ndarray:
    """fp32 weights N(0, sigma^2) with a share `outlier_rate` of elements drawn 8 times wider (trained matrices
    have heavy tails; the optimiser's scale has to trade them against the bulk)."""
    g = _rng(606, *key)
    w = g.standard_normal((N, K)).astype(np.float32) * np.float32(sigma)
    wide = g.random((N, K)) < outlier_rate
    return np.where(wide, w * np.float32(8.0), w).astype(np.float32)


def draw_sensitivities(N: int, K: int, *key: int) -> np.ndarray:
    """Positive fp32 sensitivities: squared-gradient-like, gamma(0.5) times a per-row and a per-column factor
    (mean squared gradients vary by orders of magnitude across rows and input channels)."""
    g = _rng(707, *key)
    f = g.gamma(0.5, 2.0, size=(N, K))
    f *= np.exp(g.standard_normal((N, 1))) * np.exp(g.standard_normal((1, K)))
    return f.astype(np.float32)


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float32 values (exact)."""
    return (np.asarray(a, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def f16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    """binary16 bit patterns (uint16) -> float32 values (exact)."""
    return np.asarray(a, dtype=np.uint16).view(np.float16).astype(np.float32)


def draw_codes(N: int, K: int, bits: int, *key: int) -> np.ndarray:
    """Canonical code bitstream uint8[N, K/32, 4*bits] of iid uniform codes."""
    assert K % BLOCK == 0 and bits in (2, 3, 4)
    nb = K // BLOCK
    g = _rng(101, *key)
    n = N * nb * 4 * bits
    raw = g.integers(0, 0xFFFFFFFFFFFFFFFF, size=(n + 7) // 8, dtype=np.uint64, endpoint=True)
    return raw.view(np.uint8)[:n].reshape(N, nb, 4 * bits).copy()


def draw_scales(N: int, K: int, *key: int) -> np.ndarray:
    """fp16 bit patterns uint16[N, K/32] of d = fp16(|N(0,1)| * 0.02)."""
    nb = K // BLOCK
    g = _rng(202, *key)
    d = np.abs(g.standard_normal(size=(N, nb), dtype=np.float32)) * np.float32(0.02)
    return f32_to_f16_bits(d)


def draw_activations(M: int, K: int, dtype: str, *key: int,
                     image_rows: int = 0, image_gain: float = 1.0) -> np.ndarray:
    """Activations uint16[M, K] (bit patterns of `dtype`, "f16" or "bf16"), N(0,1);
    the first `image_rows` rows are multiplied by `image_gain` before rounding."""
    g = _rng(303, *key)
    x = g.standard_normal(size=(M, K), dtype=np.float32)
    if image_rows:
        x[:image_rows] *= np.float32(image_gain)
    if dtype == "f16":
        return f32_to_f16_bits(x)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(dtype)


def draw_matrix(N: int, K: int, bits: int, *key: int) -> Tuple[np.ndarray, np.ndarray]:
    return draw_codes(N, K, bits, *key), draw_scales(N, K, *key)


# ----------------------------------------------------------------------------
# exact-arithmetic inputs: integer activations and power-of-two scales, for
# which every fp32 summation order gives the same bits.
# ----------------------------------------------------------------------------
def draw_pow2_scales(N: int, K: int, *key: int) -> np.ndarray:
    """fp16 bit patterns of scales 2^e, e uniform in {-6..-1}."""
    nb = K // BLOCK
    g = _rng(404, *key)
    e = g.integers(-6, 0, size=(N, nb))
    return f32_to_f16_bits(np.ldexp(np.float32(1.0), e).astype(np.float32))


def draw_int_activations(M: int, K: int, dtype: str, *key: int) -> np.ndarray:
    """Integer-valued activations uniform in {-4..4}."""
    g = _rng(505, *key)
    x = g.integers(-4, 5, size=(M, K)).astype(np.float32)
    return f32_to_f16_bits(x) if dtype == "f16" else f32_to_bf16_bits(x)


# ----------------------------------------------------------------------------
# backbone-shaped streams and the seeded bit allocation
# ----------------------------------------------------------------------------
def layer_shapes(model: str) -> Tuple[Tuple[Tuple[str, int, int], ...], int]:
    if model == "llama2-7b":
        return LLAMA2_7B_LAYER, LLAMA2_7B_LAYERS
    if model == "gemma-2b":
        return GEMMA_2B_LAYER, GEMMA_2B_LAYERS
    raise ValueError(model)


def seeded_allocation(shapes: Sequence[Tuple[int, int]], mean_code_bits: float,
                      seed: int = BASE_SEED) -> List[int]:
    """One bit-width from {2,3,4} per matrix with an element-weighted mean of
    code bits not above `mean_code_bits`.

    Deterministic: every matrix starts at 2 bits; a seeded permutation is walked
    cyclically; at each matrix still below 4 bits a seeded step of +1 or +2
    (clamped to 4) is applied if the remaining bit budget allows it; the walk
    ends after a full pass without an upgrade.
    """
    g = _rng(606, seed)
    n = len(shapes)
    sizes = [int(a) * int(b) for a, b in shapes]
    total = sum(sizes)
    bits = [2] * n
    budget = int(round(mean_code_bits * total)) - 2 * total
    order = list(g.permutation(n))
    changed = True
    while changed:
        changed = False
        for i in order:
            if bits[i] >= 4:
                continue
            step = min(int(g.integers(1, 3)), 4 - bits[i])
            cost = step * sizes[i]
            if cost <= budget:
                bits[i] += step
                budget -= cost
                changed = True
    return bits


def backbone_stream(model: str, allocation: str = "mixed", seed: int = BASE_SEED,
                    layers: int | None = None) -> List[MatrixSpec]:
    """The matrices of a backbone-shaped stream in layer order.

    allocation:
      "b2" / "b3" / "b4" : uniform bit-width;
      "mixed"            : seeded {2,3,4} allocation whose element-weighted mean of
                           code bits is 2.5 (3.0 bits per weight stored, scales included);
      "floor"            : every matrix at 2 bits = 2.5 bits per weight stored.
    """
    shp, L = layer_shapes(model)
    if layers is not None:
        L = layers
    flat = [(l, nm, N, K) for l in range(L) for (nm, N, K) in shp]
    if allocation in ("b2", "b3", "b4"):
        bits = [int(allocation[1])] * len(flat)
    elif allocation == "floor":
        bits = [2] * len(flat)
    elif allocation == "mixed":
        bits = seeded_allocation([(N, K) for (_, _, N, K) in flat], 2.5, seed)
    else:
        raise ValueError(allocation)
    return [MatrixSpec(i, l, nm, N, K, b) for i, ((l, nm, N, K), b) in enumerate(zip(flat, bits))]


def draw_tensor_sensitivities(model: str, *key: int) -> np.ndarray:
    """Synthetic per-tensor sensitivities [L, 7] for a backbone-shaped stream: gamma(0.7) times a log-normal
    per-layer factor (a few tensors and a few layers stand out).  Stands in for the HSIC scores of Eq. 5, which need
    a model and calibration data."""
    shp, L = layer_shapes(model)
    g = _rng(808, *key)
    return g.gamma(0.7, 1.0, size=(L, len(shp))) * np.exp(0.5 * g.standard_normal((L, 1)))


def with_bits(stream: Sequence[MatrixSpec], bits: Sequence[int]) -> List[MatrixSpec]:
    """The same stream with the given per-matrix bit-widths (e.g. from an allocator)."""
    return [dataclasses.replace(m, bits=int(b)) for m, b in zip(stream, bits)]


def stored_bits_per_weight(stream: Sequence[MatrixSpec]) -> float:
    """Bits per weight of the canonical form, fp16 block scales included."""
    tot = sum(m.weights for m in stream)
    return sum(m.weights * (m.bits + 16.0 / BLOCK) for m in stream) / tot


def iter_stream_inputs(stream: Sequence[MatrixSpec], M: int, dtype: str, seed: int = BASE_SEED,
                       prefill_profile: bool = False
                       ) -> Iterator[Tuple[MatrixSpec, np.ndarray, np.ndarray, np.ndarray]]:
    """Yield (spec, codes, scales, activations) per matrix; activations are independent
    per matrix (the stream is a weight-matmul proxy, not a dependent forward pass)."""
    for m in stream:
        codes, scales = draw_matrix(m.N, m.K, m.bits, seed, 3, m.index)
        if prefill_profile:
            x = draw_activations(M, m.K, dtype, seed, 3, m.index,
                                 image_rows=min(PREFILL_IMAGE_ROWS, M), image_gain=PREFILL_IMAGE_GAIN)
        else:
            x = draw_activations(M, m.K, dtype, seed, 3, m.index)
        yield m, codes, scales, x


# ----------------------------------------------------------------------------
# the same distributions drawn on the GPU (torch's seeded Philox generator), for the
# bench, where drawing gigabytes on the host would hold the GPU idle.  Values differ
# from the numpy draws (another generator) but follow the same recipe; the bench
# copies what the oracle needs back to the host.
# ----------------------------------------------------------------------------
# calibration-shaped inputs for the HSIC sensitivity: K samples of input hidden states X, of a matrix's output
# hidden states Z (a random linear map of X plus noise: dependent on X), and of action labels Y (a random
# low-dimensional read-out of Z plus noise)
# ----------------------------------------------------------------------------
def draw_hsic_inputs(K: int, d_in: int, d_out: int, d_act: int, *key: int, noise: float = 0.5):
    g = _rng(505, *key)
    X = g.standard_normal(size=(K, d_in), dtype=np.float32)
    P = g.standard_normal(size=(d_in, d_out), dtype=np.float32) / np.float32(np.sqrt(d_in))
    Z = (X @ P + np.float32(noise) * g.standard_normal(size=(K, d_out), dtype=np.float32)).astype(np.float32)
    R = g.standard_normal(size=(d_out, d_act), dtype=np.float32) / np.float32(np.sqrt(d_out))
    Y = np.tanh(Z @ R + np.float32(noise) * g.standard_normal(size=(K, d_act), dtype=np.float32)).astype(np.float32)
    return X, Z, Y


# ----------------------------------------------------------------------------
# non-uniform codebook variant of the format: tables of 2^bits levels
def draw_levels(kind: str, bits: int, *key: int) -> np.ndarray:
    """float32 [2^bits].  'quantile': the standard normal's quantiles at (q + 1/2) / 2^bits (dense near zero, the shape
    of tables fitted to bell-shaped weights); 'random': seeded N(0, 1) draws in no order (with a repeated value);
    'dyadic': seeded multiples of 1/8 in [-5, 5] (exact arithmetic); 'signed_dyadic': such multiples in pairs +v, -v;
    'uniform': q - 2^(bits-1), the base format."""
    n = 1 << bits
    if kind == "quantile":
        from scipy.stats import norm
        return norm.ppf((np.arange(n) + 0.5) / n).astype(np.float32)
    if kind == "random":
        t = _rng(31, bits, *key).normal(size=n).astype(np.float32)
        t[n - 1] = t[0]
        return t
    if kind == "dyadic":
        return (_rng(32, bits, *key).integers(-40, 41, size=n) / 8.0).astype(np.float32)
    if kind == "uniform":
        return (np.arange(n) - n // 2).astype(np.float32)
    if kind == "signed_dyadic":                  # pairs +v, -v of multiples of 1/8 (one pair of zeros), in no order
        r = _rng(33, bits, *key)
        mags = (r.integers(1, 41, size=n // 2) / 8.0).astype(np.float32)
        mags[0] = 0.0
        return np.concatenate([mags, -mags])[r.permutation(n)].astype(np.float32)
    raise ValueError(kind)


# two-level variant of the format: 4-bit scale and offset codes per block, two fp16 numbers per super-block
# ----------------------------------------------------------------------------
def draw_affine_params(N: int, K: int, bits: int, *key: int) -> Tuple[np.ndarray, np.ndarray]:
    """(sub uint8[N, K/32], sup uint16[N, ceil(K/256), 2]): scale codes uniform on {1..15}, offset codes uniform
    on {0..15}, D = fp16(|N(0,1)| * 0.02 / 8), M = fp16(D * 2^(bits-1) * u), u uniform on [0.5, 1.5): the block's
    zero point s_b z_b / s_b scatters around the middle of the code range."""
    nb, ns = K // BLOCK, (K + 8 * BLOCK - 1) // (8 * BLOCK)
    g = _rng(404, *key)
    a = g.integers(1, 16, size=(N, nb), dtype=np.uint8)
    c = g.integers(0, 16, size=(N, nb), dtype=np.uint8)
    D = np.abs(g.standard_normal(size=(N, ns), dtype=np.float32)) * np.float32(0.02 / 8)
    M = D * np.float32(1 << (bits - 1)) * (0.5 + g.random(size=(N, ns), dtype=np.float32))
    sup = np.stack([f32_to_f16_bits(D), f32_to_f16_bits(M)], axis=2)
    return (a | (c << 4)).astype(np.uint8), sup


# ----------------------------------------------------------------------------
# transformer blocks for the layer-by-layer decode step: the seven matrices of a layer with scales sized so
# that a matrix maps a vector of unit rms to one of rms `gain` (sub-layer outputs stay a fraction of the
# residual stream, as in a trained model), norm multipliers near one, x ~ N(0,1)
# ----------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class BlockShape:
    d_model: int
    n_heads: int
    n_kv_heads: int
    head_dim: int
    d_ff: int
    act: str
    eps: float

    def matrix_shape(self, name: str) -> Tuple[int, int]:
        dq, dkv = self.n_heads * self.head_dim, self.n_kv_heads * self.head_dim
        return {"q": (dq, self.d_model), "k": (dkv, self.d_model), "v": (dkv, self.d_model),
                "o": (self.d_model, dq), "gate": (self.d_ff, self.d_model), "up": (self.d_ff, self.d_model),
                "down": (self.d_model, self.d_ff)}[name]


BLOCK_MATRICES = ("q", "k", "v", "o", "gate", "up", "down")
BLOCK_SHAPES = {
    "llama2-7b": BlockShape(4096, 32, 32, 128, 11008, "silu", 1e-5),
    "gemma-2b": BlockShape(2048, 8, 1, 256, 16384, "gelu_tanh", 1e-6),
}
BLOCK_GAIN = {"q": 1.0, "k": 1.0, "v": 1.0, "o": 0.3, "gate": 1.0, "up": 1.0, "down": 0.6}


def code_rms(bits: int) -> float:
    """Root mean square of (q - 2^(bits-1)) for q uniform over the 2^bits codes."""
    z = 1 << (bits - 1)
    return float(np.sqrt(np.mean([(q - z) ** 2 for q in range(1 << bits)])))


def draw_gain_scales(N: int, K: int, bits: int, gain: float, *key: int) -> np.ndarray:
    """fp16 bit patterns uint16[N, K/32] of d = fp16(N(0,1) * gain / (code_rms * sqrt(K))).  The sign is kept:
    the code grid {-z .. z-1} is not symmetric, and blocks whose scale is negative use its mirror image, so the
    weights have zero mean (uniform codes under positive scales would all lean to the negative side and the
    residual stream would drift along the all-ones direction)."""
    nb = K // BLOCK
    g = _rng(202, *key)
    d = g.standard_normal(size=(N, nb), dtype=np.float32) * np.float32(gain / (code_rms(bits) * np.sqrt(K)))
    return f32_to_f16_bits(d)


def draw_norm_weights(n: int, *key: int) -> np.ndarray:
    g = _rng(909, *key)
    return (1.0 + 0.1 * g.standard_normal(size=n, dtype=np.float32)).astype(np.float32)


def draw_residual(n: int, *key: int) -> np.ndarray:
    return _rng(910, *key).standard_normal(size=n, dtype=np.float32)


def draw_block_stack(shape: BlockShape, bits: Sequence[Sequence[int]], *key: int) -> List[dict]:
    """layers[l] = {name: (codes, scales, bits) for the seven matrices, "norm_attn": g, "norm_mlp": g};
    bits[l][j] is the bit-width of matrix j (order of BLOCK_MATRICES) of layer l."""
    layers = []
    for l, row in enumerate(bits):
        layer = {}
        for j, name in enumerate(BLOCK_MATRICES):
            N, K = shape.matrix_shape(name)
            b = int(row[j])
            layer[name] = (draw_codes(N, K, b, *key, l, j), draw_gain_scales(N, K, b, BLOCK_GAIN[name], *key, l, j), b)
        layer["norm_attn"] = draw_norm_weights(shape.d_model, *key, l, 0)
        layer["norm_mlp"] = draw_norm_weights(shape.d_model, *key, l, 1)
        layers.append(layer)
    return layers


def draw_gain_matrix_torch(N: int, K: int, bits: int, gain: float, device, *key: int):
    """Device-side draw of the same distribution as draw_codes + draw_gain_scales (other random numbers)."""
    import torch
    nb = K // BLOCK
    g = _torch_gen(device, 101, *key)
    codes = torch.randint(0, 256, (N, nb, 4 * bits), dtype=torch.uint8, device=device, generator=g)
    d = torch.randn((N, nb), dtype=torch.float32, device=device, generator=g)
    d.mul_(float(gain / (code_rms(bits) * np.sqrt(K))))
    return codes, d.to(torch.float16)


# ----------------------------------------------------------------------------
def _torch_gen(device, *key: int):
    import torch
    g = torch.Generator(device=device)
    seed = int(np.random.SeedSequence([int(k) & 0xFFFFFFFF for k in key]).generate_state(1, np.uint64)[0])
    g.manual_seed(seed & 0x7FFFFFFFFFFFFFFF)
    return g


def draw_matrix_torch(N: int, K: int, bits: int, device, *key: int):
    """(codes uint8 [N, K/32, 4*bits], scales float16 [N, K/32]) on `device`."""
    import torch
    nb = K // BLOCK
    g = _torch_gen(device, 101, *key)
    codes = torch.randint(0, 256, (N, nb, 4 * bits), dtype=torch.uint8, device=device, generator=g)
    d = torch.randn((N, nb), dtype=torch.float32, device=device, generator=g).abs_().mul_(0.02)
    return codes, d.to(torch.float16)


def draw_affine_params_torch(N: int, K: int, bits: int, device, *key: int):
    """Device-side draw of the same distribution as draw_affine_params (other random numbers):
    (sub uint8 [N, K/32], sup float16 [N, ceil(K/256), 2])."""
    import torch
    nb, ns = K // BLOCK, (K + 8 * BLOCK - 1) // (8 * BLOCK)
    g = _torch_gen(device, 404, *key)
    a = torch.randint(1, 16, (N, nb), dtype=torch.uint8, device=device, generator=g)
    c = torch.randint(0, 16, (N, nb), dtype=torch.uint8, device=device, generator=g)
    D = torch.randn((N, ns), dtype=torch.float32, device=device, generator=g).abs_().mul_(0.02 / 8)
    M = D * float(1 << (bits - 1)) * (0.5 + torch.rand((N, ns), dtype=torch.float32, device=device, generator=g))
    return a | (c << 4), torch.stack([D, M], dim=2).to(torch.float16).contiguous()


def draw_activations_torch(M: int, K: int, dtype: str, device, *key: int,
                           image_rows: int = 0, image_gain: float = 1.0):
    """Activations [M, K] of torch.float16 / torch.bfloat16 on `device`."""
    import torch
    g = _torch_gen(device, 303, *key)
    x = torch.randn((M, K), dtype=torch.float32, device=device, generator=g)
    if image_rows:
        x[:image_rows] *= image_gain
    return x.to(torch.float16 if dtype == "f16" else torch.bfloat16)
