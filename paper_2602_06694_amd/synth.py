"""Seeded synthetic inputs shaped like the paper's Llama-2 workloads.

This module only *draws data*: random sign words, positive fp16 scales and
normally distributed activations rounded to the storage type.  It performs
none of the method's arithmetic (no scaling, no contraction, no packing of
+-1 values) so that the CPU oracle and the HIP library can both be fed from
it without sharing any computation.

Layer shapes follow the quantization scheme of the paper (Section 3.1,
Eq. 1: two binary factors of rank r plus an input and an output scale
vector) applied to the linear layers of Llama-2-7B / Llama-2-70B decoder
blocks (q, k, v, o, gate, up, down).
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Iterator, List, Tuple

import numpy as np

# tensor ids inside one linear layer (used to derive independent streams)
T_U, T_V, T_S_OUT, T_S_IN, T_X = 0, 1, 2, 3, 4

LINEAR_NAMES = ("q", "k", "v", "o", "gate", "up", "down")


def seed_for(cfg: int, layer: int, linear_idx: int, tensor_id: int) -> int:
    """One independent PCG64 stream per (config, layer, linear, tensor)."""
    return 1_000_003 * cfg + 7919 * layer + 101 * linear_idx + tensor_id


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(seed))


def words_per_row(cols: int) -> int:
    return (cols + 31) // 32


def gen_sign_words(rows: int, cols: int, seed: int) -> np.ndarray:
    """I.i.d. uniform +-1 signs, drawn directly as packed words.

    Returns uint32 [rows, ceil(cols/32)], row-major, bit (k mod 32) of word
    k//32 (LSB first) is the sign bit of column k (1 -> +1, 0 -> -1, the
    polarity of Fig. 2(c)); bits beyond `cols` in the last word are 0.
    Uniform random words are the same distribution as packing i.i.d. signs.
    """
    wpr = words_per_row(cols)
    w = _rng(seed).integers(0, 2**32, size=(rows, wpr), dtype=np.uint64).astype(np.uint32)
    tail = cols % 32
    if tail:
        w[:, -1] &= np.uint32((1 << tail) - 1)
    return np.ascontiguousarray(w)


def gen_signs_pm1(rows: int, cols: int, seed: int) -> np.ndarray:
    """I.i.d. uniform +-1 signs as int8 [rows, cols] (small shapes only)."""
    b = _rng(seed).integers(0, 2, size=(rows, cols), dtype=np.int8)
    return (2 * b - 1).astype(np.int8)


def gen_scales(n: int, seed: int) -> np.ndarray:
    """fp16 scale vector |N(0,1)| + 0.1 (scales are means of magnitudes in
    the paper's initialisation, Section 3.3 Step 2, hence strictly positive)."""
    v = np.abs(_rng(seed).standard_normal(n)) + 0.1
    return v.astype(np.float16)


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16, returned as uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32).astype(np.uint64)
    bias = 0x7FFF + ((u >> 16) & 1)
    return ((u + bias) >> 16).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << 16).view(np.float32)


def gen_x(batch: int, d_in: int, seed: int, dtype: str = "bf16", outlier_frac: float = 0.0,
          outlier_gain: float = 20.0) -> np.ndarray:
    """Activations ~ N(0,1), optionally with a fixed random fraction of input
    channels multiplied by `outlier_gain` (same channels for every token),
    rounded to the storage type.

    dtype "f32" -> float32 array; "f16" -> float16 array;
    "bf16" -> uint16 array holding bfloat16 bit patterns.
    """
    g = _rng(seed)
    x = g.standard_normal((batch, d_in)).astype(np.float32)
    if outlier_frac > 0.0:
        n_out = int(d_in * outlier_frac)
        ch = g.choice(d_in, size=n_out, replace=False)
        x[:, ch] *= np.float32(outlier_gain)
    if dtype == "f32":
        return x
    if dtype == "f16":
        return x.astype(np.float16)
    if dtype == "bf16":
        return f32_to_bf16_bits(x)
    raise ValueError(f"unknown dtype {dtype}")


def x_as_f64(x: np.ndarray, dtype: str) -> np.ndarray:
    """Exact widening of a stored activation array to float64."""
    if dtype == "bf16":
        return bf16_bits_to_f32(x).astype(np.float64)
    return x.astype(np.float64)


@dataclass(frozen=True)
class LinearShape:
    name: str
    d_out: int
    d_in: int
    r: int

    @property
    def weight_bits(self) -> int:
        # storage of the factorization, Appendix F.5: r(n+m) + 16(n+m)
        return self.r * (self.d_out + self.d_in) + 16 * (self.d_out + self.d_in)

    @property
    def weight_bytes(self) -> int:
        return self.weight_bits // 8

    @property
    def bpw(self) -> float:
        return self.weight_bits / (self.d_out * self.d_in)


def llama2_7b_block() -> List[LinearShape]:
    att = [LinearShape(n, 4096, 4096, 1024) for n in ("q", "k", "v", "o")]
    mlp = [LinearShape("gate", 11008, 4096, 1664), LinearShape("up", 11008, 4096, 1664),
           LinearShape("down", 4096, 11008, 1664)]
    return att + mlp


def llama2_70b_block() -> List[LinearShape]:
    return [LinearShape("q", 8192, 8192, 2240), LinearShape("k", 1024, 8192, 512),
            LinearShape("v", 1024, 8192, 512), LinearShape("o", 8192, 8192, 2240),
            LinearShape("gate", 28672, 8192, 3520), LinearShape("up", 28672, 8192, 3520),
            LinearShape("down", 8192, 28672, 3520)]


@dataclass(frozen=True)
class Config:
    cfg: int
    name: str
    n_layers: int
    block: Tuple[LinearShape, ...]
    x_dtype: str
    batches: Tuple[int, ...]
    outlier_frac: float = 0.0


CONFIGS = {
    1: Config(1, "single-1024x1024-r256", 1, (LinearShape("lin", 1024, 1024, 256),), "f32", (1,)),
    2: Config(2, "llama2-7b-attn-4096x4096-r1024", 1, (LinearShape("q", 4096, 4096, 1024),), "bf16", (1, 8)),
    3: Config(3, "llama2-7b-stack-32x7", 32, tuple(llama2_7b_block()), "bf16", (1,)),
    4: Config(4, "llama2-70b-stack-80x7", 80, tuple(llama2_70b_block()), "bf16", (1,)),
    5: Config(5, "llama2-70b-mlp-prefill", 1,
              (LinearShape("gate", 28672, 8192, 3520), LinearShape("down", 8192, 28672, 3520)),
              "bf16", (512, 2048), outlier_frac=0.01),
}


@dataclass
class LayerData:
    shape: LinearShape
    U_words: np.ndarray   # uint32 [d_out, ceil(r/32)]
    V_words: np.ndarray   # uint32 [d_in,  ceil(r/32)]
    s_out: np.ndarray     # float16 [d_out]
    s_in: np.ndarray      # float16 [d_in]


def gen_layer(cfg: int, layer: int, linear_idx: int, shape: LinearShape) -> LayerData:
    return LayerData(
        shape,
        gen_sign_words(shape.d_out, shape.r, seed_for(cfg, layer, linear_idx, T_U)),
        gen_sign_words(shape.d_in, shape.r, seed_for(cfg, layer, linear_idx, T_V)),
        gen_scales(shape.d_out, seed_for(cfg, layer, linear_idx, T_S_OUT)),
        gen_scales(shape.d_in, seed_for(cfg, layer, linear_idx, T_S_IN)),
    )


def gen_layer_x(cfg: int, layer: int, linear_idx: int, shape: LinearShape, batch: int,
                dtype: str, outlier_frac: float = 0.0) -> np.ndarray:
    return gen_x(batch, shape.d_in, seed_for(cfg, layer, linear_idx, T_X), dtype, outlier_frac)


def iter_config_layers(cfg: int, max_layers: int | None = None) -> Iterator[Tuple[int, int, LinearShape]]:
    c = CONFIGS[cfg]
    n = c.n_layers if max_layers is None else min(c.n_layers, max_layers)
    for layer in range(n):
        for li, shp in enumerate(c.block):
            yield layer, li, shp


# ---- a decoder stack whose layers feed one another --------------------------------------------
# The seven projections of a block in the order a decoder calls them, as levels of mutually
# independent layers, and which layer's output each one reads when the stack is run as a chain
# (the attention, normalisation and activation kernels that sit in between in a real model are
# not part of this path): o reads q's output, gate and up read o's, down reads gate's, and the q, k,
# v of the next block read down's.
BLOCK_LEVEL = (0, 0, 0, 1, 2, 2, 3)
BLOCK_SOURCE = (-1, -1, -1, 0, 3, 3, 4)       # index inside the block; -1: the previous block's down (or the stack's input)


def chain_spec(n_blocks: int):
    """(level, source) of every layer of n_blocks chained blocks; source -1 = the stack's input."""
    level, src = [], []
    for b in range(n_blocks):
        for li in range(7):
            level.append(4 * b + BLOCK_LEVEL[li])
            src.append(7 * b + BLOCK_SOURCE[li] if BLOCK_SOURCE[li] >= 0 else (7 * b - 1 if b else -1))
    return level, src


def gen_chained_stack(cfg: int, n_blocks: int | None = None) -> List[LayerData]:
    """The layers of config 3 / 4 with their scale vectors multiplied by powers of two (exact in fp16)
    such that activations keep a magnitude near one along the chain q -> o -> gate -> down -> q ...:
    a layer with i.i.d. signs multiplies the rms of its input by about 1.17 sqrt(r d_in), which a real
    model's normalisation layers would absorb.  Only the data changes; the operator is the same."""
    import math
    c = CONFIGS[cfg]
    n_blocks = c.n_layers if n_blocks is None else n_blocks
    out: List[LayerData] = []
    carry = {}                                   # log2 of the rms at each layer's output, relative to the stack's input
    _, src = chain_spec(n_blocks)
    for b in range(n_blocks):
        for li, shp in enumerate(c.block):
            i = 7 * b + li
            d = gen_layer(cfg, b, li, shp)
            at_input = carry[src[i]] if src[i] >= 0 else 0.0
            gain = math.log2(1.17 * math.sqrt(shp.r * shp.d_in))
            k = int(round(at_input + gain))      # bring the output back to about one
            k = max(0, min(k, 18))               # (the scales stay normal fp16 numbers: 0.1 * 2^-9 > 6.1e-5)
            k_in = k // 2
            s_in = (d.s_in.astype(np.float32) * np.float32(2.0 ** -k_in)).astype(np.float16)
            s_out = (d.s_out.astype(np.float32) * np.float32(2.0 ** -(k - k_in))).astype(np.float16)
            carry[i] = at_input + gain - k
            out.append(LayerData(shp, d.U_words, d.V_words, s_out, s_in))
    return out


def gen_admm_problem(n: int, m: int, r: int, seed: int) -> Tuple[np.ndarray, np.ndarray, np.ndarray]:
    """Inputs of the latent-binary factorisation of one matrix (no arithmetic of the method here): a target
    W [n, m] shaped like a trained weight matrix (a decaying low-rank part plus dense noise, standard deviation
    about 0.02) and start factors U0 [n, r], V0 [m, r] (i.i.d. normal, scaled so that U0 V0^T has W's scale)."""
    g = _rng(seed)
    k = max(1, min(n, m) // 8)
    decay = 1.0 / np.sqrt(1.0 + np.arange(k))
    low = (g.standard_normal((n, k)) * decay) @ g.standard_normal((k, m))
    w = 0.02 * (0.7 * low / np.sqrt((decay ** 2).sum()) + 0.7 * g.standard_normal((n, m)))
    s = np.sqrt(0.02 / np.sqrt(r))
    u0 = s * g.standard_normal((n, r))
    v0 = s * g.standard_normal((m, r))
    return w, u0, v0
