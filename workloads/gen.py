"""Seeded generators for decoder shapes, weights, hidden states and request-length mixes.

All tensors are returned as numpy ``uint16`` arrays holding bf16 bit patterns (the storage format
of the weights and activations on the wire), plus exact conversions to and from float32.  The five
named shapes are the seeded synthetic configurations of this build: a tiny 2-layer decoder and
7B-, 8B-GQA-, 13B- and 70B-shaped Llama-family decoders.  They stand in for the trained models and
request traces used in the paper's evaluation (section 6, "Evaluated traces and models"), which are
not available here.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


@dataclass(frozen=True)
class DecoderShape:
    name: str
    L: int          # decoder layers
    H: int          # hidden size
    Hq: int         # query heads
    Hkv: int        # key/value heads
    d: int          # head dim
    F: int          # SwiGLU FFN width
    eps: float = 1e-5
    rope_base: float = 10000.0
    seed: int = 0

    @property
    def n_qkv(self) -> int:
        return (self.Hq + 2 * self.Hkv) * self.d

    @property
    def params_per_layer(self) -> int:
        return self.H * self.d * (2 * self.Hq + 2 * self.Hkv) + 3 * self.H * self.F + 2 * self.H


CONFIGS = {
    "tiny": DecoderShape("tiny", L=2, H=256, Hq=4, Hkv=4, d=64, F=688, rope_base=10000.0, seed=0),
    "7b": DecoderShape("7b", L=32, H=4096, Hq=32, Hkv=32, d=128, F=11008, rope_base=10000.0, seed=1),
    "8b_gqa": DecoderShape("8b_gqa", L=32, H=4096, Hq=32, Hkv=8, d=128, F=14336, rope_base=500000.0, seed=2),
    "13b": DecoderShape("13b", L=40, H=5120, Hq=40, Hkv=40, d=128, F=13824, rope_base=10000.0, seed=3),
    "70b": DecoderShape("70b", L=80, H=8192, Hq=64, Hkv=8, d=128, F=28672, rope_base=500000.0, seed=4),
}

# Tensors of one decoder layer, in the order used everywhere in this build.  Projection matrices
# are stored [out_features, in_features] (row = one output feature).
TENSOR_ORDER = ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")
_TAG = {n: i for i, n in enumerate(TENSOR_ORDER)}
_TAG_HIDDEN = 100
_TAG_KV = 101
_TAG_LEN = 102


def tensor_shapes(s: DecoderShape) -> dict:
    return {
        "g1": (s.H,),
        "wq": (s.Hq * s.d, s.H),
        "wk": (s.Hkv * s.d, s.H),
        "wv": (s.Hkv * s.d, s.H),
        "wo": (s.H, s.Hq * s.d),
        "g2": (s.H,),
        "wg": (s.F, s.H),
        "wu": (s.F, s.H),
        "wd": (s.H, s.F),
    }


def bf16_bits_from_f32(x: np.ndarray) -> np.ndarray:
    """Round float32 to bf16 (round-to-nearest-even), returning the 16-bit patterns."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32)
    # NaN never occurs in the generated data; finite/inf values round correctly with this bias.
    bias = ((u >> 16) & 1) + np.uint32(0x7FFF)
    return ((u + bias) >> 16).astype(np.uint16)


def f32_from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << 16).view(np.float32)


def _normal_bits(rng: np.random.Generator, shape, scale: float, shift: float = 0.0) -> np.ndarray:
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.uint16)
    step = 1 << 24
    for o in range(0, n, step):        # bounded temporaries for the 70B-shaped layer
        m = min(step, n - o)
        v = rng.standard_normal(m, dtype=np.float32)
        v *= np.float32(scale)
        if shift:
            v += np.float32(shift)
        out[o:o + m] = bf16_bits_from_f32(v)
    return out.reshape(shape)


def layer_weights_bits(s: DecoderShape, layer: int) -> dict:
    """bf16 bit patterns of one layer's nine tensors.

    Projection matrices are N(0, 0.02^2).  The two RMSNorm gains are 1 + N(0, 0.02^2), so that a
    path that forgot to apply a gain would not match.
    """
    out = {}
    for name, shape in tensor_shapes(s).items():
        rng = np.random.default_rng([s.seed, _TAG[name], layer])
        if name in ("g1", "g2"):
            out[name] = _normal_bits(rng, shape, 0.02, 1.0)
        else:
            out[name] = _normal_bits(rng, shape, 0.02)
    return out


def hidden_bits(s: DecoderShape, T: int, step: int = 0, scale: float = 1.0) -> np.ndarray:
    """[T, H] hidden states, N(0, scale^2) rounded to bf16; `step` selects an independent draw.  The
    configurations use scale 1; tests of narrow shapes use a smaller one so that the layer's update is
    not small against the residual stream it is added to."""
    rng = np.random.default_rng([s.seed, _TAG_HIDDEN, step])
    return _normal_bits(rng, (T, s.H), scale)


def kv_prefill_bits(s: DecoderShape, layer: int, slot: int, length: int):
    """Pre-existing K and V of one (layer, sequence): two [length, Hkv, d] arrays, N(0,1) -> bf16."""
    rng = np.random.default_rng([s.seed, _TAG_KV, layer, slot])
    k = _normal_bits(rng, (length, s.Hkv, s.d), 1.0)
    v = _normal_bits(rng, (length, s.Hkv, s.d), 1.0)
    return k, v


def lognormal_lengths(seed: int, n: int, median: float, sigma: float, lo: int, hi: int) -> np.ndarray:
    """Prompt lengths round(exp(N(ln median, sigma))) clipped to [lo, hi]."""
    rng = np.random.default_rng([seed, _TAG_LEN, 0])
    v = np.exp(rng.normal(np.log(median), sigma, size=n))
    return np.clip(np.rint(v), lo, hi).astype(np.int64)


def uniform_lengths(seed: int, n: int, lo: int, hi: int) -> np.ndarray:
    """KV-cache lengths, integers uniform on [lo, hi] inclusive."""
    rng = np.random.default_rng([seed, _TAG_LEN, 1])
    return rng.integers(lo, hi + 1, size=n).astype(np.int64)
