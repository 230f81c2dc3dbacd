"""CPU oracle for layer-by-layer decoder execution.  TEST INFRASTRUCTURE ONLY.

This module is the slow, plain definition that the HIP path is checked against.  Only the test
suite, the smoke check and the CPU-baseline leg of the benchmark may import it; the product
package never does, and it imports nothing from the product package.

What it computes.  The paper treats a model as a stack of L layers that a request passes through
one after another (section 2.1, "Serving within an instance"), first with the whole prompt
(prefill) and then one token at a time against a KV cache kept for the request (decode).  A
scaled instance may execute only the layers it has loaded and then hands the activation to the
other instance, which executes the rest (section 4, challenge C#2); the pipeline constraint
S_i + T_i = L (section 5.2, constraint C1) says every layer is executed exactly once, so a split
run computes the same function as an unsplit one.  The oracle is therefore the plain definition
of an L-layer pre-norm Llama-family decoder stack applied to hidden states, evaluated in float64
with no tiling, no online softmax, no splitting of reductions and no streaming.  The paper does
not spell out the arithmetic inside a layer; the conventions below are this build's readings:

  * pre-norm residual blocks, RMSNorm with gain, no biases;
  * rotary embedding pairs element j with element j + d/2 of a head, angle pos * base**(-2j/d),
    computed in float64;
  * attention scale 1/sqrt(d); causal: a token at absolute position p sees keys 0..p inclusive;
  * grouped-query attention: query head h reads key/value head h // (Hq // Hkv);
  * MLP is silu(x Wg^T) * (x Wu^T) followed by Wd, silu(z) = z / (1 + exp(-z));
  * projection matrices are stored [out_features, in_features].

Everything is float64 and nothing is rounded to bf16 inside; inputs are whatever the caller
passes (the tests pass bf16-representable values).

Pins (tests/test_oracle_*.py): brute-force attention with Python loops, softmax rows summing to
one, first causal token returning its V row, zero queries giving the running mean of V, grouped
heads against repeated heads, PyTorch's CPU scaled_dot_product_attention / rms_norm / linear /
silu on whole layers, rotary norm preservation / relative-position property / complex-number
form / the d = 2 rotation, RMSNorm of a constant vector, SiLU identities, zeroed Wo / Wd,
single-entry weight matrices (orientation), prefill-vs-decode consistency, batch independence,
exact equality of split and unsplit runs, and the paper's 7-layer cooperative-throughput example.
Every function of this module, whole layers included, is covered by one of these pins.  The paper
prints no numeric layer outputs, so there are no golden hidden-state values to store: the whole-layer
pin is the independent composition of PyTorch's CPU routines, not a printed number.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np


@dataclass
class OracleShape:
    L: int
    H: int
    Hq: int
    Hkv: int
    d: int
    F: int
    eps: float = 1e-5
    rope_base: float = 10000.0


@dataclass
class OracleBatch:
    """A packed ragged batch: sequence s owns rows q_start[s]..q_start[s+1] of the hidden states,
    lives in KV slot seq_slot[s] and already has kv_len_before[s] cached positions."""
    q_start: list
    seq_slot: list
    kv_len_before: list

    @property
    def B(self) -> int:
        return len(self.seq_slot)

    @property
    def T(self) -> int:
        return int(self.q_start[-1])


@dataclass
class OracleKV:
    """KV cache: (layer, slot) -> [K, V], each a float64 array [len, Hkv, d] that grows."""
    store: dict = field(default_factory=dict)

    def get(self, layer, slot, Hkv, d):
        key = (layer, slot)
        if key not in self.store:
            self.store[key] = [np.zeros((0, Hkv, d)), np.zeros((0, Hkv, d))]
        return self.store[key]

    def put(self, layer, slot, k, v):
        self.store[(layer, slot)] = [np.array(k, dtype=np.float64), np.array(v, dtype=np.float64)]


def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    """y = x / sqrt(mean(x^2) + eps) * gain, per row."""
    x = np.asarray(x, dtype=np.float64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, dtype=np.float64)


def rope(x: np.ndarray, pos: np.ndarray, base: float) -> np.ndarray:
    """Rotate each head vector of x [T, heads, d] by its token's absolute position."""
    x = np.asarray(x, dtype=np.float64)
    T, nh, d = x.shape
    half = d // 2
    j = np.arange(half, dtype=np.float64)
    theta = np.asarray(base, dtype=np.float64) ** (-2.0 * j / d)          # [half]
    ang = np.asarray(pos, dtype=np.float64)[:, None] * theta[None, :]     # [T, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    lo, hi = x[..., :half], x[..., half:]
    return np.concatenate([lo * c - hi * s, hi * c + lo * s], axis=-1)


def softmax_rows(scores: np.ndarray) -> np.ndarray:
    m = np.max(scores, axis=-1, keepdims=True)
    e = np.exp(scores - m)
    return e / np.sum(e, axis=-1, keepdims=True)


def attention_weights(q: np.ndarray, K: np.ndarray, q_pos: np.ndarray) -> np.ndarray:
    """Causal softmax weights for one head: q [n, d], K [len, d], q_pos [n] absolute positions.
    Key j is visible to query i iff j <= q_pos[i]."""
    d = q.shape[-1]
    scores = (q @ K.T) / np.sqrt(float(d))
    keypos = np.arange(K.shape[0])
    scores = np.where(keypos[None, :] <= np.asarray(q_pos)[:, None], scores, -np.inf)
    return softmax_rows(scores)


def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, q_pos: np.ndarray) -> np.ndarray:
    """q [n, Hq, d]; K, V [len, Hkv, d]; returns [n, Hq, d]."""
    n, Hq, d = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    out = np.empty((n, Hq, d), dtype=np.float64)
    for h in range(Hq):
        kvh = h // G
        w = attention_weights(q[:, h, :], K[:, kvh, :], q_pos)
        out[:, h, :] = w @ V[:, kvh, :]
    return out


def silu(z: np.ndarray) -> np.ndarray:
    return z / (1.0 + np.exp(-z))


def linear(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """y = x W^T for a weight stored [out_features, in_features]."""
    return np.asarray(x, dtype=np.float64) @ np.asarray(w, dtype=np.float64).T


def swiglu(m: np.ndarray, wg: np.ndarray, wu: np.ndarray) -> np.ndarray:
    return silu(linear(m, wg)) * linear(m, wu)


def layer_forward(shape: OracleShape, w: dict, layer: int, x: np.ndarray, batch: OracleBatch,
                  kv: OracleKV) -> np.ndarray:
    """One decoder layer over a packed batch.  `w` maps tensor names (g1, wq, wk, wv, wo, g2, wg,
    wu, wd) to float arrays.  Appends this layer's K/V for the new tokens to `kv`."""
    s = shape
    x = np.asarray(x, dtype=np.float64)
    W = {k: np.asarray(v, dtype=np.float64) for k, v in w.items()}
    T = x.shape[0]
    n = rmsnorm(x, W["g1"], s.eps)
    q = linear(n, W["wq"]).reshape(T, s.Hq, s.d)
    k = linear(n, W["wk"]).reshape(T, s.Hkv, s.d)
    v = linear(n, W["wv"]).reshape(T, s.Hkv, s.d)
    o = np.empty((T, s.Hq, s.d), dtype=np.float64)
    for b in range(batch.B):
        r0, r1 = int(batch.q_start[b]), int(batch.q_start[b + 1])
        if r1 == r0:
            continue
        before = int(batch.kv_len_before[b])
        pos = before + np.arange(r1 - r0)
        qb = rope(q[r0:r1], pos, s.rope_base)
        kb = rope(k[r0:r1], pos, s.rope_base)
        cache = kv.get(layer, int(batch.seq_slot[b]), s.Hkv, s.d)
        assert cache[0].shape[0] == before, "kv_len_before does not match the cache"
        cache[0] = np.concatenate([cache[0], kb], axis=0)
        cache[1] = np.concatenate([cache[1], v[r0:r1]], axis=0)
        o[r0:r1] = attention(qb, cache[0], cache[1], pos)
    hmid = x + linear(o.reshape(T, s.Hq * s.d), W["wo"])
    m = rmsnorm(hmid, W["g2"], s.eps)
    return hmid + linear(swiglu(m, W["wg"], W["wu"]), W["wd"])


def run_layers(shape: OracleShape, weights, a: int, b: int, x: np.ndarray, batch: OracleBatch,
               kv: OracleKV) -> np.ndarray:
    """Layers [a, b) in order.  `weights[l]` is layer l's tensor dict (or a callable l -> dict)."""
    for l in range(a, b):
        w = weights(l) if callable(weights) else weights[l]
        x = layer_forward(shape, w, l, x, batch, kv)
    return x


def cooperative_run(shape: OracleShape, weights, k: int, x: np.ndarray, batch: OracleBatch,
                    kv_target: OracleKV, kv_source: OracleKV):
    """Section 4's cooperative execution: the scaled (target) instance executes layers [0, k),
    hands the activation over, and the source instance executes [k, L).  Returns the output and
    the number of layers each instance executed (target, source)."""
    mid = run_layers(shape, weights, 0, k, x, batch, kv_target)
    handed = np.array(mid, copy=True)            # the forwarded activation
    out = run_layers(shape, weights, k, shape.L, handed, batch, kv_source)
    return out, (k, shape.L - k)


def source_throughput(L: int, k: int) -> float:
    """Requests per layer-time the overloaded instance sustains when the scaled instance has
    taken over its first k layers (section 4's 7-layer example): it executes L - k layers per
    request."""
    return 1.0 / (L - k)
