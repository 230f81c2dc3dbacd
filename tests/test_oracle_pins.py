"""Pins for the CPU oracle: everything here checks oracle/decoder.py against something that is
not the oracle — Python-loop brute force, closed forms, invariants, PyTorch CPU library routines
and the one worked example the paper prints for this path."""
import math
import os

import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import decoder as O

RNG = np.random.default_rng(1234)


def _rand(*shape):
    return RNG.standard_normal(shape)


# ---------------------------------------------------------------- attention

def _brute_attention(q, K, V, q_pos):
    """Explicit loops, math.exp, no numpy reductions."""
    n, Hq, d = q.shape
    Hkv = K.shape[1]
    G = Hq // Hkv
    out = np.zeros((n, Hq, d))
    for i in range(n):
        for h in range(Hq):
            kvh = h // G
            sc = []
            for j in range(q_pos[i] + 1):
                acc = 0.0
                for e in range(d):
                    acc += q[i, h, e] * K[j, kvh, e]
                sc.append(acc / math.sqrt(d))
            mx = max(sc)
            ex = [math.exp(v - mx) for v in sc]
            tot = sum(ex)
            for j, e_ in enumerate(ex):
                for e in range(d):
                    out[i, h, e] += (e_ / tot) * V[j, kvh, e]
    return out


@pytest.mark.parametrize("Hq,Hkv,before", [(2, 2, 0), (4, 2, 0), (4, 1, 3), (3, 3, 5)])
def test_attention_matches_brute_force(Hq, Hkv, before):
    n, d = 5, 4
    q = _rand(n, Hq, d)
    K = _rand(before + n, Hkv, d)
    V = _rand(before + n, Hkv, d)
    pos = before + np.arange(n)
    got = O.attention(q, K, V, pos)
    np.testing.assert_allclose(got, _brute_attention(q, K, V, pos), rtol=1e-12, atol=1e-13)


def test_softmax_rows_sum_to_one_and_mask():
    q = _rand(6, 8)
    K = _rand(9, 8)
    pos = 3 + np.arange(6)
    w = O.attention_weights(q, K, pos)
    np.testing.assert_allclose(w.sum(-1), 1.0, rtol=0, atol=1e-14)
    for i in range(6):
        assert np.all(w[i, pos[i] + 1:] == 0.0)
        assert np.all(w[i, :pos[i] + 1] > 0.0)


def test_first_causal_token_returns_its_v_row_exactly():
    q = _rand(4, 2, 8)
    K = _rand(4, 2, 8)
    V = _rand(4, 2, 8)
    out = O.attention(q, K, V, np.arange(4))
    assert np.array_equal(out[0], V[0])


def test_zero_query_gives_running_mean_of_v():
    n, H, d = 7, 2, 4
    K = _rand(n, H, d)
    V = _rand(n, H, d)
    out = O.attention(np.zeros((n, H, d)), K, V, np.arange(n))
    want = np.cumsum(V, axis=0) / np.arange(1, n + 1)[:, None, None]
    np.testing.assert_allclose(out, want, rtol=1e-13, atol=1e-14)


def test_gqa_equals_mha_with_repeated_kv_heads():
    n, Hq, Hkv, d = 6, 8, 2, 4
    q = _rand(n, Hq, d)
    K = _rand(n, Hkv, d)
    V = _rand(n, Hkv, d)
    pos = np.arange(n)
    got = O.attention(q, K, V, pos)
    Kr = np.repeat(K, Hq // Hkv, axis=1)
    Vr = np.repeat(V, Hq // Hkv, axis=1)
    want = O.attention(q, Kr, Vr, pos)
    assert np.array_equal(got, want)
    # and a wrong mapping (interleaved instead of contiguous groups) must differ
    Kw = np.tile(K, (1, Hq // Hkv, 1))
    assert not np.allclose(got, O.attention(q, Kw, Vr, pos))


def test_attention_matches_torch_sdpa():
    n, Hq, Hkv, d = 33, 4, 2, 16
    q = _rand(n, Hq, d)
    K = _rand(n, Hkv, d)
    V = _rand(n, Hkv, d)
    got = O.attention(q, K, V, np.arange(n))
    tq = torch.from_numpy(q).permute(1, 0, 2)[None]
    tk = torch.from_numpy(np.repeat(K, 2, axis=1)).permute(1, 0, 2)[None]
    tv = torch.from_numpy(np.repeat(V, 2, axis=1)).permute(1, 0, 2)[None]
    want = F.scaled_dot_product_attention(tq, tk, tv, is_causal=True)[0].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(got, want, rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- rotary embedding

def test_rope_preserves_norm_and_is_identity_at_zero():
    x = _rand(5, 3, 16)
    pos = np.array([0, 1, 7, 100, 4000])
    y = O.rope(x, pos, 10000.0)
    np.testing.assert_allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1), rtol=1e-13)
    assert np.array_equal(y[0], x[0])
    assert not np.allclose(y[1], x[1])


def test_rope_inner_product_depends_on_relative_position_only():
    q = _rand(1, 1, 32)
    k = _rand(1, 1, 32)
    def ip(m, n):
        return float(np.sum(O.rope(q, np.array([m]), 500000.0) * O.rope(k, np.array([n]), 500000.0)))
    assert abs(ip(5, 2) - ip(105, 102)) < 1e-11
    assert abs(ip(5, 2) - ip(1005, 1002)) < 1e-10
    assert abs(ip(5, 2) - ip(2, 5)) > 1e-3          # direction matters


def test_rope_d2_is_a_plane_rotation():
    # d = 2: one pair, theta_0 = 1, so position p rotates (1, 0) to (cos p, sin p).
    y = O.rope(np.array([[[1.0, 0.0]]]), np.array([3]), 10000.0)
    np.testing.assert_allclose(y[0, 0], [math.cos(3.0), math.sin(3.0)], rtol=0, atol=1e-15)
    y = O.rope(np.array([[[0.0, 1.0]]]), np.array([3]), 10000.0)
    np.testing.assert_allclose(y[0, 0], [-math.sin(3.0), math.cos(3.0)], rtol=0, atol=1e-15)


def test_rope_matches_complex_multiplication_with_half_split_pairs():
    d, base = 8, 10000.0
    x = _rand(4, 2, d)
    pos = np.array([0, 3, 17, 911])
    y = O.rope(x, pos, base)
    for t in range(4):
        for j in range(d // 2):
            theta = base ** (-2.0 * j / d)
            z = complex(x[t, 1, j], x[t, 1, j + d // 2]) * complex(math.cos(pos[t] * theta), math.sin(pos[t] * theta))
            assert abs(y[t, 1, j] - z.real) < 1e-12 and abs(y[t, 1, j + d // 2] - z.imag) < 1e-12
    # frequency of the pair j falls with j: the last pair barely turns at position 1
    y1 = O.rope(np.ones((1, 1, d)), np.array([1]), base)
    assert abs(y1[0, 0, d // 2 - 1] - 1.0) < 2e-3 and abs(y1[0, 0, 0] - 1.0) > 0.2


# ---------------------------------------------------------------- RMSNorm / SiLU

def test_rmsnorm_constant_vector_closed_form():
    c, eps = 3.0, 1e-5
    g = _rand(16)
    y = O.rmsnorm(np.full((2, 16), c), g, eps)
    np.testing.assert_allclose(y, np.broadcast_to(c / math.sqrt(c * c + eps) * g, (2, 16)), rtol=1e-15)


def test_rmsnorm_scale_invariance_unit_mean_square_and_torch():
    x = _rand(4, 64)
    g = np.ones(64)
    y = O.rmsnorm(x, g, 1e-5)
    np.testing.assert_allclose(np.mean(y * y, -1), 1.0, rtol=1e-4)
    np.testing.assert_allclose(O.rmsnorm(1000.0 * x, g, 1e-5), O.rmsnorm(100.0 * x, g, 1e-5), rtol=1e-6)
    g = _rand(64)
    want = F.rms_norm(torch.from_numpy(x), (64,), torch.from_numpy(g), 1e-5).numpy()
    np.testing.assert_allclose(O.rmsnorm(x, g, 1e-5), want, rtol=1e-12)
    # eps sits inside the square root, added to the mean (not to the sum, not outside)
    tiny = np.full((1, 4), 1e-3)
    np.testing.assert_allclose(O.rmsnorm(tiny, np.ones(4), 1e-5), 1e-3 / math.sqrt(1e-6 + 1e-5), rtol=1e-14)


def test_silu_identities():
    z = np.linspace(-20, 20, 81)
    assert O.silu(np.array([0.0]))[0] == 0.0
    np.testing.assert_allclose(O.silu(z) - O.silu(-z), z, rtol=1e-14, atol=1e-14)
    assert abs(O.silu(np.array([40.0]))[0] - 40.0) < 1e-12
    np.testing.assert_allclose(O.silu(z), F.silu(torch.from_numpy(z)).numpy(), rtol=1e-13, atol=1e-15)


# ---------------------------------------------------------------- whole layer

def _shape(**kw):
    base = dict(L=3, H=32, Hq=4, Hkv=2, d=8, F=48, eps=1e-5, rope_base=10000.0)
    base.update(kw)
    return O.OracleShape(**base)


def _weights(s, seed=0, scale=0.2):
    r = np.random.default_rng(seed)
    out = []
    for _ in range(s.L):
        out.append({
            "g1": 1 + 0.1 * r.standard_normal(s.H), "g2": 1 + 0.1 * r.standard_normal(s.H),
            "wq": scale * r.standard_normal((s.Hq * s.d, s.H)),
            "wk": scale * r.standard_normal((s.Hkv * s.d, s.H)),
            "wv": scale * r.standard_normal((s.Hkv * s.d, s.H)),
            "wo": scale * r.standard_normal((s.H, s.Hq * s.d)),
            "wg": scale * r.standard_normal((s.F, s.H)),
            "wu": scale * r.standard_normal((s.F, s.H)),
            "wd": scale * r.standard_normal((s.H, s.F)),
        })
    return out


def _torch_rope(x, pos, base):
    # complex-number form on interleaved pairs (xj, x_{j+d/2}) -> independent of oracle.rope
    T, nh, d = x.shape
    j = torch.arange(d // 2, dtype=torch.float64)
    ang = pos[:, None].double() * base ** (-2.0 * j / d)[None]
    z = torch.complex(x[..., : d // 2], x[..., d // 2:]) * torch.polar(torch.ones_like(ang), ang)[:, None, :]
    return torch.cat([z.real, z.imag], dim=-1)


def _torch_layer(s, w, x, before=0):
    """One layer on one sequence using PyTorch CPU library routines in float64."""
    t = {k: torch.from_numpy(np.asarray(v)) for k, v in w.items()}
    x = torch.from_numpy(x)
    T = x.shape[0]
    pos = before + torch.arange(T)
    n = F.rms_norm(x, (s.H,), t["g1"], s.eps)
    q = F.linear(n, t["wq"]).view(T, s.Hq, s.d)
    k = F.linear(n, t["wk"]).view(T, s.Hkv, s.d)
    v = F.linear(n, t["wv"]).view(T, s.Hkv, s.d)
    q, k = _torch_rope(q, pos, s.rope_base), _torch_rope(k, pos, s.rope_base)
    o = F.scaled_dot_product_attention(q.permute(1, 0, 2)[None], k.permute(1, 0, 2)[None],
                                       v.permute(1, 0, 2)[None], is_causal=True, enable_gqa=True)
    o = o[0].permute(1, 0, 2).reshape(T, s.Hq * s.d)
    h = x + F.linear(o, t["wo"])
    m = F.rms_norm(h, (s.H,), t["g2"], s.eps)
    return (h + F.linear(F.silu(F.linear(m, t["wg"])) * F.linear(m, t["wu"]), t["wd"])).numpy()


def test_layer_stack_matches_torch_library_routines():
    s = _shape()
    W = _weights(s)
    x = _rand(11, s.H)
    batch = O.OracleBatch([0, 11], [0], [0])
    got = O.run_layers(s, W, 0, s.L, x, batch, O.OracleKV())
    want = x
    for l in range(s.L):
        want = _torch_layer(s, W[l], want)
    np.testing.assert_allclose(got, want, rtol=1e-9, atol=1e-11)


def test_weight_orientation_single_entry_matrices():
    # wq with a single 1 at [out=i, in=j] must route normalised input feature j to q feature i.
    s = _shape(L=1, Hq=4, Hkv=4)
    w = {k: np.zeros_like(v) for k, v in _weights(s)[0].items()}
    w["g1"][:] = 1.0
    w["g2"][:] = 1.0
    # make v = copy of input feature 5 into v feature 2, and wo route attention feature 2 to hidden 9
    w["wv"][2, 5] = 1.0
    w["wo"][9, 2] = 1.0
    x = _rand(1, s.H)
    out = O.layer_forward(s, w, 0, x, O.OracleBatch([0, 1], [0], [0]), O.OracleKV())
    n = O.rmsnorm(x, np.ones(s.H), s.eps)
    want = x.copy()
    want[0, 9] += n[0, 5]          # single token: attention returns V
    np.testing.assert_allclose(out, want, rtol=1e-14)


def test_zero_wd_and_zero_wo():
    s = _shape(L=1)
    w = _weights(s)[0]
    x = _rand(5, s.H)
    b = O.OracleBatch([0, 5], [0], [0])
    w0 = dict(w, wo=np.zeros_like(w["wo"]), wd=np.zeros_like(w["wd"]))
    assert np.array_equal(O.layer_forward(s, w0, 0, x, b, O.OracleKV()), x)
    # wo = 0: output = x + mlp(x), independent of attention weights
    w1 = dict(w, wo=np.zeros_like(w["wo"]))
    w2 = dict(w1, wq=2 * w["wq"])
    assert np.array_equal(O.layer_forward(s, w1, 0, x, b, O.OracleKV()),
                          O.layer_forward(s, w2, 0, x, b, O.OracleKV()))


def test_mlp_closed_form_single_unit():
    # H = F-independent check of silu(gate) * up * down on a hand-computable case
    s = _shape(L=1, H=8, Hq=1, Hkv=1, d=8, F=8)
    w = {k: np.zeros_like(v) for k, v in _weights(s)[0].items()}
    w["g1"][:] = 1.0
    w["g2"][:] = 1.0
    w["wg"][3, 0] = 2.0
    w["wu"][3, 1] = 3.0
    w["wd"][4, 3] = 0.5
    x = _rand(1, 8)
    out = O.layer_forward(s, w, 0, x, O.OracleBatch([0, 1], [0], [0]), O.OracleKV())
    m = x / math.sqrt(float(np.mean(x * x)) + s.eps)
    gate, up = 2.0 * m[0, 0], 3.0 * m[0, 1]
    want = x.copy()
    want[0, 4] += 0.5 * (gate / (1 + math.exp(-gate))) * up
    np.testing.assert_allclose(out, want, rtol=1e-13)


def test_prefill_then_decode_equals_longer_prefill():
    s = _shape()
    W = _weights(s)
    x = _rand(9, s.H)
    full = O.run_layers(s, W, 0, s.L, x, O.OracleBatch([0, 9], [0], [0]), O.OracleKV())
    kv = O.OracleKV()
    first = O.run_layers(s, W, 0, s.L, x[:8], O.OracleBatch([0, 8], [0], [0]), kv)
    last = O.run_layers(s, W, 0, s.L, x[8:], O.OracleBatch([0, 1], [0], [8]), kv)
    np.testing.assert_allclose(first, full[:8], rtol=1e-12, atol=1e-13)
    np.testing.assert_allclose(last, full[8:], rtol=1e-10, atol=1e-12)


def test_packed_batch_equals_each_sequence_alone():
    s = _shape()
    W = _weights(s)
    lens = [3, 1, 6]
    x = _rand(sum(lens), s.H)
    starts = np.concatenate([[0], np.cumsum(lens)])
    kv = O.OracleKV()
    # sequence 1 is a decode token with 4 cached positions
    pre_k, pre_v = [], []
    for l in range(s.L):
        k0, v0 = _rand(4, s.Hkv, s.d), _rand(4, s.Hkv, s.d)
        kv.put(l, 11, k0, v0)
        pre_k.append(k0)
        pre_v.append(v0)
    got = O.run_layers(s, W, 0, s.L, x, O.OracleBatch(list(starts), [10, 11, 12], [0, 4, 0]), kv)
    for i, (slot, before) in enumerate([(10, 0), (11, 4), (12, 0)]):
        kv1 = O.OracleKV()
        if before:
            for l in range(s.L):
                kv1.put(l, slot, pre_k[l], pre_v[l])
        xi = x[starts[i]:starts[i + 1]]
        alone = O.run_layers(s, W, 0, s.L, xi, O.OracleBatch([0, lens[i]], [slot], [before]), kv1)
        # (BLAS may block a matmul differently for a different row count: equal to rounding)
        np.testing.assert_allclose(got[starts[i]:starts[i + 1]], alone, rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("k", [0, 1, 2, 3])
def test_split_run_is_exactly_the_unsplit_run(k):
    s = _shape()
    W = _weights(s)
    x = _rand(6, s.H)
    b = O.OracleBatch([0, 4, 6], [0, 1], [0, 0])
    whole = O.run_layers(s, W, 0, s.L, x, b, O.OracleKV())
    out, counts = O.cooperative_run(s, W, k, x, b, O.OracleKV(), O.OracleKV())
    assert np.array_equal(out, whole)
    assert counts == (k, s.L - k)


def test_paper_cooperative_throughput_example():
    path = os.path.join(os.path.dirname(__file__), "golden", "coop_throughput.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for L, k, num, den in rows:
        L, k = int(L), int(k)
        assert abs(O.source_throughput(L, k) - int(num) / int(den)) < 1e-15
        # the count that the split runner reports is the one the closed form uses
        s = _shape(L=L)
        _, counts = O.cooperative_run(s, _weights(s), k, _rand(2, s.H), O.OracleBatch([0, 2], [0], [0]),
                                      O.OracleKV(), O.OracleKV())
        assert counts[1] == L - k and abs(1.0 / counts[1] - O.source_throughput(L, k)) < 1e-15
