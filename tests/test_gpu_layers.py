"""Whole-path parity on the GPU, through the C ABI: layer ingest, frontier, gated execution,
prefill + decode over the KV cache, boundary hand-off and split runs, against the CPU oracle."""
import numpy as np
import pytest

import workloads as W
from oracle import decoder as O
from tests import _util as U

pytestmark = pytest.mark.gpu

TINY = W.CONFIGS["tiny"]


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def _tol(fp32):
    return U.FP32_TOL if fp32 else U.BF16_TOL


def _run_gpu(inst, a, b, batch, x_dev):
    inst.run_layers(a, b, batch, x_dev)
    inst.sync()


# ------------------------------------------------------------------ config 1: the tiny decoder

@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
def test_tiny_prefill_then_decode_with_layer_streaming(torch, fp32):
    """2 layers; prefill of 64 tokens then 8 decode steps with fresh inputs; layer 1 is requested
    only after layer 0 has run (the frontier moves 0 -> 1 -> 2)."""
    s, os_ = TINY, U.oracle_shape(TINY)
    inst = U.make_instance(s, max_seqs=2, max_seq_len=128, max_tokens=64, kv_tokens=256, fp32=fp32)
    inst.kv_reserve(0, 72)
    bits = {l: W.layer_weights_bits(s, l) for l in range(s.L)}
    wts = {l: U.oracle_weights(bits[l]) for l in range(s.L)}
    pinned = {l: inst.pinned_blob(inst.pack_layer(bits[l])) for l in range(s.L)}

    xbits = W.hidden_bits(s, 64, step=0)
    x = U.to_device(xbits, fp32)
    torch.cuda.synchronize()
    batch = inst.batch([0, 64], [0], [0])
    obatch = O.OracleBatch([0, 64], [0], [0])
    okv = O.OracleKV()

    assert inst.frontier() == 0
    with pytest.raises(Exception) as ei:
        inst.run_layers(0, 1, batch, x)
    assert "BZ_ENOTLOADED" in str(ei.value)

    inst.load_layer(0, pinned[0])
    inst.wait_layer(0)
    assert inst.frontier() == 1 and inst.layer_ready(0) and not inst.layer_ready(1)
    assert np.array_equal(inst.readback_layer(0), pinned[0].numpy())
    _run_gpu(inst, 0, 1, batch, x)
    want1 = O.run_layers(os_, wts, 0, 1, U.f64(xbits), obatch, okv)
    assert U.rel_err(U.from_device(x), want1) <= _tol(fp32)

    inst.load_layer(1, pinned[1])
    with pytest.raises(Exception) as ei:
        inst.load_layer(1, pinned[1])
    assert "BZ_EBUSY" in str(ei.value)
    _run_gpu(inst, 1, 2, batch, x)               # gated on layer 1's event, no explicit wait
    assert inst.frontier() == 2
    assert np.array_equal(inst.readback_layer(1), pinned[1].numpy())
    want2 = O.run_layers(os_, wts, 1, 2, want1, obatch, okv)
    err = U.rel_err(U.from_device(x), want2)
    assert err <= _tol(fp32), err
    U.assert_rms(U.from_device(x), want2, U.RMS_FP32 if fp32 else U.RMS_BF16)

    # cache contents after prefill: K (rotated) and V of both layers
    for l in range(s.L):
        k = np.empty((64, s.Hkv, s.d), dtype=np.float32 if fp32 else np.uint16)
        v = np.empty_like(k)
        inst.kv_read(l, 0, 0, 64, k, v)
        kk = k.astype(np.float64) if fp32 else U.f64(k)
        vv = v.astype(np.float64) if fp32 else U.f64(v)
        assert U.rel_err(kk, okv.store[(l, 0)][0]) <= _tol(fp32)
        assert U.rel_err(vv, okv.store[(l, 0)][1]) <= _tol(fp32)

    # 8 decode steps, each with a fresh seeded input row
    dbatch = inst.batch([0, 1], [0], [64])
    worst = 0.0
    for step in range(8):
        dbits = W.hidden_bits(s, 1, step=1 + step)
        xd = U.to_device(dbits, fp32)
        torch.cuda.synchronize()
        _run_gpu(inst, 0, 2, dbatch, xd)
        want = O.run_layers(os_, wts, 0, 2, U.f64(dbits), O.OracleBatch([0, 1], [0], [64 + step]), okv)
        worst = max(worst, U.rel_err(U.from_device(xd), want))
        inst.batch_advance(dbatch)
    assert worst <= _tol(fp32), worst
    st = inst.stats()
    assert st["bytes_ingested"] == 2 * inst.layer_bytes and st["layers_requested"] == 2
    assert st["tokens_run"] == 64 * 2 + 8 * 2
    inst.close()


def test_tiny_split_is_bit_exact_and_uses_two_instances(torch):
    """Cooperative execution: instance T runs [0,k), hands the activation over (device and host
    paths), instance S runs [k,L); output bits equal the unsplit run for every k, in prefill and in
    the decode steps that follow."""
    s = TINY
    def fresh():
        inst = U.make_instance(s, max_seqs=2, max_seq_len=128, max_tokens=64, kv_tokens=256)
        inst.kv_reserve(0, 80)
        U.load_all_layers(inst, s)
        return inst
    xbits = W.hidden_bits(s, 64, step=0)
    dsteps = [W.hidden_bits(s, 1, step=1 + i) for i in range(3)]

    def run(k, via_host):
        tgt, src = fresh(), fresh()
        outs = []
        for i, bits in enumerate([xbits] + dsteps):
            T = bits.shape[0]
            before = 0 if i == 0 else 64 + i - 1
            batch = tgt.batch([0, T], [0], [before])
            x = U.to_device(bits, False)
            torch.cuda.synchronize()
            tgt.run_layers(0, k, batch, x)
            if via_host:
                buf = np.empty((T, s.H), dtype=np.uint16)
                tgt.export_boundary(x, T, buf)
                y = torch.zeros_like(x)
                torch.cuda.synchronize()
                src.import_boundary(y, T, buf)
            else:
                buf = torch.zeros_like(x)
                y = torch.zeros_like(x)
                torch.cuda.synchronize()
                tgt.export_boundary(x, T, buf)
                tgt.sync()
                src.import_boundary(y, T, buf)
            src.run_layers(k, s.L, batch, y)
            src.sync()
            outs.append(y.view(torch.int16).cpu().numpy().copy())
        tgt.close(); src.close()
        return outs

    whole = run(0, False)          # k = 0: everything on one instance
    for k in (1, 2):
        for via_host in (False, True):
            got = run(k, via_host)
            for a, b in zip(whole, got):
                assert np.array_equal(a, b), (k, via_host)


def test_nowait_reports_not_ready_and_frontier_is_prefix(torch):
    s = TINY
    inst = U.make_instance(s, max_seqs=1, max_seq_len=64, max_tokens=16, kv_tokens=64)
    inst.kv_reserve(0, 16)
    bits1 = W.layer_weights_bits(s, 1)
    p1 = inst.pinned_blob(inst.pack_layer(bits1))
    inst.load_layer(1, p1)                      # out of order: layer 1 first
    inst.wait_layer(1)
    assert inst.frontier() == 0 and inst.layer_ready(1)
    x = U.to_device(W.hidden_bits(s, 4), False)
    torch.cuda.synchronize()
    batch = inst.batch([0, 4], [0], [0])
    from paper_2412_17246_amd import BZ_RUN_NOWAIT
    with pytest.raises(Exception) as ei:
        inst.run_layers(0, 2, batch, x, BZ_RUN_NOWAIT)
    assert "BZ_ENOTLOADED" in str(ei.value)
    inst.run_layers(1, 2, batch, x, BZ_RUN_NOWAIT)      # only [1,2) needs to be resident
    inst.sync()
    p0 = inst.pinned_blob(inst.pack_layer(W.layer_weights_bits(s, 0)))
    inst.load_layer(0, p0)
    inst.wait_layer(0)
    assert inst.frontier() == 2
    ms0, ms1 = inst.layer_ready_ms(0), inst.layer_ready_ms(1)
    assert 0.0 <= ms1 <= ms0
    # capacity errors: more new tokens than the slot holds
    big = inst.batch([0, 16], [0], [20])         # 20 + 16 > the 32 positions the slot holds
    xb = U.to_device(W.hidden_bits(s, 16), False)
    with pytest.raises(Exception) as ei:
        inst.run_layers(0, 2, big, xb)
    assert "BZ_ECAPACITY" in str(ei.value)
    inst.unload_layer(1)
    assert inst.frontier() == 1
    inst.close()


# ------------------------------------------------------------------ ragged / mixed batches, GQA

MIX = W.DecoderShape("mix", L=2, H=512, Hq=8, Hkv=2, d=128, F=1024, rope_base=500000.0, seed=21)
MIX64 = W.DecoderShape("mix64", L=2, H=256, Hq=4, Hkv=2, d=64, F=512, rope_base=10000.0, seed=22)
MHA = W.DecoderShape("mha", L=1, H=512, Hq=4, Hkv=4, d=128, F=768, rope_base=10000.0, seed=23)
G8 = W.DecoderShape("g8", L=1, H=1024, Hq=8, Hkv=1, d=128, F=512, rope_base=500000.0, seed=24)
# 24 query heads in 12 kv groups: three heads per XCD, which the groups of two do not tile
H24 = W.DecoderShape("h24", L=1, H=768, Hq=24, Hkv=12, d=64, F=512, rope_base=10000.0, seed=25)


def _mixed_case(torch, s, fp32, seqs):
    """seqs: list of (new_tokens, kv_len_before).  Sequences with a non-empty cache get seeded
    pre-existing K/V in every layer, written through the C ABI."""
    os_ = U.oracle_shape(s)
    total_cap = sum((n + b + 31) // 32 * 32 for n, b in seqs) + 32      # slots are multiples of 32 positions
    T = sum(n for n, _ in seqs)
    inst = U.make_instance(s, max_seqs=len(seqs), max_seq_len=max(n + b for n, b in seqs) + 1,
                           max_tokens=T, kv_tokens=total_cap, fp32=fp32)
    bits = {l: W.layer_weights_bits(s, l) for l in range(s.L)}
    wts = {l: U.oracle_weights(bits[l]) for l in range(s.L)}
    U.load_all_layers(inst, s)
    okv = O.OracleKV()
    for i, (n, before) in enumerate(seqs):
        inst.kv_reserve(i, max(n + before, 1))
        if before:
            for l in range(s.L):
                kb, vb = W.kv_prefill_bits(s, l, i, before)
                okv.put(l, i, U.f64(kb), U.f64(vb))
                if fp32:
                    inst.kv_write(l, i, 0, before, W.f32_from_bf16_bits(kb), W.f32_from_bf16_bits(vb))
                else:
                    inst.kv_write(l, i, 0, before, kb, vb)
    q_start = np.concatenate([[0], np.cumsum([n for n, _ in seqs])])
    slots = list(range(len(seqs)))
    befores = [b for _, b in seqs]
    # hidden states of rms 1/16: with these narrow shapes a layer adds an update of rms 0.03 .. 0.3, which next to
    # a residual stream of rms 1 would be a small part of the output, and the gates on the output would see a
    # mistake inside the layer diluted by that factor
    xbits = W.hidden_bits(s, T, step=3, scale=1.0 / 16)
    x = U.to_device(xbits, fp32)
    torch.cuda.synchronize()
    batch = inst.batch(q_start, slots, befores)
    inst.run_layers(0, s.L, batch, x)
    inst.sync()
    want = O.run_layers(os_, wts, 0, s.L, U.f64(xbits), O.OracleBatch(list(q_start), slots, befores), okv)
    got = U.from_device(x)
    inst.close()
    U.assert_rms(got, want, U.RMS_FP32 if fp32 else U.RMS_BF16)
    return got, want, q_start


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("shape", [MIX, MIX64, MHA, G8, H24], ids=lambda s: s.name)
def test_mixed_ragged_batch(torch, fp32, shape):
    # prefill of several tiles + ragged tail, a 1-token prefill-from-empty, chunked prefill on top of
    # a cache, an empty sequence, and decode tokens whose caches straddle the 256-position chunks
    seqs = [(200, 0), (37, 0), (1, 299), (130, 70), (0, 5), (1, 0), (1, 255), (1, 256), (1, 700), (2, 0)]
    got, want, q_start = _mixed_case(torch, shape, fp32, seqs)
    tol = _tol(fp32)
    assert U.rel_err(got, want) <= tol
    for i in range(len(seqs)):                       # every sequence on its own, too
        a, b = q_start[i], q_start[i + 1]
        if b > a:
            assert U.rel_err(got[a:b], want[a:b]) <= tol, (i, seqs[i])


def _random_case(case):
    """A seeded random decoder shape (head size, heads per group, widths that are multiples of 8 only) and batch."""
    import random
    rnd = random.Random(case)
    d = rnd.choice([64, 128])
    Hkv = rnd.choice([1, 2, 3, 4, 6])
    Hq = Hkv * rnd.choice([1, 2, 4, 8])
    s = W.DecoderShape(f"r{case}", L=rnd.choice([1, 2]), H=8 * rnd.randint(8, 160), Hq=Hq, Hkv=Hkv, d=d,
                       F=8 * rnd.randint(8, 200), rope_base=rnd.choice([10000.0, 500000.0]), seed=1000 + case)
    kind = rnd.choice(["mixed", "decode", "prefill", "small"])
    seqs = []
    for _ in range(rnd.randint(1, 12)):
        if kind == "decode":
            seqs.append((1, rnd.choice([0, 1, 31, 255, 256, 257, rnd.randint(0, 1500)])))
        elif kind == "prefill":
            seqs.append((rnd.choice([2, 17, 128, 129, rnd.randint(2, 400)]), rnd.choice([0, 0, rnd.randint(0, 300)])))
        elif kind == "small":
            seqs.append((rnd.choice([0, 1, 1, 2, 5]), rnd.choice([0, 3, 40, 300])))
        else:
            seqs.append((rnd.choice([0, 1, 1, 1, 3, 64, rnd.randint(1, 300)]),
                         rnd.choice([0, 0, 15, 16, 255, 256, rnd.randint(0, 900)])))
    seqs = [(n, b if (n or b) else 1) for n, b in seqs]      # _mixed_case's arena has room for one empty sequence
    if sum(n for n, _ in seqs) == 0:
        seqs.append((1, 7))
    return s, seqs


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("case", range(16))
def test_random_shapes_and_batches(torch, fp32, case):
    # widths, head counts and length mixes nobody picked by hand (three and six kv heads, widths like 8 * 37)
    shape, seqs = _random_case(case)
    got, want, _ = _mixed_case(torch, shape, fp32, seqs)
    assert U.rel_err(got, want) <= _tol(fp32), (shape, seqs)


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("scale", [0.0, 1e-30, 1e-6, 1e4, 1e30], ids=lambda v: f"x{v:g}")
def test_extreme_finite_hidden_states(torch, fp32, scale):
    # all-zero input, magnitudes at both ends of the bf16 range: nothing overflows into inf or nan on the way (the
    # norms rescale, the softmax subtracts its maximum) and the output still follows the oracle
    s = W.DecoderShape("ext", L=2, H=256, Hq=4, Hkv=2, d=64, F=512, rope_base=10000.0, seed=5)
    bits = {l: W.layer_weights_bits(s, l) for l in range(s.L)}
    inst = U.make_instance(s, max_seqs=2, max_seq_len=400, max_tokens=301, kv_tokens=480, fp32=fp32)
    U.load_all_layers(inst, s)
    inst.kv_reserve(0, 300)
    inst.kv_reserve(1, 100)
    xf = W.f32_from_bf16_bits(W.hidden_bits(s, 301, step=2)) * np.float32(scale)
    xb = W.bf16_bits_from_f32(xf.astype(np.float32))
    x = U.to_device(xb, fp32)
    torch.cuda.synchronize()
    inst.run_layers(0, s.L, inst.batch([0, 300, 301], [0, 1], [0, 0]), x)      # a 300-token prompt and a 1-token one
    inst.sync()
    got = U.from_device(x)
    inst.close()
    want = O.run_layers(U.oracle_shape(s), {l: U.oracle_weights(bits[l]) for l in range(s.L)}, 0, s.L, U.f64(xb),
                        O.OracleBatch([0, 300, 301], [0, 1], [0, 0]), O.OracleKV())
    assert np.isfinite(got).all()
    if scale == 0.0:
        assert not got.any()
    else:
        assert U.rel_err(got, want) <= _tol(fp32)


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("shape", [MIX, G8], ids=lambda s: s.name)
def test_small_mixed_batch_takes_the_decode_sized_kernels(torch, fp32, shape):
    # at most 64 rows in all, so the projections leave split-K partial sums that the rotary/append and norm
    # kernels fold; the batch still holds prefills long enough to write whole 16-position groups of V
    # (from partial sums), a chunked prefill that starts inside a group, and decode tokens
    seqs = [(20, 0), (1, 40), (17, 16), (1, 0), (19, 7), (1, 300)]
    assert sum(n for n, _ in seqs) <= 64
    got, want, q_start = _mixed_case(torch, shape, fp32, seqs)
    tol = _tol(fp32)
    assert U.rel_err(got, want) <= tol
    for i in range(len(seqs)):
        a, b = q_start[i], q_start[i + 1]
        assert U.rel_err(got[a:b], want[a:b]) <= tol, (i, seqs[i])


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("shape", [MIX64, G8], ids=lambda s: s.name)
def test_long_caches(torch, fp32, shape):
    # decode over caches of more than 16 chunks of 256 positions (the combine step then takes its partial
    # results in several batches), at and just past a chunk boundary, and a chunked prefill whose new
    # tokens sit on top of a long cache, and one prefill of several thousand tokens from an empty cache
    seqs = [(1, 9000), (1, 4095), (1, 4096), (70, 5000), (1, 4351), (3001, 0)]
    got, want, q_start = _mixed_case(torch, shape, fp32, seqs)
    tol = _tol(fp32)
    for i in range(len(seqs)):
        a, b = q_start[i], q_start[i + 1]
        assert U.rel_err(got[a:b], want[a:b]) <= tol, (i, seqs[i])


ODD = [W.DecoderShape("odd264", L=2, H=264, Hq=3, Hkv=3, d=64, F=520, rope_base=10000.0, seed=31),
       W.DecoderShape("odd328", L=2, H=328, Hq=6, Hkv=3, d=128, F=344, rope_base=500000.0, seed=32),
       W.DecoderShape("odd1096", L=1, H=1096, Hq=16, Hkv=2, d=64, F=1000, rope_base=10000.0, seed=33)]


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("rows", ["decode-sized", "hundreds"])
@pytest.mark.parametrize("shape", ODD, ids=lambda s: s.name)
def test_widths_that_are_no_multiple_of_a_tile(torch, fp32, shape, rows):
    # hidden and MLP widths that are multiples of 8 only (every reduction dimension ends in a partial 64-wide
    # k-tile, so the projections take the kernel with a K tail), 3, 6 and 16 query heads, all four group sizes
    # between them; a decode-sized batch and one of a few hundred rows
    seqs = [(5, 0), (1, 37), (1, 300), (2, 31), (1, 0)] if rows == "decode-sized" else \
           [(150, 0), (1, 64), (97, 33), (1, 511), (40, 200)]
    got, want, q_start = _mixed_case(torch, shape, fp32, seqs)
    tol = _tol(fp32)
    for i in range(len(seqs)):
        a, b = q_start[i], q_start[i + 1]
        assert U.rel_err(got[a:b], want[a:b]) <= tol, (i, seqs[i])


@pytest.mark.parametrize("shape", [MIX64, G8], ids=lambda s: s.name)
def test_caches_of_tens_of_thousands_of_positions(torch, shape):
    # far beyond the benchmark's 4096: a decode step over 70000 cached positions (274 chunks, 18 batches of
    # partial results in the combine step; rotary angles up to 70000 * theta), two new tokens on top of 65535
    # (the prefill kernel walks 1024 tiles of keys and ends one position past a power of two), a cache of
    # exactly 32768, and a short neighbour so that the work list mixes 1-chunk and 274-chunk sequences
    seqs = [(1, 70000), (2, 65535), (1, 32768), (1, 5)]
    got, want, q_start = _mixed_case(torch, shape, False, seqs)
    for i in range(len(seqs)):
        a, b = q_start[i], q_start[i + 1]
        assert U.rel_err(got[a:b], want[a:b]) <= U.BF16_TOL, (i, seqs[i])


@pytest.mark.parametrize("extra", [0, 90], ids=["105rows", "195rows"])
@pytest.mark.parametrize("shape", [MIX, G8], ids=lambda s: s.name)
def test_mixed_batch_of_65_to_256_rows(torch, shape, extra):
    # beyond the 64 rows of a decode-sized batch the split-K projections work in blocks of 128 rows (one block
    # up to 128 rows, two up to 256) and still leave partial sums for the rotary/append and norm kernels to fold
    seqs = [(40, 0), (1, 40), (33, 16), (1, 0), (19, 7), (1, 300), (1, 255), (9, 100)]
    if extra:
        seqs.append((extra, 3))
    rows = sum(n for n, _ in seqs)
    assert (64 < rows <= 128) if not extra else (128 < rows <= 256)
    got, want, q_start = _mixed_case(torch, shape, False, seqs)
    for i in range(len(seqs)):
        a, b = q_start[i], q_start[i + 1]
        assert U.rel_err(got[a:b], want[a:b]) <= U.BF16_TOL, (i, seqs[i])


def test_first_causal_token_rows_follow_the_oracle(torch):
    """Rows whose attention sees a single key (row 0 of a prefill sequence; a decode token on an empty
    cache), inside an ordinary layer with random weights, against the oracle at the usual tolerance.  The
    exact form of the invariant is the next test."""
    s = MHA
    inst = U.make_instance(s, max_seqs=2, max_seq_len=64, max_tokens=8, kv_tokens=128)
    inst.kv_reserve(0, 8); inst.kv_reserve(1, 8)
    U.load_all_layers(inst, s)
    x = U.to_device(W.hidden_bits(s, 4, step=0), False)
    torch.cuda.synchronize()
    batch = inst.batch([0, 3, 4], [0, 1], [0, 0])
    inst.run_layers(0, 1, batch, x)
    inst.sync()
    os_ = U.oracle_shape(s)
    wts = U.oracle_weights(W.layer_weights_bits(s, 0))
    xr = U.f64(W.hidden_bits(s, 4, step=0))
    want = O.run_layers(os_, {0: wts}, 0, 1, xr, O.OracleBatch([0, 3, 4], [0, 1], [0, 0]), O.OracleKV())
    got = U.from_device(x)
    assert U.rel_err(got[[0, 3]], want[[0, 3]]) <= U.BF16_TOL
    inst.close()


VROW_SHAPES = [
    W.DecoderShape("vrow_mha128", L=1, H=256, Hq=2, Hkv=2, d=128, F=128, rope_base=10000.0, seed=41),
    W.DecoderShape("vrow_gqa64", L=1, H=256, Hq=4, Hkv=1, d=64, F=64, rope_base=500000.0, seed=42),
    W.DecoderShape("vrow_g8", L=1, H=1024, Hq=8, Hkv=1, d=128, F=64, rope_base=10000.0, seed=43),
]


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("shape", VROW_SHAPES, ids=lambda s: s.name)
def test_first_causal_token_output_is_its_v_row_bit_for_bit(torch, fp32, shape):
    """The invariant itself, exactly.  A layer with H = Hq*d, Wo = identity and Wg = Wu = Wd = 0 returns
    x + attention output.  For a token that sees one key the softmax weight is exactly 1, so its output
    minus its input is the V row of that position (of its kv head, repeated for every query head of the
    group) - to the bit: output == round(x + v), one rounding of a sum of two stored values.  Prefill
    kernel: row 0 of sequences of 3, 130 (two query tiles) and 300 tokens; decode kernel: one token on an
    empty cache.  V is read back from the cache through the C ABI."""
    s = shape
    assert s.H == s.Hq * s.d
    G = s.Hq // s.Hkv
    bits = W.layer_weights_bits(s, 0)
    bits["wo"] = W.bf16_bits_from_f32(np.eye(s.H, dtype=np.float32))
    for name in ("wg", "wu", "wd"):
        bits[name] = np.zeros_like(bits[name])
    lens = [3, 1, 130, 300, 1]
    q_start = [0] + list(np.cumsum(lens))
    T, B = int(q_start[-1]), len(lens)
    inst = U.make_instance(s, max_seqs=B, max_seq_len=512, max_tokens=T, kv_tokens=sum((n + 31) // 32 * 32 for n in lens) + 32,
                           fp32=fp32)
    for i, n in enumerate(lens):
        inst.kv_reserve(i, n)
    inst.load_layer(0, inst.pinned_blob(inst.pack_layer(bits)))
    xbits = W.hidden_bits(s, T, step=9)
    x = U.to_device(xbits, fp32)
    x_in = x.clone()
    torch.cuda.synchronize()
    inst.run_layers(0, 1, inst.batch(q_start, list(range(B)), [0] * B), x)
    inst.sync()
    for i in range(B):
        row = int(q_start[i])
        k = np.empty((1, s.Hkv, s.d), dtype=np.float32 if fp32 else np.uint16)
        v = np.empty_like(k)
        inst.kv_read(0, i, 0, 1, k, v)
        v32 = v.astype(np.float32) if fp32 else W.f32_from_bf16_bits(v)
        v_heads = np.repeat(v32[0], G, axis=0).reshape(s.H)               # query head h reads kv head h // G
        assert np.any(v_heads != 0)
        x32 = x_in[row].float().cpu().numpy()
        want = x32 + v_heads                                             # float32 sum, as on the GPU
        if fp32:
            got = x[row].cpu().numpy()
            assert np.array_equal(got, want), (i, np.max(np.abs(got - want)))
        else:
            got = x[row].view(torch.int16).cpu().numpy().view(np.uint16)
            assert np.array_equal(got, W.bf16_bits_from_f32(want)), i
    inst.close()


def test_prefill_then_decode_matches_longer_prefill_on_the_gpu(torch):
    s = MIX
    n = 140
    xbits = W.hidden_bits(s, n + 1, step=5)
    def run(split):
        inst = U.make_instance(s, max_seqs=1, max_seq_len=256, max_tokens=n + 1, kv_tokens=256)
        inst.kv_reserve(0, n + 1)
        U.load_all_layers(inst, s)
        if not split:
            x = U.to_device(xbits, False); torch.cuda.synchronize()
            inst.run_layers(0, s.L, inst.batch([0, n + 1], [0], [0]), x); inst.sync()
            out = U.from_device(x)[n]
        else:
            x = U.to_device(xbits[:n], False); y = U.to_device(xbits[n:], False); torch.cuda.synchronize()
            inst.run_layers(0, s.L, inst.batch([0, n], [0], [0]), x)
            inst.run_layers(0, s.L, inst.batch([0, 1], [0], [n]), y); inst.sync()
            out = U.from_device(y)[0]
        inst.close()
        return out
    a, b = run(False), run(True)
    assert U.rel_err(b, a) <= U.BF16_TOL


def test_gqa_decode_live_split_is_bit_exact_over_steps(torch):
    """8B-GQA-like shape (4 query heads per kv head, d = 128), 4 layers, continuous decode of 6
    sequences whose caches straddle the 256-position chunks; a live split at layer 2 with two
    instance handles and a boundary hand-off every step must reproduce the unsplit bits."""
    s = W.DecoderShape("gqa_split", L=4, H=512, Hq=8, Hkv=2, d=128, F=1024, rope_base=500000.0, seed=31)
    lens = [5, 255, 256, 300, 511, 700]
    B, steps, k = len(lens), 5, 2

    def fresh(layers):
        inst = U.make_instance(s, max_seqs=B, max_seq_len=768, max_tokens=B, kv_tokens=sum(lens) + 64 * B)
        U.load_all_layers(inst, s, layers)
        for i, n in enumerate(lens):
            inst.kv_reserve(i, n + steps)
            for l in layers:
                kb, vb = W.kv_prefill_bits(s, l, i, n)
                inst.kv_write(l, i, 0, n, kb, vb)
        return inst

    whole, tgt, src = fresh(range(4)), fresh(range(0, k)), fresh(range(k, 4))
    bw = whole.batch(list(range(B + 1)), list(range(B)), lens)
    bs = tgt.batch(list(range(B + 1)), list(range(B)), lens)
    for step in range(steps):
        bits = W.hidden_bits(s, B, step=40 + step)
        a, b = U.to_device(bits, False), U.to_device(bits, False)
        c = torch.zeros_like(b)
        buf = np.empty((B, s.H), dtype=np.uint16)
        torch.cuda.synchronize()
        whole.run_layers(0, 4, bw, a)
        whole.batch_advance(bw)
        tgt.run_layers(0, k, bs, b)
        tgt.export_boundary(b, B, buf)          # through host memory: waits for the target's stream
        src.import_boundary(c, B, buf)
        src.run_layers(k, 4, bs, c)
        src.sync()
        tgt.batch_advance(bs)                   # shared batch: advance once, after both halves ran
        tgt.sync()
        whole.sync()
        assert torch.equal(a.view(torch.int16), c.view(torch.int16)), step
    for inst in (whole, tgt, src):
        inst.close()


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
def test_decode_steps_across_chunk_boundaries_follow_the_oracle(torch, fp32):
    """Continuous decode with batch_advance while caches grow past multiples of 256 positions: the list of
    cache chunks the attention visits is rebuilt on the device every step."""
    s, os_ = MIX, U.oracle_shape(MIX)
    lens = [254, 255, 510, 3, 767]
    B, steps = len(lens), 4
    inst = U.make_instance(s, max_seqs=B, max_seq_len=1024, max_tokens=B, kv_tokens=sum(lens) + 64 * B, fp32=fp32)
    bits = {l: W.layer_weights_bits(s, l) for l in range(s.L)}
    wts = {l: U.oracle_weights(bits[l]) for l in range(s.L)}
    U.load_all_layers(inst, s)
    okv = O.OracleKV()
    for i, n in enumerate(lens):
        inst.kv_reserve(i, n + steps)
        for l in range(s.L):
            kb, vb = W.kv_prefill_bits(s, l, i, n)
            okv.put(l, i, U.f64(kb), U.f64(vb))
            if fp32:
                inst.kv_write(l, i, 0, n, W.f32_from_bf16_bits(kb), W.f32_from_bf16_bits(vb))
            else:
                inst.kv_write(l, i, 0, n, kb, vb)
    batch = inst.batch(list(range(B + 1)), list(range(B)), lens)
    for step in range(steps):
        xbits = W.hidden_bits(s, B, step=60 + step)
        x = U.to_device(xbits, fp32)
        torch.cuda.synchronize()
        inst.run_layers(0, s.L, batch, x)
        inst.batch_advance(batch)
        inst.sync()
        want = O.run_layers(os_, wts, 0, s.L, U.f64(xbits),
                            O.OracleBatch(list(range(B + 1)), list(range(B)), [n + step for n in lens]), okv)
        got = U.from_device(x)
        for i in range(B):
            assert U.rel_err(got[i:i + 1], want[i:i + 1]) <= _tol(fp32), (step, i)
    inst.close()


def test_batch_advance_reports_when_its_chunk_list_is_full(torch):
    s = TINY
    inst = U.make_instance(s, max_seqs=1, max_seq_len=64, max_tokens=1, kv_tokens=64)
    batch = inst.batch([0, 1], [0], [0])
    room = (1 + 64) * 256 - 1                   # the cache may grow to 65 chunks of 256 positions
    for _ in range(room):
        inst.batch_advance(batch)
    with pytest.raises(Exception) as ei:
        inst.batch_advance(batch)
    assert "BZ_ECAPACITY" in str(ei.value)
    inst.sync()
    inst.close()


def test_decode_batch_of_300_sequences_with_advance(torch):
    """More decode sequences than the 256 threads of the kernel that rebuilds the chunk list: the list is
    built in several passes with a running offset."""
    s, os_ = TINY, U.oracle_shape(TINY)
    B, steps = 300, 2
    lens = [(37 * i) % 290 + 1 for i in range(B)]            # 1..290: some sequences cross 256 while stepping
    inst = U.make_instance(s, max_seqs=B, max_seq_len=320, max_tokens=B, kv_tokens=sum(lens) + 64 * B)
    bits = {l: W.layer_weights_bits(s, l) for l in range(s.L)}
    wts = {l: U.oracle_weights(bits[l]) for l in range(s.L)}
    U.load_all_layers(inst, s)
    okv = O.OracleKV()
    for i, n in enumerate(lens):
        inst.kv_reserve(i, n + steps)
        for l in range(s.L):
            kb, vb = W.kv_prefill_bits(s, l, i, n)
            okv.put(l, i, U.f64(kb), U.f64(vb))
            inst.kv_write(l, i, 0, n, kb, vb)
    batch = inst.batch(list(range(B + 1)), list(range(B)), lens)
    for step in range(steps):
        xbits = W.hidden_bits(s, B, step=80 + step)
        x = U.to_device(xbits, False)
        torch.cuda.synchronize()
        inst.run_layers(0, s.L, batch, x)
        inst.batch_advance(batch)
        inst.sync()
        want = O.run_layers(os_, wts, 0, s.L, U.f64(xbits),
                            O.OracleBatch(list(range(B + 1)), list(range(B)), [n + step for n in lens]), okv)
        assert U.rel_err(U.from_device(x), want) <= U.BF16_TOL, step
    inst.close()


def test_slots_reused_out_of_order_and_sequences_in_any_slot_order(torch):
    """Slots released and reserved again land in holes of the arena, and a batch may name its slots in any
    order: sequence s of the batch lives where seq_slot[s] says, not at position s."""
    s = MIX
    os_ = U.oracle_shape(s)
    inst = U.make_instance(s, max_seqs=6, max_seq_len=400, max_tokens=256, kv_tokens=96 + 64 + 160 + 128)
    bits = {l: W.layer_weights_bits(s, l) for l in range(s.L)}
    wts = {l: U.oracle_weights(bits[l]) for l in range(s.L)}
    U.load_all_layers(inst, s)
    inst.kv_reserve(0, 96)
    inst.kv_reserve(1, 64)
    inst.kv_reserve(2, 160)
    inst.kv_release(1)
    inst.kv_reserve(5, 40)                      # into the hole slot 1 left (40 rounds up to its 64 positions)
    inst.kv_reserve(1, 128)                     # behind everything else
    assert inst.kv_free_tokens() == 0           # 96 + 64 + 160 + 128 positions, all taken
    # (new tokens, cached before) per sequence, and the slot each one lives in
    seqs = [(30, 0), (1, 95), (50, 60), (1, 127), (7, 20)]
    slots = [5, 0, 2, 1, 3]
    inst.kv_release(5)
    inst.kv_reserve(3, 27)                      # 32 positions at the start of the hole
    inst.kv_reserve(5, 30)                      # the other 32
    okv = O.OracleKV()
    for (n, before), slot in zip(seqs, slots):
        for l in range(s.L):
            if before:
                kb, vb = W.kv_prefill_bits(s, l, slot, before)
                okv.put(l, slot, U.f64(kb), U.f64(vb))
                inst.kv_write(l, slot, 0, before, kb, vb)
    q_start = np.concatenate([[0], np.cumsum([n for n, _ in seqs])])
    befores = [b for _, b in seqs]
    T = int(q_start[-1])
    xbits = W.hidden_bits(s, T, step=9, scale=1.0 / 16)
    x = U.to_device(xbits, False)
    torch.cuda.synchronize()
    inst.run_layers(0, s.L, inst.batch(q_start, slots, befores), x)
    inst.sync()
    got = U.from_device(x)
    want = O.run_layers(os_, wts, 0, s.L, U.f64(xbits), O.OracleBatch(list(q_start), slots, befores), okv)
    for i in range(len(seqs)):
        a, b = q_start[i], q_start[i + 1]
        assert U.rel_err(got[a:b], want[a:b]) <= U.BF16_TOL, (i, seqs[i], slots[i])
    U.assert_rms(got, want, U.RMS_BF16)
    # what the layers appended went to the right slots: read back sequence 4's cache (slot 3) in layer 1
    n, before = seqs[4]
    kk = torch.empty(before + n, s.Hkv, s.d, dtype=torch.bfloat16, device="cuda")
    vv = torch.empty_like(kk)
    inst.kv_read(1, 3, 0, before + n, kk, vv)
    inst.sync()
    assert U.rel_err(U.from_device(kk), okv.store[(1, 3)][0]) <= U.BF16_TOL
    assert U.rel_err(U.from_device(vv), okv.store[(1, 3)][1]) <= U.BF16_TOL
    inst.close()
