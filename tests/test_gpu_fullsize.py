"""Parity at the real shapes, in the launch configurations the benchmark times: one decoder layer of
the 7B and 8B-GQA shapes, teacher-forced with seeded inputs, against the CPU oracle.  Where the
whole output is too expensive for the oracle, sampled sequences are compared (the oracle computes a
sequence on its own exactly as it does inside a batch)."""
import numpy as np
import pytest

import workloads as W
from oracle import decoder as O
from tests import _util as U

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def _one_layer_shape(base, layer_seed_shift=0):
    return W.DecoderShape(base.name, 1, base.H, base.Hq, base.Hkv, base.d, base.F, base.eps, base.rope_base, base.seed)


@pytest.mark.parametrize("layer", [0, 16])
def test_7b_layer_small_ragged_batch_whole_output(torch, layer):
    base = W.CONFIGS["7b"]
    s = _one_layer_shape(base)
    lens = [211, 122]                       # M = 333: the 128-row tile kernel with a ragged tail
    T = sum(lens)
    bits = W.layer_weights_bits(base, layer)
    inst = U.make_instance(s, max_seqs=2, max_seq_len=256, max_tokens=T, kv_tokens=512)
    for i, n in enumerate(lens):
        inst.kv_reserve(i, n)
    inst.load_layer(0, inst.pinned_blob(inst.pack_layer(bits)))
    xbits = W.hidden_bits(base, T, step=100 + layer)
    x = U.to_device(xbits, False)
    torch.cuda.synchronize()
    q_start = [0, lens[0], T]
    inst.run_layers(0, 1, inst.batch(q_start, [0, 1], [0, 0]), x)
    inst.sync()
    got = U.from_device(x)
    inst.close()
    want = O.run_layers(U.oracle_shape(s), {0: U.oracle_weights(bits)}, 0, 1, U.f64(xbits),
                        O.OracleBatch(q_start, [0, 1], [0, 0]), O.OracleKV())
    err = U.rel_err(got, want)
    assert err <= U.BF16_TOL, err


def test_7b_layer_bench_batch_sampled_sequences(torch):
    """The benchmark's own batch (8 requests, 6768 tokens: the 256x256 tile kernel, full prefill
    attention grid); the oracle recomputes the shortest request and the first 160 tokens of the
    longest one."""
    base = W.CONFIGS["7b"]
    s = _one_layer_shape(base)
    lens = W.lognormal_lengths(base.seed, 8, 512.0, 0.6, 16, 2048)
    q_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int64)
    T = int(q_start[-1])
    bits = W.layer_weights_bits(base, 0)
    inst = U.make_instance(s, max_seqs=8, max_seq_len=int(lens.max()) + 1, max_tokens=T, kv_tokens=T + 8 * 32)
    for i, n in enumerate(lens):
        inst.kv_reserve(i, int(n))
    inst.load_layer(0, inst.pinned_blob(inst.pack_layer(bits)))
    xbits = W.hidden_bits(base, T, step=0)
    x = U.to_device(xbits, False)
    torch.cuda.synchronize()
    inst.run_layers(0, 1, inst.batch(q_start, list(range(8)), [0] * 8), x)
    inst.sync()
    got = U.from_device(x)
    inst.close()
    wts = {0: U.oracle_weights(bits)}
    osh = U.oracle_shape(s)
    shortest, longest = int(np.argmin(lens)), int(np.argmax(lens))
    for seq, n in ((shortest, int(lens[shortest])), (longest, 160)):
        a = int(q_start[seq])
        want = O.run_layers(osh, wts, 0, 1, U.f64(xbits[a:a + n]), O.OracleBatch([0, n], [0], [0]), O.OracleKV())
        err = U.rel_err(got[a:a + n], want)
        assert err <= U.BF16_TOL, (seq, err)
    assert np.all(np.isfinite(got))


def test_8b_gqa_decode_step_full_batch(torch):
    """64 sequences with seeded caches of length uniform[256, 4096], one decode step through one
    layer at the real shape: whole output against the oracle."""
    base = W.CONFIGS["8b_gqa"]
    s = _one_layer_shape(base)
    B = 64
    lens = W.uniform_lengths(base.seed, B, 256, 4096)
    bits = W.layer_weights_bits(base, 0)
    inst = U.make_instance(s, max_seqs=B, max_seq_len=4097 + 1, max_tokens=B, kv_tokens=int(lens.sum()) + 33 * B)
    okv = O.OracleKV()
    for i, n in enumerate(lens):
        n = int(n)
        inst.kv_reserve(i, n + 1)
        kb, vb = W.kv_prefill_bits(base, 0, i, n)
        inst.kv_write(0, i, 0, n, kb, vb)
        okv.put(0, i, U.f64(kb), U.f64(vb))
    inst.load_layer(0, inst.pinned_blob(inst.pack_layer(bits)))
    xbits = W.hidden_bits(base, B, step=7)
    x = U.to_device(xbits, False)
    torch.cuda.synchronize()
    q_start = list(range(B + 1))
    befores = [int(n) for n in lens]
    inst.run_layers(0, 1, inst.batch(q_start, list(range(B)), befores), x)
    inst.sync()
    got = U.from_device(x)
    inst.close()
    want = O.run_layers(U.oracle_shape(s), {0: U.oracle_weights(bits)}, 0, 1, U.f64(xbits),
                        O.OracleBatch(q_start, list(range(B)), befores), okv)
    err = U.rel_err(got, want)
    assert err <= U.BF16_TOL, err
    for i in (int(np.argmin(lens)), int(np.argmax(lens))):       # shortest and longest cache on their own
        assert U.rel_err(got[i:i + 1], want[i:i + 1]) <= U.BF16_TOL


@pytest.mark.parametrize("streams", [1, 2])
def test_7b_layer_run_enqueued_while_its_weights_arrive(torch, streams):
    """run_layers is issued right behind load_layer, while the 405 MB of the layer are on their way (on one
    copy stream, or cut in halves over two): the stages wait for the tensor groups they read, and the output
    has the bits of a run on the resident layer."""
    base = W.CONFIGS["7b"]
    s = _one_layer_shape(base)
    lens = [211, 122]
    T = sum(lens)
    inst = U.make_instance(s, max_seqs=2, max_seq_len=256, max_tokens=T, kv_tokens=512)
    for i, n in enumerate(lens):
        inst.kv_reserve(i, n)
    inst.set_ingest_streams(streams)
    blob = inst.pinned_blob(inst.pack_layer(W.layer_weights_bits(base, 3)))
    xbits = W.hidden_bits(base, T, step=11)
    x1, x2 = U.to_device(xbits, False), U.to_device(xbits, False)
    batch = inst.batch([0, lens[0], T], [0, 1], [0, 0])
    torch.cuda.synchronize()
    inst.load_layer(0, blob)
    inst.run_layers(0, 1, batch, x1)
    in_flight = not inst.layer_ready(0)
    inst.sync()
    assert inst.layer_ready(0) and inst.frontier() == 1
    inst.run_layers(0, 1, batch, x2)          # same inputs, same cache positions, layer resident
    inst.sync()
    assert in_flight, "the layer had landed before the run was enqueued: the test did not exercise the gating"
    assert torch.equal(x1.view(torch.int16), x2.view(torch.int16))
    assert np.array_equal(inst.readback_layer(0), blob.numpy())
    inst.close()
