"""Serving-loop behaviour of the C ABI on the GPU: batches that live in caller memory and are rebuilt every
step (continuous batching), a batch shared by two instances on different streams with no host
synchronisation in between, ordering against the caller's own stream, and the checks on ingest sources."""
import numpy as np
import pytest

import workloads as W
from oracle import decoder as O
from tests import _util as U

pytestmark = pytest.mark.gpu

SHAPE = W.DecoderShape("serve", L=2, H=512, Hq=8, Hkv=2, d=128, F=1024, rope_base=500000.0, seed=51)


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def _fresh(torch, s, lens, extra, layers=None, stream=None):
    from paper_2412_17246_amd import Instance
    inst = Instance(s, max_seqs=len(lens), max_seq_len=1024, max_tokens=256, kv_tokens=sum(lens) + (extra + 64) * len(lens),
                    compute_stream=stream)
    U.load_all_layers(inst, s, layers)
    for i, n in enumerate(lens):
        inst.kv_reserve(i, n + extra)
        for l in (range(s.L) if layers is None else layers):
            kb, vb = W.kv_prefill_bits(s, l, i, n)
            inst.kv_write(l, i, 0, n, kb, vb)
    inst.sync()
    return inst


def test_continuous_batching_with_a_batch_rebuilt_in_place_every_step(torch):
    """Six sequences with caches; every step a different subset decodes (one leaves, another joins) and one
    step mixes in a prefill chunk.  Instance A builds a fresh batch per step with the allocating call;
    instance B rebuilds one batch object in lent memory, asynchronously, and runs three steps ahead of the
    device without any host synchronisation.  Outputs must be the same bits, and follow the oracle."""
    s = SHAPE
    lens = [5, 255, 256, 300, 511, 40]
    a, b = _fresh(torch, s, lens, 16), _fresh(torch, s, lens, 16)
    storage = b.batch_storage(max_seqs=6, max_tokens=64, max_seq_len=1024)
    cur = list(lens)
    steps = []           # (q_start, slots, befores)
    members = [0, 1, 2, 3]
    for step in range(6):
        if step == 3:    # slot 5 joins with a 9-token chunk (chunked prefill on top of its cache), the rest decode
            slots = members + [5]
            new = [1] * len(members) + [9]
        else:
            slots = list(members)
            new = [1] * len(members)
        steps.append((list(np.concatenate([[0], np.cumsum(new)])), slots, [cur[i] for i in slots]))
        for i, n in zip(slots, new):
            cur[i] += n
        members = members[1:] + [(members[-1] + 1) % 5]      # one sequence leaves, another joins
    xs = [U.to_device(W.hidden_bits(s, int(q[-1]), step=60 + i, scale=1.0 / 16), False) for i, (q, _, _) in enumerate(steps)]
    ya = [x.clone() for x in xs]
    yb = [x.clone() for x in xs]
    torch.cuda.synchronize()
    for i, (q, slots, befores) in enumerate(steps):
        batch = a.batch(q, slots, befores)
        a.run_layers(0, s.L, batch, ya[i])
        a.sync()
        batch.close()
    held = None
    for i, (q, slots, befores) in enumerate(steps):          # no sync inside this loop
        if held is None:
            held = b.batch(q, slots, befores, storage=storage)
        else:
            held.rebuild(q, slots, befores)
        b.run_layers(0, s.L, held, yb[i], after_current_stream=False)
    b.sync()
    for i in range(len(steps)):
        assert torch.equal(ya[i].view(torch.int16), yb[i].view(torch.int16)), i
    # a description that does not fit the lent memory is refused and leaves the batch usable
    with pytest.raises(Exception) as ei:
        held.rebuild([0, 200000], [0], [0])              # 800 KB of per-token entries alone
    assert "BZ_ECAPACITY" in str(ei.value)
    with pytest.raises(Exception) as ei:
        a.batch([0, 1], [0], [0]).rebuild([0, 1], [0], [0])
    assert "BZ_ESTATE" in str(ei.value)
    held.close()
    # oracle: replay the same steps
    os_ = U.oracle_shape(s)
    wts = {l: U.oracle_weights(W.layer_weights_bits(s, l)) for l in range(s.L)}
    okv = O.OracleKV()
    for i, n in enumerate(lens):
        for l in range(s.L):
            kb, vb = W.kv_prefill_bits(s, l, i, n)
            okv.put(l, i, U.f64(kb), U.f64(vb))
    for i, (q, slots, befores) in enumerate(steps):
        xbits = W.hidden_bits(s, int(q[-1]), step=60 + i, scale=1.0 / 16)
        want = O.run_layers(os_, wts, 0, s.L, U.f64(xbits), O.OracleBatch([int(v) for v in q], slots, befores), okv)
        assert U.rel_err(U.from_device(yb[i]), want) <= U.BF16_TOL, i
    a.close(); b.close()


def test_batch_shared_by_two_instances_on_different_streams_without_host_syncs(torch):
    """A split pair with a compute stream each, one shared decode batch, five steps enqueued back to back:
    target runs [0,1) on its stream, hands over on the device, source runs [1,2) on its own stream and
    advances the shared batch there; the only host synchronisation is at the very end.  The library orders
    the advance behind the target's run and the target's next run behind the advance.  Output bits equal
    those of one instance running whole layers with a sync after every call."""
    s = SHAPE
    lens = [5, 255, 256, 300, 511, 700]
    B, steps = len(lens), 5
    st_t, st_s = torch.cuda.Stream(), torch.cuda.Stream()
    whole = _fresh(torch, s, lens, steps)
    tgt = _fresh(torch, s, lens, steps, layers=[0], stream=st_t)
    src = _fresh(torch, s, lens, steps, layers=[1], stream=st_s)
    xs = [U.to_device(W.hidden_bits(s, B, step=80 + i, scale=1.0 / 16), False) for i in range(steps)]
    want = [x.clone() for x in xs]
    got = [x.clone() for x in xs]
    bufs = [torch.zeros_like(x) for x in xs]
    torch.cuda.synchronize()
    bw = whole.batch(list(range(B + 1)), list(range(B)), lens)
    for i in range(steps):
        whole.run_layers(0, s.L, bw, want[i])
        whole.batch_advance(bw)
        whole.sync()
    shared = tgt.batch(list(range(B + 1)), list(range(B)), lens)
    for i in range(steps):                                   # nothing in this loop waits on the host
        tgt.run_layers(0, 1, shared, got[i], after_current_stream=False)
        tgt.export_boundary(got[i], B, bufs[i])             # device to device, on the target's stream
        src.wait_stream(st_t)                               # the source's stream waits for the hand-off
        src.import_boundary(got[i], B, bufs[i])
        src.run_layers(1, 2, shared, got[i], after_current_stream=False)
        src.batch_advance(shared)                           # on the source's stream
    tgt.sync(); src.sync()
    for i in range(steps):
        assert torch.equal(want[i].view(torch.int16), got[i].view(torch.int16)), i
    whole.close(); tgt.close(); src.close()


def test_run_layers_is_ordered_behind_the_callers_stream(torch):
    """The input is produced on torch's current stream by a long chain of kernels and handed to run_layers at
    once, with no synchronisation by the caller: the binding orders the compute stream behind the current
    stream, and signal_stream orders the reader behind the compute stream."""
    s = SHAPE
    lens = [64]
    inst = _fresh(torch, s, lens, 8)
    ref = _fresh(torch, s, lens, 8)
    base = U.to_device(W.hidden_bits(s, 1, step=90, scale=1.0 / 16), False)
    torch.cuda.synchronize()
    x = base.clone()
    big = torch.ones(64 << 20, dtype=torch.float32, device="cuda")
    for _ in range(20):
        big.mul_(1.0001)                                     # keeps the current stream busy for a while
    x.copy_(base * 2.0)                                      # the value run_layers must see
    batch = inst.batch([0, 1], [0], [64])
    inst.run_layers(0, s.L, batch, x)
    inst.signal_stream()
    out = x.clone()                                          # on the current stream, behind the compute stream
    torch.cuda.synchronize()
    y = (base * 2.0).clone()
    torch.cuda.synchronize()
    ref.run_layers(0, s.L, ref.batch([0, 1], [0], [64]), y)
    ref.sync()
    assert torch.equal(out.view(torch.int16), y.view(torch.int16))
    inst.close(); ref.close()


def test_ingest_sources_must_be_page_locked(torch):
    s = W.CONFIGS["tiny"]
    inst = U.make_instance(s, max_seqs=1, max_seq_len=64, max_tokens=16, kv_tokens=64)
    blob = inst.pack_layer(W.layer_weights_bits(s, 0))       # ordinary numpy memory
    with pytest.raises(Exception) as ei:
        inst.lib  # noqa: B018
        inst._check(inst.lib.bz_load_layer(inst.handle, 0, blob.ctypes.data, blob.size), "bz_load_layer")
    assert "BZ_EINVAL" in str(ei.value)
    assert inst.frontier() == 0 and not inst.layer_ready(0)
    pinned = inst.pinned_blob(blob)
    half = blob.size // 2 // 256 * 256
    with pytest.raises(Exception) as ei:                     # one shard from pageable memory
        from paper_2412_17246_amd.binding import bz_shard
        arr = (bz_shard * 2)(bz_shard(pinned.data_ptr(), 0, half, 0, 0),
                             bz_shard(blob.ctypes.data + half, half, blob.size - half, 0, 0))
        inst._check(inst.lib.bz_load_layer_sharded(inst.handle, 0, arr, 2), "bz_load_layer_sharded")
    assert "BZ_EINVAL" in str(ei.value)
    inst.load_layer(0, pinned)                               # the refusals left the layer requestable
    inst.wait_layer(0)
    assert np.array_equal(inst.readback_layer(0), blob)
    inst.drop_sources()
    assert not inst._keep
    inst.close()


def test_second_ingest_stream_lent_by_the_caller(torch):
    """Two instances take the same caller-made stream as their second ingest stream: layers loaded over two streams
    arrive bit for bit, the stream outlives the instances, and the instance's own streams are refused."""
    s = W.CONFIGS["tiny"]
    lent = torch.cuda.Stream()
    blobs, insts = [], []
    for k in range(2):
        inst = U.make_instance(s, max_seqs=1, max_seq_len=64, max_tokens=16, kv_tokens=64)
        inst.lend_second_copy_stream(lent)
        inst.lend_second_copy_stream(lent)                   # again: nothing to do
        inst.set_ingest_streams(2)
        for bad in (inst.copy_stream, inst.compute_stream):
            with pytest.raises(Exception) as ei:
                inst.lend_second_copy_stream(bad)
            assert "BZ_EINVAL" in str(ei.value)
        insts.append(inst)
    for l in range(s.L):
        blob = insts[0].pack_layer(W.layer_weights_bits(s, l))
        blobs.append(blob)
        for inst in insts:
            inst.load_layer(l, inst.pinned_blob(blob))
    for inst in insts:
        for l in range(s.L):
            inst.wait_layer(l)
            assert np.array_equal(inst.readback_layer(l), blobs[l])
        assert inst.frontier() == s.L
    # a stream the library made itself is replaced by the lent one (and destroyed); loading goes on over the new one
    own = U.make_instance(s, max_seqs=1, max_seq_len=64, max_tokens=16, kv_tokens=64)
    own.set_ingest_streams(2)
    own.load_layer(0, own.pinned_blob(blobs[0]))
    own.lend_second_copy_stream(lent)                        # waits for the halves still on the old stream
    own.load_layer(1, own.pinned_blob(blobs[1]))
    own.sync()
    assert np.array_equal(own.readback_layer(0), blobs[0]) and np.array_equal(own.readback_layer(1), blobs[1])
    for inst in insts + [own]:
        inst.close()
    with torch.cuda.stream(lent):                            # still a working stream
        t = torch.ones(8, device="cuda") * 3
    lent.synchronize()
    assert float(t.sum()) == 24.0


def test_batch_storage_bound_holds_for_the_extreme_batches(torch):
    """bz_batch_storage_bytes(max_seqs, max_tokens, max_seq_len) is enough for every batch within those limits:
    all sequences decoding on caches of the maximum length, one token per sequence of prefill, one long
    prefill, and the mix; a batch beyond the limits is refused, not truncated."""
    from paper_2412_17246_amd import load_library
    from paper_2412_17246_amd.binding import Batch
    lib = load_library(False)
    max_seqs, max_tokens, max_seq_len = 48, 4096, 2048
    n = int(lib.bz_batch_storage_bytes(max_seqs, max_tokens, max_seq_len))
    assert n > 0 and n % 32 == 0
    assert lib.bz_batch_storage_bytes(0, 1, 1) == 0 and lib.bz_batch_storage_bytes(1, 0, 1) == 0
    dev = torch.empty(n, dtype=torch.uint8, device="cuda")
    pinned = torch.empty(2 * n, dtype=torch.uint8, pin_memory=True)
    st = torch.cuda.Stream()
    slots = list(range(max_seqs))
    cases = [
        (list(range(max_seqs + 1)), slots, [max_seq_len - 1] * max_seqs),                 # all decode, longest caches
        ([0, max_tokens], [0], [0]),                                                       # one long prefill
        ([0] + [2 * (i + 1) for i in range(max_seqs)], slots, [0] * max_seqs),            # many two-token prefills
        ([0, max_tokens - (max_seqs - 1)] + [max_tokens - (max_seqs - 1) + i for i in range(1, max_seqs)], slots,
         [0] + [max_seq_len - 1] * (max_seqs - 1)),                                        # one prefill + the rest decoding
    ]
    held = None
    for q, sl, kb in cases:
        if held is None:
            held = Batch(lib, q, sl, kb, storage=(dev, pinned, st))
        else:
            held.rebuild(q, sl, kb)
        assert held.T == q[-1] and held.B == len(sl)
    st.synchronize()
    with pytest.raises(Exception) as ei:                                                   # 64 x the tokens the storage was sized for
        held.rebuild([0, 64 * max_tokens], [0], [0])
    assert "BZ_ECAPACITY" in str(ei.value)
    assert held.T == cases[-1][0][-1]                                                      # the refused description changed nothing
    held.close()
    with pytest.raises(Exception):                                                         # staging too small for two halves
        Batch(lib, [0, 1], [0], [0], storage=(dev, pinned[:n], st))
