"""The two-instance request scheduler on the GPU: whatever schedule real timing produces, every
request's output must equal the unsplit run bit for bit, every layer must run exactly once and in
order, and the target may only run layers that were resident when the decision was taken."""
import numpy as np
import pytest

import workloads as W
from tests import _util as U

pytestmark = pytest.mark.gpu

SHAPE = W.DecoderShape("zz", L=6, H=512, Hq=8, Hkv=2, d=128, F=1024, rope_base=500000.0, seed=41)
REQS = [(70, 45), (130, 3), (33, 200), (64, 64), (257, 1)]       # two prompts per request batch


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


def _instance(n_slots, tokens):
    return U.make_instance(SHAPE, max_seqs=n_slots, max_seq_len=512, max_tokens=max(a + b for a, b in REQS),
                           kv_tokens=tokens)


@pytest.mark.parametrize("policy_name", ["zigzag", "best_effort"])
def test_scheduler_outputs_are_bit_exact_and_trace_is_valid(torch, policy_name):
    from paper_2412_17246_amd import BZ_ZZ_BEST_EFFORT, BZ_ZZ_ZIGZAG, Scheduler
    policy = BZ_ZZ_ZIGZAG if policy_name == "zigzag" else BZ_ZZ_BEST_EFFORT
    s, L = SHAPE, SHAPE.L
    n_slots = 2 * len(REQS)
    tokens = sum((a + 31) // 32 * 32 + (b + 31) // 32 * 32 for a, b in REQS) + 64
    bits = {l: W.layer_weights_bits(s, l) for l in range(L)}

    # reference: one fully loaded instance, every request unsplit
    ref = _instance(n_slots, tokens)
    blobs = {l: ref.pinned_blob(ref.pack_layer(bits[l])) for l in range(L)}
    for l in range(L):
        ref.load_layer(l, blobs[l])
    want, inputs = [], []
    for r, (a, b) in enumerate(REQS):
        ref.kv_reserve(2 * r, a)
        ref.kv_reserve(2 * r + 1, b)
        xb = W.hidden_bits(s, a + b, step=60 + r)
        inputs.append(xb)
        x = U.to_device(xb, False)
        torch.cuda.synchronize()
        ref.run_layers(0, L, ref.batch([0, a, a + b], [2 * r, 2 * r + 1], [0, 0]), x)
        ref.sync()
        want.append(x.view(torch.int16).cpu().numpy().copy())
    ref.close()

    src, tgt = _instance(n_slots, tokens), _instance(n_slots, tokens)
    for l in range(L):
        src.load_layer(l, blobs[l])
    src.sync()
    for inst in (src, tgt):
        for r, (a, b) in enumerate(REQS):
            inst.kv_reserve(2 * r, a)
            inst.kv_reserve(2 * r + 1, b)
    sched = Scheduler(tgt, src, policy)
    outs = []
    for r, (a, b) in enumerate(REQS):
        xt = U.to_device(inputs[r], False)
        xs = torch.zeros_like(xt)
        outs.append(xs)
        sched.submit(tgt.batch([0, a, a + b], [2 * r, 2 * r + 1], [0, 0]), xt, xs)
    # slow the target's ingest down: a large dummy host->device copy on its copy stream before each layer
    big_host = torch.empty(96 << 20, dtype=torch.uint8, pin_memory=True)
    big_dev = torch.empty(96 << 20, dtype=torch.uint8, device="cuda")
    torch.cuda.synchronize()
    for l in range(L):
        if l > 0:
            with torch.cuda.stream(tgt.copy_stream):
                big_dev.copy_(big_host, non_blocking=True)
        tgt.load_layer(l, blobs[l])
    sched.run()
    tgt.sync()
    src.sync()
    for r in range(len(REQS)):
        assert np.array_equal(outs[r].view(torch.int16).cpu().numpy(), want[r]), r

    trace = sched.trace()
    for r in range(len(REQS)):
        ev = [e for e in trace if e["request"] == r]
        on_t = [e for e in ev if e["instance"] == 0]
        on_s = [e for e in ev if e["instance"] == 1]
        T = sched.layers_on_target(r)
        nxt = 0
        for e in on_t:                                    # target: consecutive layers, each resident when chosen
            assert e["layer_a"] == nxt and e["layer_b"] > e["layer_a"] and e["layer_b"] <= e["frontier"]
            nxt = e["layer_b"]
        assert nxt == T
        if T < L:
            assert len(on_s) == 1 and (on_s[0]["layer_a"], on_s[0]["layer_b"]) == (T, L)
        if policy == BZ_ZZ_ZIGZAG:
            assert all(e["layer_b"] - e["layer_a"] == 1 for e in on_t)
        else:
            assert 1 <= T <= L // 2
    src_order = [e["request"] for e in trace if e["instance"] == 1]
    assert src_order == sorted(src_order)                 # the source serves requests in arrival order
    assert tgt.frontier() == L
    sched.close(); tgt.close(); src.close()
