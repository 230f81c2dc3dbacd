#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

Default workload `prefill_stream` (the configuration the headline metric is quoted on): a
Llama-2-7B-shaped decoder (32 layers) whose weights start in pinned host memory.  One step = scale
start to first token: every layer is requested with load_layer (chunked host->HBM copies on the
copy stream) and, at the same moment, one packed prefill batch of 8 requests (lognormal lengths)
is sent through run_layers(0, L), each layer gated on its own ingest event, so resident layers
execute while later ones are still arriving.  Hidden states, KV cache and workspaces are resident
in HBM before the timed region; the weights' trip over the host link is the method's own ingest
step and is inside it.  The all-resident rate of the same batch is reported beside it.

Other workloads (`--workload`), used for the design notes and profiles, not by the round driver:
  decode       8B-GQA-shaped, 64 sequences with caches of length uniform[256,4096]; a step is one
               decode step through all layers; `--split k` hands the activation from an instance
               running [0,k) to one running [k,L) every step and checks bit-equality first
  mixed_ttft   13B-shaped, layers [0,20) resident, [20,40) ingested from t0 while one mixed batch
               (16 prefill + 48 decode sequences) runs behind the frontier
  `--shape 70b --requests 4 --fixed-len 2048 --distinct-blobs 4` gives the 70B-shaped streamed
  prefill (layer i is fed from pinned blob i mod 4: byte counts and shapes are real, the host
  copy is smaller than 137 GB).

Prints ONE JSON line.  `--gpus N` with N > 1 is refused: this build is single-GPU by construction.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402

PEAK_BF16_TFLOPS = 2500.0     # MI355X dense bf16 MFMA
PEAK_HBM_GBPS = 8000.0
# Bytes moved per launch of the dominant kernel of the default workload (gate/up projection, M = 6768):
# rocprofv3 --pmc FETCH_SIZE and --pmc WRITE_SIZE of this script, scaled by what the same counters read for
# a 1 GiB device copy (x2.0 and x1.0); see profiles/gemm_big_kernel_7b_prefill_stream.txt.  L2-miss traffic
# summed over the 8 XCD L2s, mostly served by the Infinity Cache.
# The gate/up figure covers the three launches of that projection (whole tiles, split last-round tiles,
# their fix-up); the decode-attention figure covers the split-KV kernel and the combine.
MEASURED_TRAFFIC = {("7b", 32, 6768, "gemm_gateup"): 1.881e9 + 0.150e9 + 0.069e9 + 0.061e9 + 0.061e9,
                    ("8b_gqa", 32, 64, "attn_decode"): 0.5671e9 + 0.0114e9}


# ------------------------------------------------------------------------------- helpers

def with_layers(base, n_layers):
    if not n_layers:
        return base
    return W.DecoderShape(base.name, n_layers, base.H, base.Hq, base.Hkv, base.d, base.F, base.eps,
                          base.rope_base, base.seed)


def gen_layer_blob_gpu(torch, inst, shape, gen, pinned=True):
    """Draws one layer's nine tensors on the GPU (seeded) into a pinned host (or device) blob."""
    if pinned:
        blob = torch.empty(inst.layer_bytes, dtype=torch.uint8, pin_memory=True)
    else:
        blob = torch.empty(inst.layer_bytes, dtype=torch.uint8, device="cuda")
    view = blob.view(torch.bfloat16)
    for name, shp in W.tensor_shapes(shape).items():
        n = int(np.prod(shp))
        off = getattr(inst.layout, name) // 2
        step = 1 << 27
        for o in range(0, n, step):
            m = min(step, n - o)
            t = torch.randn(m, generator=gen, device="cuda", dtype=torch.float32) * 0.02
            if name in ("g1", "g2"):
                t += 1.0
            view[off + o:off + o + m].copy_(t.to(torch.bfloat16))
    return blob


def fill_kv(torch, inst, shape, gen, slot, length, layers=None):
    """Seeded N(0,1) K and V for positions [0, length) of the given layers (default all) of one slot."""
    for l in (range(shape.L) if layers is None else layers):
        k = torch.randn(length, shape.Hkv, shape.d, generator=gen, device="cuda").to(torch.bfloat16)
        v = torch.randn(length, shape.Hkv, shape.d, generator=gen, device="cuda").to(torch.bfloat16)
        torch.cuda.synchronize()
        inst.kv_write(l, slot, 0, length, k, v)
    inst.sync()


def oracle_threads():
    try:
        from threadpoolctl import threadpool_info
        return int(max([p.get("num_threads", 1) for p in threadpool_info()] or [1]))
    except Exception:
        return int(os.cpu_count() or 1)


def cpu_baseline_prefill(shape):
    """The CPU oracle (as it stands) on one layer of the real shape over a bounded sample: one
    request of n prompt tokens; reported as tokens/s through all L layers."""
    from oracle import decoder as O
    n = 256
    osh = O.OracleShape(L=shape.L, H=shape.H, Hq=shape.Hq, Hkv=shape.Hkv, d=shape.d, F=shape.F,
                        eps=shape.eps, rope_base=shape.rope_base)
    wts = {k: W.f32_from_bf16_bits(v).astype(np.float64) for k, v in W.layer_weights_bits(shape, 0).items()}
    x = W.f32_from_bf16_bits(W.hidden_bits(shape, n, step=0)).astype(np.float64)
    reps, used = 0, 0.0
    while reps < 1 or (used < 10.0 and reps < 64):
        t0 = time.perf_counter()
        O.run_layers(osh, {0: wts}, 0, 1, x, O.OracleBatch([0, n], [0], [0]), O.OracleKV())
        used += time.perf_counter() - t0
        reps += 1
    return {"value": n / (used / reps * shape.L), "unit": "tokens/s", "cores": oracle_threads(), "kind": "oracle",
            "sample": f"float64 numpy oracle, 1 layer of the {shape.name} shape, one request of {n} prompt tokens, "
                      f"{reps} repetitions, scaled by 1/L to whole-model tokens/s"}


def cpu_baseline_decode(shape, lens):
    """The CPU oracle on one decode step of one layer at the real batch and cache lengths."""
    from oracle import decoder as O
    B = len(lens)
    osh = O.OracleShape(L=shape.L, H=shape.H, Hq=shape.Hq, Hkv=shape.Hkv, d=shape.d, F=shape.F,
                        eps=shape.eps, rope_base=shape.rope_base)
    wts = {k: W.f32_from_bf16_bits(v).astype(np.float64) for k, v in W.layer_weights_bits(shape, 0).items()}
    rng = np.random.default_rng(5)
    x = W.f32_from_bf16_bits(W.hidden_bits(shape, B, step=0)).astype(np.float64)
    reps, used = 0, 0.0
    while reps < 1 or (used < 10.0 and reps < 16):
        kv = O.OracleKV()
        for i, n in enumerate(lens):
            kv.put(0, i, rng.standard_normal((int(n), shape.Hkv, shape.d)), rng.standard_normal((int(n), shape.Hkv, shape.d)))
        t0 = time.perf_counter()
        O.run_layers(osh, {0: wts}, 0, 1, x, O.OracleBatch(list(range(B + 1)), list(range(B)), [int(n) for n in lens]), kv)
        used += time.perf_counter() - t0
        reps += 1
    return {"value": B / (used / reps * shape.L), "unit": "tokens/s", "cores": oracle_threads(), "kind": "oracle",
            "sample": f"float64 numpy oracle, 1 layer of the {shape.name} shape, one decode step of {B} sequences at the "
                      f"benchmark's cache lengths, {reps} repetitions, scaled by 1/L to whole-model tokens/s"}


def pick_ingest_streams(args, inst, reset, one_step, torch):
    """Untimed, after the warm-up steps: steps with the layers travelling on one copy stream and on two,
    on the benchmark's own host buffers; the faster setting is kept for the timed steps.  (Two
    concurrent transfers usually keep the host link busier, but from some pinned allocations they are
    slower than one, and a compute-bound step does not gain from them.)"""
    if args.ingest_streams:
        inst.set_ingest_streams(args.ingest_streams)
        return args.ingest_streams
    took = {}
    if args.warmup == 0:                  # nothing has run yet: the first trial must not carry the one-time costs
        reset()
        one_step()
        inst.sync()
    for n in (1, 2):
        inst.set_ingest_streams(n)
        for trial in range(2):            # the first step on a setting carries its one-time costs: keep the second
            reset()
            t0 = time.perf_counter()
            one_step()
            inst.sync()
            torch.cuda.synchronize()
            took[n] = time.perf_counter() - t0
    best = 2 if took[2] < took[1] else 1
    inst.set_ingest_streams(best)
    return best


def base_record(metric, value, unit, args, ms_per_step, workload, extra_cfg):
    cfg = {"workload": workload}
    cfg.update(extra_cfg)
    return {"metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic", "config": cfg}


def gemm_roofline(prof):
    classes = [k for k in prof if k.startswith("gemm") and prof[k]["launches"]]
    dom = max(classes, key=lambda k: prof[k]["ms"])
    d = prof[dom]
    achieved = d["flops"] / (d["ms"] * 1e-3) / 1e12
    allf = sum(prof[k]["flops"] for k in classes)
    allms = sum(prof[k]["ms"] for k in classes)
    return ({"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
             "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None, "launches": d["launches"],
             "avg_ms": d["ms"] / d["launches"]},
            allf / (allms * 1e-3) / 1e12)


# ------------------------------------------------------------------------------- workloads

def run_prefill_stream(args, torch, Instance):
    base = W.CONFIGS[args.shape]
    shape = with_layers(base, args.layers)
    if args.fixed_len:
        lens = np.full(args.requests, args.fixed_len, dtype=np.int64)
    else:
        lens = W.lognormal_lengths(shape.seed, args.requests, 512.0, 0.6, 16, 2048)
    q_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, B = int(q_start[-1]), len(lens)
    stream = torch.cuda.Stream()
    inst = Instance(shape, max_seqs=B, max_seq_len=int(lens.max()) + 1, max_tokens=T,
                    kv_tokens=int(lens.sum()) + 32 * B, chunk_bytes=args.chunk_mib << 20, compute_stream=stream)
    for i, n in enumerate(lens):
        inst.kv_reserve(i, int(n))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(shape.seed)
    n_blobs = min(shape.L, args.distinct_blobs) if args.distinct_blobs else shape.L
    blobs = [gen_layer_blob_gpu(torch, inst, shape, gen) for _ in range(n_blobs)]
    shard_views = []
    if args.shards > 1:
        step = -(-inst.layer_bytes // args.shards // 256) * 256
        for b in blobs:
            shard_views.append([(b[o:min(o + step, inst.layer_bytes)], o) for o in range(0, inst.layer_bytes, step)])
    x0 = torch.from_numpy(W.hidden_bits(shape, T, step=0).view(np.int16).copy()).view(torch.bfloat16).cuda()
    x = torch.empty_like(x0)
    batch = inst.batch(q_start, list(range(B)), [0] * B)
    torch.cuda.synchronize()

    def one_step():                       # scale start -> first token; returns once everything is enqueued
        inst.reset_clock()
        for l in range(shape.L):
            if args.shards > 1:           # the same bytes as k parallel shards (section 5.1, sharded transfer)
                inst.load_layer_sharded(l, shard_views[l % n_blobs])
            else:
                inst.load_layer(l, blobs[l % n_blobs])
        inst.run_layers(0, shape.L, batch, x)

    def reset():
        for l in range(shape.L):
            inst.unload_layer(l)
        x.copy_(x0)
        torch.cuda.synchronize()

    for _ in range(args.warmup):
        reset()
        one_step()
        inst.sync()
    n_streams = pick_ingest_streams(args, inst, reset, one_step, torch)
    inst.profile_enable(True)
    inst.profile_read()
    total, ingest_ms = 0.0, []
    for _ in range(args.steps):           # resets are outside the clock
        reset()
        t0 = time.perf_counter()
        one_step()
        inst.sync()
        torch.cuda.synchronize()
        total += time.perf_counter() - t0
        ingest_ms.append(inst.layer_ready_ms(shape.L - 1))
    prof = inst.profile_read()
    inst.profile_enable(False)
    ms_per_step = total / args.steps * 1e3

    x.copy_(x0)                           # all layers resident: compute-only rate of the same batch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        inst.run_layers(0, shape.L, batch, x)
    inst.sync()
    resident_s = (time.perf_counter() - t0) / 3

    roof, all_tf = gemm_roofline(prof)
    roof["traffic"] = MEASURED_TRAFFIC.get((shape.name, shape.L, T, roof["kernel"]))
    out = base_record("prefill tokens/s on partially loaded model", T * args.steps / total, "tokens/s", args,
                      ms_per_step,
                      f"{shape.name}-shaped decoder, {shape.L} layers streamed from pinned host memory while a packed "
                      f"prefill batch of {B} requests ({T} tokens) runs behind the frontier",
                      {"shape": shape.name, "layers": shape.L, "requests": B, "tokens": T,
                       "lengths": [int(v) for v in lens], "distinct_host_blobs": n_blobs,
                       "shards_per_layer": max(1, args.shards), "ingest_streams": n_streams})
    out.update({
        "ttft_ms": ms_per_step,
        "ingest_GBps": shape.L * inst.layer_bytes / (float(np.median(ingest_ms)) * 1e-3) / 1e9,
        "resident_prefill_tokens_per_s": T / resident_s,
        "resident_ms": resident_s * 1e3,
        "gemm_TFLOPs_all_classes": all_tf,
        "kernel_ms_per_step": {k: v["ms"] / args.steps for k, v in prof.items() if v["launches"]},
        "roofline": roof,
    })
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_prefill(base)
    inst.close()
    return out


def run_decode(args, torch, Instance):
    base = W.CONFIGS[args.shape if args.shape != "7b" else "8b_gqa"]
    shape = with_layers(base, args.layers)
    B = args.requests if args.requests != 8 else 64
    lo, hi = (512, 4096) if base.name == "70b" else (256, 4096)
    lens = W.uniform_lengths(base.seed, B, lo, hi)
    if args.fixed_len:                    # every cache the same length (no short sequences, no ragged last chunks)
        lens = np.full(B, args.fixed_len, dtype=np.int64)
        lo = hi = args.fixed_len
    n_steps = 2 * args.steps + args.warmup + 4     # every step appends a position: profiled steps, then the timed ones
    stream = torch.cuda.Stream()
    gen = torch.Generator(device="cuda")
    gen.manual_seed(base.seed)

    def make_instance():
        inst = Instance(shape, max_seqs=B, max_seq_len=hi + n_steps + 8, max_tokens=B,
                        kv_tokens=int(lens.sum()) + B * (n_steps + 40), compute_stream=stream)
        for i, n in enumerate(lens):
            inst.kv_reserve(i, int(n) + n_steps + 8)
        return inst

    inst = make_instance()
    blobs = []
    for l in range(shape.L):
        blob = gen_layer_blob_gpu(torch, inst, shape, gen, pinned=False)
        torch.cuda.synchronize()
        inst.load_layer_from_device(l, blob)
        inst.sync()
        if args.split:
            blobs.append(blob)            # the split pair loads the same bytes later
        else:
            inst._keep.clear()            # layer is resident: the staging blob can go
            del blob
    gen_kv = torch.Generator(device="cuda")
    gen_kv.manual_seed(base.seed + 100)
    for i, n in enumerate(lens):
        fill_kv(torch, inst, shape, gen_kv, i, int(n))
    xs = torch.randn(n_steps, B, shape.H, generator=gen, device="cuda").to(torch.bfloat16)
    batch = inst.batch(list(range(B + 1)), list(range(B)), [int(n) for n in lens])
    torch.cuda.synchronize()

    split_note = None
    start = 0
    if args.split:
        # live split (cooperative execution): the target instance runs layers [0,k) with its own caches,
        # hands the activation over, the source instance runs [k,L) with its own; outputs are compared
        # bit for bit with the unsplit instance over 4 steps
        k = args.split
        tgt, src = make_instance(), make_instance()
        for l in range(shape.L):
            (tgt if l < k else src).load_layer_from_device(l, blobs[l])
        tgt.sync()
        src.sync()
        gen_kv.manual_seed(base.seed + 100)
        for i, n in enumerate(lens):
            for l in range(shape.L):
                kk = torch.randn(int(n), shape.Hkv, shape.d, generator=gen_kv, device="cuda").to(torch.bfloat16)
                vv = torch.randn(int(n), shape.Hkv, shape.d, generator=gen_kv, device="cuda").to(torch.bfloat16)
                torch.cuda.synchronize()
                (tgt if l < k else src).kv_write(l, i, 0, int(n), kk, vv)
        tgt.sync()
        src.sync()
        batch2 = tgt.batch(list(range(B + 1)), list(range(B)), [int(n) for n in lens])
        buf = torch.empty(B, shape.H, dtype=torch.bfloat16, device="cuda")
        ok = True
        for st in range(4):
            a = xs[st].clone()
            b = xs[st].clone()
            c = torch.empty_like(b)
            torch.cuda.synchronize()
            inst.run_layers(0, shape.L, batch, a)
            inst.batch_advance(batch)
            tgt.run_layers(0, k, batch2, b)
            tgt.export_boundary(b, B, buf)
            src.import_boundary(c, B, buf)        # both instances share the compute stream: ordered
            src.run_layers(k, shape.L, batch2, c)
            src.batch_advance(batch2)
            inst.sync()
            src.sync()
            ok = ok and torch.equal(a.view(torch.int16), c.view(torch.int16))
        split_note = {"split_layer": k, "bit_exact_steps": 4, "bit_exact": bool(ok)}
        tgt.close()
        src.close()
        if not ok:
            raise SystemExit("split run is not bit-exact")
        start = 4

    for st in range(start, start + args.warmup):
        inst.run_layers(0, shape.L, batch, xs[st])
        inst.batch_advance(batch)
    inst.sync()
    inst.profile_enable(True)
    inst.profile_read()
    t0 = time.perf_counter()
    for st in range(start + args.warmup, start + args.warmup + args.steps):
        inst.run_layers(0, shape.L, batch, xs[st % n_steps])
        inst.batch_advance(batch)
    inst.sync()
    torch.cuda.synchronize()
    total = time.perf_counter() - t0
    prof = inst.profile_read()
    inst.profile_enable(False)

    # the profiled steps pay two events per kernel; time the same number of steps again without them
    t0 = time.perf_counter()
    for st in range(args.steps):
        inst.run_layers(0, shape.L, batch, xs[st % n_steps])
        inst.batch_advance(batch)
    inst.sync()
    plain = time.perf_counter() - t0

    d = prof["attn_decode"]
    achieved = d["bytes"] / (d["ms"] * 1e-3) / 1e9
    out = base_record("decode tokens/s", B * args.steps / plain, "tokens/s", args, plain / args.steps * 1e3,
                      f"{shape.name}-shaped decoder, {shape.L} layers resident, continuous decode of {B} sequences "
                      f"with cache lengths uniform[{lo},{hi}]",
                      {"shape": shape.name, "layers": shape.L, "sequences": B, "mean_cache_len": float(lens.mean())})
    out.update({
        "ms_per_step_with_profiling_events": total / args.steps * 1e3,
        "weights_GB_per_step": shape.L * inst.layer_bytes / 1e9,
        "kv_GB_per_step": d["bytes"] / args.steps / 1e9,
        "kernel_ms_per_step": {k: v["ms"] / args.steps for k, v in prof.items() if v["launches"]},
        "roofline": {"bound": "hbm", "kernel": "attn_decode", "achieved": achieved, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBPS,
                     "traffic": MEASURED_TRAFFIC.get((shape.name, shape.L, B, "attn_decode")), "launches": d["launches"],
                     "avg_ms": d["ms"] / d["launches"]},
    })
    if split_note:
        out["split"] = split_note
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_decode(base, lens)
    inst.close()
    return out


def run_mixed_ttft(args, torch, Instance):
    base = W.CONFIGS["13b"]
    shape = with_layers(base, args.layers)
    resident = shape.L // 2
    p_lens = W.lognormal_lengths(base.seed, 16, 768.0, 0.6, 32, 4096)
    d_lens = W.uniform_lengths(base.seed, 48, 128, 2048)
    lens_new = [int(n) for n in p_lens] + [1] * 48
    befores = [0] * 16 + [int(n) for n in d_lens]
    q_start = np.concatenate([[0], np.cumsum(lens_new)]).astype(np.int32)
    T, B = int(q_start[-1]), len(lens_new)
    caps = [n + b for n, b in zip(lens_new, befores)]
    stream = torch.cuda.Stream()
    inst = Instance(shape, max_seqs=B, max_seq_len=max(caps) + 1, max_tokens=T, kv_tokens=sum(caps) + 32 * B,
                    chunk_bytes=args.chunk_mib << 20, compute_stream=stream)
    for i, c in enumerate(caps):
        inst.kv_reserve(i, c)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(base.seed)
    blobs = [gen_layer_blob_gpu(torch, inst, shape, gen) for _ in range(shape.L)]
    for i in range(16, B):
        fill_kv(torch, inst, shape, gen, i, befores[i])
    x0 = torch.from_numpy(W.hidden_bits(shape, T, step=0).view(np.int16).copy()).view(torch.bfloat16).cuda()
    x = torch.empty_like(x0)
    batch = inst.batch(q_start, list(range(B)), befores)
    for l in range(resident):
        inst.load_layer(l, blobs[l])
    inst.sync()

    def reset():
        for l in range(resident, shape.L):
            inst.unload_layer(l)
        x.copy_(x0)
        torch.cuda.synchronize()

    def one_step():
        inst.reset_clock()
        for l in range(resident, shape.L):
            inst.load_layer(l, blobs[l])
        inst.run_layers(0, shape.L, batch, x)

    for _ in range(args.warmup):
        reset()
        one_step()
        inst.sync()
    n_streams = pick_ingest_streams(args, inst, reset, one_step, torch)
    inst.profile_enable(True)
    inst.profile_read()
    total, ingest_ms = 0.0, []
    for _ in range(args.steps):
        reset()
        t0 = time.perf_counter()
        one_step()
        inst.sync()
        torch.cuda.synchronize()
        total += time.perf_counter() - t0
        ingest_ms.append(inst.layer_ready_ms(shape.L - 1))
    prof = inst.profile_read()
    inst.profile_enable(False)
    ttft = total / args.steps * 1e3
    compute_ms = sum(v["ms"] for v in prof.values()) / args.steps
    ing = float(np.median(ingest_ms))
    roof, all_tf = gemm_roofline(prof)
    out = base_record("prefill tokens/s on partially loaded model", T * args.steps / total, "tokens/s", args, ttft,
                      f"{shape.name}-shaped decoder, layers [0,{resident}) resident and [{resident},{shape.L}) ingested from "
                      f"scale start while one mixed batch (16 prefill requests + 48 decode sequences, {T} rows) runs",
                      {"shape": shape.name, "layers": shape.L, "rows": T, "prefill_lengths": [int(n) for n in p_lens],
                       "ingest_streams": n_streams})
    out.update({"ttft_ms": ttft, "ingest_ms": ing,
                "ingest_GBps": (shape.L - resident) * inst.layer_bytes / (ing * 1e-3) / 1e9,
                "kernel_ms_sum_per_step": compute_ms, "overlap_efficiency": max(ing, compute_ms) / ttft,
                "gemm_TFLOPs_all_classes": all_tf,
                "kernel_ms_per_step": {k: v["ms"] / args.steps for k, v in prof.items() if v["launches"]},
                "roofline": roof})
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_prefill(base)
    inst.close()
    return out


def run_zigzag(args, torch, Instance):
    """Several queued prefill batches (2000 tokens each, the batch size of the paper's example) served by a
    loaded source instance and a target instance whose layers stream in from pinned host memory, under the
    ZigZag or the best-effort policy.  Both instances share this one GPU, so the run shows correctness and
    scheduling overhead, not the two-GPU throughput gain."""
    from paper_2412_17246_amd import BZ_ZZ_BEST_EFFORT, BZ_ZZ_ZIGZAG, Scheduler
    base = W.CONFIGS[args.shape]
    shape = with_layers(base, args.layers)
    n_req, tok = args.requests if args.requests != 8 else 6, args.fixed_len or 2000
    stream_t, stream_s = torch.cuda.Stream(), torch.cuda.Stream()

    def make(stream):
        inst = Instance(shape, max_seqs=n_req, max_seq_len=tok + 1, max_tokens=tok, kv_tokens=n_req * (tok + 32),
                        chunk_bytes=args.chunk_mib << 20, compute_stream=stream)
        for r in range(n_req):
            inst.kv_reserve(r, tok)
        return inst

    tgt, src = make(stream_t), make(stream_s)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(base.seed)
    blobs = [gen_layer_blob_gpu(torch, tgt, shape, gen) for _ in range(shape.L)]
    for l in range(shape.L):
        src.load_layer(l, blobs[l])
    src.sync()
    x0 = [torch.from_numpy(W.hidden_bits(shape, tok, step=r).view(np.int16).copy()).view(torch.bfloat16).cuda()
          for r in range(n_req)]
    results = {}
    for name, policy in (("zigzag", BZ_ZZ_ZIGZAG), ("best_effort", BZ_ZZ_BEST_EFFORT)):
        times = []
        for it in range(args.warmup + args.steps):
            for l in range(shape.L):
                tgt.unload_layer(l)
            xt = [x.clone() for x in x0]
            xs = [torch.empty_like(x) for x in x0]
            sched = Scheduler(tgt, src, policy)
            batches = [tgt.batch([0, tok], [r], [0]) for r in range(n_req)]
            for r in range(n_req):
                sched.submit(batches[r], xt[r], xs[r])
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for l in range(shape.L):
                tgt.load_layer(l, blobs[l])
            sched.run()
            dt = time.perf_counter() - t0
            if it >= args.warmup:
                times.append(dt)
            cfgs = [sched.layers_on_target(r) for r in range(n_req)]
            n_events = len(sched.trace())
            sched.close()
        results[name] = {"ms": float(np.mean(times)) * 1e3, "layers_on_target": cfgs, "decisions": n_events}
    zz = results["zigzag"]
    out = base_record("prefill tokens/s on partially loaded model", n_req * tok / (zz["ms"] * 1e-3), "tokens/s", args,
                      zz["ms"],
                      f"{shape.name}-shaped decoder, {n_req} queued prefill batches of {tok} tokens, source instance resident, "
                      f"target instance streaming {shape.L} layers from pinned host memory, ZigZag policy (one GPU shared)",
                      {"shape": shape.name, "layers": shape.L, "requests": n_req, "tokens_per_request": tok})
    out["policies"] = results
    tgt.close()
    src.close()
    return out


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None)
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--workload", default="prefill_stream", choices=["prefill_stream", "decode", "mixed_ttft", "zigzag"])
    ap.add_argument("--shape", default="7b", choices=list(W.CONFIGS))
    ap.add_argument("--layers", type=int, default=0, help="use only the first N layers of the shape (debugging)")
    ap.add_argument("--requests", type=int, default=8)
    ap.add_argument("--fixed-len", type=int, default=0, help="prefill_stream: every request has this many tokens; decode: every cache has this length")
    ap.add_argument("--distinct-blobs", type=int, default=0, help="prefill_stream: feed layer i from pinned blob i mod m")
    ap.add_argument("--ingest-streams", type=int, default=0, choices=[0, 1, 2],
                    help="copy streams a layer travels on (0 = try both after warm-up and keep the faster)")
    ap.add_argument("--shards", type=int, default=1, help="prefill_stream: ingest every layer as this many parallel shards")
    ap.add_argument("--split", type=int, default=0, help="decode: also run a live split at this layer and compare bits")
    ap.add_argument("--chunk-mib", type=int, default=0, help="ingest chunk size in MiB (0 = library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2
    if args.steps is None:
        args.steps = 128 if args.workload == "decode" else 5
    if args.warmup is None:
        args.warmup = 8 if args.workload == "decode" else 2

    import torch
    from paper_2412_17246_amd import Instance

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    fn = {"prefill_stream": run_prefill_stream, "decode": run_decode, "mixed_ttft": run_mixed_ttft,
          "zigzag": run_zigzag}[args.workload]
    print(json.dumps(fn(args, torch, Instance)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
