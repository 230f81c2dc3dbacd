#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

Default (`--workload all`, what the round driver runs): ONE JSON line whose headline is the largest
single-GPU configuration, with the other configurations as extra keys of the same line.

  headline  70B-shaped decoder (80 layers, 136.9 GB of weights) streamed from pinned host memory behind a
            4 x 2048-token prefill batch.  One step = scale start to first token: every layer is requested
            with load_layer (chunked host->HBM copies on the copy stream) and, at the same moment, the packed
            batch is sent through run_layers(0, L), each layer gated on its own ingest event, so resident
            layers execute while later ones are still arriving.  Hidden states, KV cache and workspaces are
            resident in HBM before the timed region; the weights' trip over the host link is the method's own
            ingest step and is inside it.  Layer i is fed from pinned blob i mod 4 (the host copy of all 80
            would be 137 GB): byte counts and shapes are real.  `--steps` / `--warmup` apply to this leg.
  configs.cfg5_70b_decode      the same instance, all layers now resident: 256 decode steps of 32 sequences
                               with caches uniform[512,4096]
  configs.cfg2_7b_prefill_stream   7B-shaped, 32 layers streamed behind an 8-request prefill batch (6768 tokens)
  configs.cfg3_8b_gqa_decode   8B-GQA-shaped, 64 sequences, caches uniform[256,4096], 128 decode steps, with a
                               live split at layer 16 (two instance handles) checked bit for bit first
  configs.cfg4_13b_mixed_ttft  13B-shaped, layers [0,20) resident, [20,40) ingested from t0 behind one mixed
                               batch (16 prefill requests + 48 decode sequences): TTFT, overlap efficiency

Single legs (`--workload prefill_stream | decode | mixed_ttft | zigzag`) are what the profiles under
profiles/ were taken with; see each file for its command.

Prints ONE JSON line on stdout (progress goes to stderr).  `--gpus N` with N > 1 is refused: this build is
single-GPU by construction.
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
# HBM-side traffic per launch of a dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this
# script, each scaled by what the same counter reads for a device copy of known size.  Keyed by (shape, rows,
# kernel class); the value names the summary under profiles/ that holds the counters and the command.  A
# workload without an entry reports "traffic": null.  The algorithmic bytes are computed, not looked up.
MEASURED_TRAFFIC = {
    # gate/up projection of the large-tile kernel: L2-miss traffic summed over the eight XCD L2s (FETCH_SIZE) plus
    # bytes written (WRITE_SIZE); most of the fetches are served by the Infinity Cache, the counters cannot tell
    ("70b", 8192, "gemm_gateup"): (11.283e9 + 0.470e9, "profiles/gemm_big_kernel_prefill_counters.txt"),
    ("7b", 6768, "gemm_gateup"): (1.881e9 + 0.149e9 + 0.069e9 + 0.051e9 + 0.051e9 + 0.001e9,
                                  "profiles/gemm_big_kernel_prefill_counters.txt"),
    ("13b", 11970, "gemm_gateup"): (5.582e9 + 0.331e9, "profiles/gemm_big_kernel_prefill_counters.txt"),
    # decode attention: split-KV kernel (fetch + partial results written) and the combine's fetch
    ("8b_gqa", 64, "attn_decode"): (0.5671e9 + 0.0098e9 + 0.0113e9, "profiles/attn_decode_and_skinny_gemm_decode_counters.txt"),
    ("70b", 32, "attn_decode"): (0.2936e9 + 0.0101e9 + 0.0117e9, "profiles/attn_decode_and_skinny_gemm_decode_counters.txt"),
}


def traffic_of(shape_name, rows, kernel):
    hit = MEASURED_TRAFFIC.get((shape_name, rows, kernel))
    return (hit[0], hit[1]) if hit else (None, None)


_STREAMS = {}


def bench_streams(torch):
    """One compute stream and two copy streams for the whole process, shared by every instance the benchmark
    creates.  A process has four hardware queues and the runtime deals streams onto them as they are created:
    an instance whose copy stream lands on the queue of its compute stream runs its copies and its kernels one
    after the other (measured: the 7B-shaped streamed prefill took ingest + compute, 313 ms, instead of 233 ms,
    when its streams were the eighth and ninth the process had created)."""
    if not _STREAMS:
        _STREAMS["compute"] = torch.cuda.Stream()
        _STREAMS["copy"] = torch.cuda.Stream()
        _STREAMS["copy2"] = torch.cuda.Stream()
    return _STREAMS["compute"], _STREAMS["copy"]


def lend_second_copy_stream(inst, torch):
    """The process-wide second ingest stream (see bench_streams) for an instance that loads from the host."""
    bench_streams(torch)
    inst.lend_second_copy_stream(_STREAMS["copy2"])


def note(msg):
    print(f"[bench {time.strftime('%H:%M:%S')}] {msg}", file=sys.stderr, flush=True)


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
    note(f"a streamed step took {took[1] * 1e3:.1f} ms with one copy stream, {took[2] * 1e3:.1f} ms with two")
    inst.set_ingest_streams(best)
    return best


def base_record(metric, value, unit, args, ms_per_step, workload, extra_cfg):
    cfg = {"workload": workload}
    cfg.update(extra_cfg)
    return {"metric": metric, "value": value, "unit": unit, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
            "dtype": "bf16", "data": "synthetic", "config": cfg}


def gemm_roofline(prof, shape_name, rows):
    """Roofline record of the GEMM class with the largest summed time, from the library's own HIP events on
    the compute stream (bz_profile_*), plus the rate over all GEMM classes."""
    classes = [k for k in prof if k.startswith("gemm") and prof[k]["launches"]]
    dom = max(classes, key=lambda k: prof[k]["ms"])
    d = prof[dom]
    achieved = d["flops"] / (d["ms"] * 1e-3) / 1e12
    allf = sum(prof[k]["flops"] for k in classes)
    allms = sum(prof[k]["ms"] for k in classes)
    traffic, source = traffic_of(shape_name, rows, dom)
    per_class = {k: prof[k]["flops"] / (prof[k]["ms"] * 1e-3) / 1e12 / PEAK_BF16_TFLOPS for k in classes}
    return ({"bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
             "frac": achieved / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_profile": source,
             "algorithmic_bytes": d["bytes"] / d["launches"], "algorithmic_flops": d["flops"] / d["launches"],
             "launches": d["launches"], "avg_ms": d["ms"] / d["launches"], "frac_by_class": per_class},
            allf / (allms * 1e-3) / 1e12)


def decode_leg(inst, torch, shape, batch, xs, n_steps, steps, warmup, start, B):
    """Timed decode steps on a resident instance: `steps` steps with the library's per-kernel events (for the
    roofline record), then the same number without them (the reported rate)."""
    for st in range(start, start + warmup):
        inst.run_layers(0, shape.L, batch, xs[st % n_steps], after_current_stream=False)
        inst.batch_advance(batch)
    inst.sync()
    inst.profile_enable(True)
    inst.profile_read()
    t0 = time.perf_counter()
    for st in range(start + warmup, start + warmup + steps):
        inst.run_layers(0, shape.L, batch, xs[st % n_steps], after_current_stream=False)
        inst.batch_advance(batch)
    inst.sync()
    torch.cuda.synchronize()
    total = time.perf_counter() - t0
    prof = inst.profile_read()
    inst.profile_enable(False)
    t0 = time.perf_counter()
    for st in range(steps):
        inst.run_layers(0, shape.L, batch, xs[st % n_steps], after_current_stream=False)
        inst.batch_advance(batch)
    inst.sync()
    plain = time.perf_counter() - t0
    d = prof["attn_decode"]
    achieved = d["bytes"] / (d["ms"] * 1e-3) / 1e9
    traffic, source = traffic_of(shape.name, B, "attn_decode")
    weights_gb = shape.L * inst.layer_bytes / 1e9
    kv_gb = d["bytes"] / steps / 1e9
    return {
        "decode_tokens_per_s": B * steps / plain,
        "ms_per_step": plain / steps * 1e3,
        "steps": steps,
        "ms_per_step_with_profiling_events": total / steps * 1e3,
        "weights_GB_per_step": weights_gb,
        "kv_GB_per_step": kv_gb,
        "hbm_roofline_frac_whole_step": (weights_gb + kv_gb) / (plain / steps) / PEAK_HBM_GBPS,
        "kernel_ms_per_step": {k: v["ms"] / steps for k, v in prof.items() if v["launches"]},
        "roofline": {"bound": "hbm", "kernel": "attn_decode", "achieved": achieved, "peak": PEAK_HBM_GBPS, "unit": "GB/s",
                     "frac": achieved / PEAK_HBM_GBPS, "traffic": traffic, "traffic_profile": source,
                     "algorithmic_bytes": d["bytes"] / d["launches"], "launches": d["launches"],
                     "avg_ms": d["ms"] / d["launches"]},
    }


def live_split_check(torch, make_instance, shape, blobs, lens, kv_seed, xs, k, steps, whole=None, whole_batch=None):
    """Cooperative execution at the real shape: a target instance holding layers [0,k) and a source instance
    holding [k,L), each with the caches of its own layers, against one instance holding everything.  Every
    step hands the activation over at the boundary and advances the caches by one position.  Returns the list
    of per-step bit-equality flags.  `whole` / `whole_batch`: an existing fully loaded instance (with caches
    filled from the same `kv_seed`) and its batch; created here when absent."""
    B = len(lens)
    own_whole = whole is None
    insts = [make_instance(), make_instance()] + ([make_instance()] if own_whole else [])
    tgt, src = insts[0], insts[1]
    if own_whole:
        whole = insts[2]
    for l in range(shape.L):
        (tgt if l < k else src).load_layer_from_device(l, blobs[l])
        if own_whole:
            whole.load_layer_from_device(l, blobs[l])
    for inst in insts:
        inst.sync()
    gen_kv = torch.Generator(device="cuda")
    gen_kv.manual_seed(kv_seed)
    for i, n in enumerate(lens):
        for l in range(shape.L):
            kk = torch.randn(int(n), shape.Hkv, shape.d, generator=gen_kv, device="cuda").to(torch.bfloat16)
            vv = torch.randn(int(n), shape.Hkv, shape.d, generator=gen_kv, device="cuda").to(torch.bfloat16)
            torch.cuda.synchronize()
            (tgt if l < k else src).kv_write(l, i, 0, int(n), kk, vv)
            if own_whole:
                whole.kv_write(l, i, 0, int(n), kk, vv)
    for inst in insts:
        inst.sync()
    if whole_batch is None:
        whole_batch = whole.batch(list(range(B + 1)), list(range(B)), [int(n) for n in lens])
    batch2 = tgt.batch(list(range(B + 1)), list(range(B)), [int(n) for n in lens])
    buf = torch.empty(B, shape.H, dtype=torch.bfloat16, device="cuda")
    flags = []
    for st in range(steps):
        a = xs[st].clone()
        b = xs[st].clone()
        c = torch.empty_like(b)
        torch.cuda.synchronize()
        whole.run_layers(0, shape.L, whole_batch, a, after_current_stream=False)
        whole.batch_advance(whole_batch)
        tgt.run_layers(0, k, batch2, b, after_current_stream=False)
        tgt.export_boundary(b, B, buf)
        src.import_boundary(c, B, buf)            # the instances share one compute stream: ordered
        src.run_layers(k, shape.L, batch2, c, after_current_stream=False)
        src.batch_advance(batch2)
        whole.sync()
        src.sync()
        flags.append(bool(torch.equal(a.view(torch.int16), c.view(torch.int16))))
    for inst in insts:
        inst.close()
    return flags


# ------------------------------------------------------------------------------- workloads

def run_prefill_stream(args, torch, Instance, then_decode=None):
    """Streamed prefill leg.  `then_decode` = dict(B, lo, hi, steps, warmup): afterwards, with every layer
    resident, the same instance serves that many decode steps of B sequences with caches uniform[lo, hi];
    the function then returns (prefill record, decode record)."""
    base = W.CONFIGS[args.shape]
    shape = with_layers(base, args.layers)
    if args.fixed_len:
        lens = np.full(args.requests, args.fixed_len, dtype=np.int64)
    else:
        lens = W.lognormal_lengths(shape.seed, args.requests, 512.0, 0.6, 16, 2048)
    q_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    T, B = int(q_start[-1]), len(lens)
    max_seqs, max_len, kv_tokens = B, int(lens.max()) + 1, int(lens.sum()) + 32 * B
    if then_decode:
        dB, d_steps_total = then_decode["B"], 2 * then_decode["steps"] + then_decode["warmup"] + 4
        d_lens = W.uniform_lengths(base.seed, dB, then_decode["lo"], then_decode["hi"])
        max_seqs = max(B, dB)
        max_len = max(max_len, then_decode["hi"] + d_steps_total + 8)
        kv_tokens = max(kv_tokens, int(d_lens.sum()) + dB * (d_steps_total + 40))
    stream, copy_stream = bench_streams(torch)
    inst = Instance(shape, max_seqs=max_seqs, max_seq_len=max_len, max_tokens=T,
                    kv_tokens=kv_tokens, chunk_bytes=args.chunk_mib << 20, compute_stream=stream, copy_stream=copy_stream)
    lend_second_copy_stream(inst, torch)
    for i, n in enumerate(lens):
        inst.kv_reserve(i, int(n))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(shape.seed)
    n_blobs = min(shape.L, args.distinct_blobs) if args.distinct_blobs else shape.L
    blobs = [gen_layer_blob_gpu(torch, inst, shape, gen) for _ in range(n_blobs)]
    note(f"{shape.name}: instance and {n_blobs} pinned layer blobs ready ({inst.layer_bytes / 1e6:.0f} MB each)")
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
        inst.run_layers(0, shape.L, batch, x, after_current_stream=False)

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
    note(f"{shape.name}: warm-up done, {n_streams} copy stream(s); timing {args.steps} steps")
    inst.profile_enable(True)
    inst.profile_read()
    total, ingest_ms = 0.0, []
    for i in range(args.steps):           # resets are outside the clock
        reset()
        t0 = time.perf_counter()
        one_step()
        inst.sync()
        torch.cuda.synchronize()
        total += time.perf_counter() - t0
        ingest_ms.append(inst.layer_ready_ms(shape.L - 1))
        if total > 20.0 * (1 + i // 8):
            note(f"{shape.name}: step {i + 1}/{args.steps}")
    prof = inst.profile_read()
    inst.profile_enable(False)
    ms_per_step = total / args.steps * 1e3

    x.copy_(x0)                           # all layers resident: compute-only rate of the same batch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(3):
        inst.run_layers(0, shape.L, batch, x, after_current_stream=False)
    inst.sync()
    resident_s = (time.perf_counter() - t0) / 3
    # The same kernels launched back to back (no waiting for layers in between), with the library's events.  In
    # the streamed steps the compute stream idles between layers whenever the host link is the bottleneck, and a
    # kernel that starts after an idle gap runs at the lower clock the power management has fallen back to
    # (measured on this chip: the same GEMM 1.45 PFLOP/s back to back, 1.17 with 20 ms of idling before each launch).
    inst.profile_enable(True)
    inst.profile_read()
    for _ in range(2):
        inst.run_layers(0, shape.L, batch, x, after_current_stream=False)
    prof_res = inst.profile_read()
    inst.profile_enable(False)
    roof_res, all_tf_res = gemm_roofline(prof_res, shape.name, T)

    roof, all_tf = gemm_roofline(prof, shape.name, T)
    roof["note"] = ("timed (streamed) steps: the compute stream idles between layers while the host link is the bottleneck, "
                    "and a launch after an idle gap runs at the clock the power management fell back to; the same launches "
                    "back to back are in roofline_back_to_back")
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
        "ingested_GB_per_step": shape.L * inst.layer_bytes / 1e9,
        "resident_prefill_tokens_per_s": T / resident_s,
        "resident_ms": resident_s * 1e3,
        "gemm_TFLOPs_all_classes": all_tf,
        "kernel_ms_per_step": {k: v["ms"] / args.steps for k, v in prof.items() if v["launches"]},
        "roofline": roof,
        "roofline_back_to_back": roof_res,
        "gemm_TFLOPs_all_classes_back_to_back": all_tf_res,
        "kernel_ms_per_pass_back_to_back": {k: v["ms"] / 2 for k, v in prof_res.items() if v["launches"]},
    })
    dec = None
    if then_decode:
        # every layer is resident now; the prefill batch's slots go, the decode sequences' come
        for i in range(B):
            inst.kv_release(i)
        for i, n in enumerate(d_lens):
            inst.kv_reserve(i, int(n) + d_steps_total + 8)
        gen_kv = torch.Generator(device="cuda")
        gen_kv.manual_seed(base.seed + 100)
        for i, n in enumerate(d_lens):
            fill_kv(torch, inst, shape, gen_kv, i, int(n))
        note(f"{shape.name}: caches of {dB} decode sequences filled; {then_decode['steps']} decode steps")
        xs = torch.randn(d_steps_total, dB, shape.H, generator=gen, device="cuda").to(torch.bfloat16)
        dbatch = inst.batch(list(range(dB + 1)), list(range(dB)), [int(n) for n in d_lens])
        torch.cuda.synchronize()
        dec = decode_leg(inst, torch, shape, dbatch, xs, d_steps_total, then_decode["steps"], then_decode["warmup"], 0, dB)
        dec["workload"] = (f"{shape.name}-shaped decoder, {shape.L} layers resident, continuous decode of {dB} sequences "
                           f"with cache lengths uniform[{then_decode['lo']},{then_decode['hi']}]")
        dec["mean_cache_len"] = float(d_lens.mean())
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_prefill(base)
    inst.close()
    return (out, dec) if then_decode else out


def run_decode(args, torch, Instance):
    base = W.CONFIGS[args.shape if args.shape != "7b" else "8b_gqa"]
    shape = with_layers(base, args.layers)
    B = args.requests if args.requests != 8 else 64
    lo, hi = (512, 4096) if base.name == "70b" else (256, 4096)
    lens = W.uniform_lengths(base.seed, B, lo, hi)
    if args.fixed_len:                    # every cache the same length (no short sequences, no ragged last chunks)
        lens = np.full(B, args.fixed_len, dtype=np.int64)
        lo = hi = args.fixed_len
    n_split_steps = 8 if args.split else 0
    n_steps = 2 * args.steps + args.warmup + 4 + n_split_steps     # every step appends a position
    stream, copy_stream = bench_streams(torch)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(base.seed)

    def make_instance():
        inst = Instance(shape, max_seqs=B, max_seq_len=hi + n_steps + 8, max_tokens=B,
                        kv_tokens=int(lens.sum()) + B * (n_steps + 40), compute_stream=stream, copy_stream=copy_stream)
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
            inst.drop_sources()           # layer is resident: the staging blob can go
            del blob
    gen_kv = torch.Generator(device="cuda")
    gen_kv.manual_seed(base.seed + 100)
    for i, n in enumerate(lens):
        fill_kv(torch, inst, shape, gen_kv, i, int(n))
    note(f"{shape.name}: {shape.L} layers resident, caches of {B} sequences filled")
    xs = torch.randn(n_steps, B, shape.H, generator=gen, device="cuda").to(torch.bfloat16)
    batch = inst.batch(list(range(B + 1)), list(range(B)), [int(n) for n in lens])
    torch.cuda.synchronize()

    split_note = None
    if args.split:
        # live split (cooperative execution) against this instance, bit for bit, over steps that take at least
        # one cache across a 256-position chunk boundary of the decode-attention kernel
        flags = live_split_check(torch, make_instance, shape, blobs, lens, base.seed + 100, xs, args.split, n_split_steps,
                                 whole=inst, whole_batch=batch)
        crossed = sum(1 for n in lens if int(n) // 256 != (int(n) + n_split_steps) // 256)
        split_note = {"split_layer": args.split, "bit_exact_steps": len(flags), "bit_exact": all(flags),
                      "caches_that_crossed_a_chunk_boundary": crossed}
        blobs.clear()
        inst.drop_sources()
        if not all(flags):
            raise SystemExit("split run is not bit-exact")
        note(f"{shape.name}: live split at layer {args.split} bit-exact over {len(flags)} steps")

    dec = decode_leg(inst, torch, shape, batch, xs, n_steps, args.steps, args.warmup, n_split_steps, B)
    out = base_record("decode tokens/s", dec["decode_tokens_per_s"], "tokens/s", args, dec["ms_per_step"],
                      f"{shape.name}-shaped decoder, {shape.L} layers resident, continuous decode of {B} sequences "
                      f"with cache lengths uniform[{lo},{hi}]",
                      {"shape": shape.name, "layers": shape.L, "sequences": B, "mean_cache_len": float(lens.mean())})
    out.update({k: v for k, v in dec.items() if k not in ("decode_tokens_per_s", "ms_per_step", "steps")})
    if split_note:
        out["split"] = split_note
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_decode(base, lens)
    inst.close()
    return out


def run_continuous(args, torch, Instance):
    """Continuous batching (paper section 6): a decode loop whose membership changes every step - one sequence
    leaves, one with a cache of its own joins.  Three ways to tell the library: (a) membership frozen, the batch
    advanced on the device (lower bound on the step time); (b) one batch object in lent memory rebuilt in place
    every step, asynchronously; (c) a new batch per step with the allocating, synchronous call (the only way
    before the in-place form existed).  Reports ms per step and the host time spent enqueueing a step."""
    base = W.CONFIGS[args.shape if args.shape != "7b" else "8b_gqa"]
    shape = with_layers(base, args.layers)
    B = args.requests if args.requests != 8 else 64
    pool = B + 32                                     # slots: B active + spares that rotate in
    lens = W.uniform_lengths(base.seed, pool, 256, 4096)
    steps = args.steps
    stream, copy_stream = bench_streams(torch)
    inst = Instance(shape, max_seqs=pool, max_seq_len=4096 + 3 * steps + 16, max_tokens=B,
                    kv_tokens=int(lens.sum()) + pool * (3 * steps + 48), compute_stream=stream, copy_stream=copy_stream)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(base.seed)
    for l in range(shape.L):
        blob = gen_layer_blob_gpu(torch, inst, shape, gen, pinned=False)
        torch.cuda.synchronize()
        inst.load_layer_from_device(l, blob)
        inst.sync()
        inst.drop_sources()
        del blob
    gen_kv = torch.Generator(device="cuda")
    gen_kv.manual_seed(base.seed + 100)
    for i, n in enumerate(lens):
        inst.kv_reserve(i, int(n) + 3 * steps + 16)
        fill_kv(torch, inst, shape, gen_kv, i, int(n))
    note(f"{shape.name}: {shape.L} layers resident, caches of {pool} sequences filled")
    xs = torch.randn(8, B, shape.H, generator=gen, device="cuda").to(torch.bfloat16)
    cur = [int(n) for n in lens]                      # cache length per slot, as the host tracks it
    q = list(range(B + 1))
    torch.cuda.synchronize()

    def members(step):                                # slots active at `step`: a window sliding over the pool
        return [(step + j) % pool for j in range(B)]

    out = {}
    modes = set(args.continuous_modes.split(","))
    if not modes or not modes <= {"frozen", "in_place", "new"}:
        raise SystemExit("--continuous-modes takes a comma-separated subset of frozen,in_place,new")
    if "frozen" in modes:
        # (a) frozen membership, device-side advance
        batch = inst.batch(q, members(0), [cur[s] for s in members(0)])
        for _ in range(4):
            inst.run_layers(0, shape.L, batch, xs[0], after_current_stream=False)
            inst.batch_advance(batch)
        inst.sync()
        t0 = time.perf_counter()
        for st in range(steps):
            inst.run_layers(0, shape.L, batch, xs[st % 8], after_current_stream=False)
            inst.batch_advance(batch)
        host = time.perf_counter() - t0
        inst.sync()
        out["frozen_membership_advance"] = {"ms_per_step": (time.perf_counter() - t0) / steps * 1e3,
                                            "host_enqueue_ms_per_step": host / steps * 1e3}
        for s in members(0):
            cur[s] += steps + 4
        batch.close()
    if "in_place" in modes:
        # (b) rebuilt in place every step
        storage = inst.batch_storage(B, B, 4096 + 3 * steps + 16)
        batch = inst.batch(q, members(0), [cur[s] for s in members(0)], storage=storage)
        t0 = time.perf_counter()
        for st in range(steps):
            m = members(st)
            if st:
                batch.rebuild(q, m, [cur[s] for s in m])
            inst.run_layers(0, shape.L, batch, xs[st % 8], after_current_stream=False)
            for s in m:
                cur[s] += 1
        host = time.perf_counter() - t0
        inst.sync()
        out["rebuilt_in_place"] = {"ms_per_step": (time.perf_counter() - t0) / steps * 1e3,
                                   "host_enqueue_ms_per_step": host / steps * 1e3}
        batch.close()
    if "new" in modes:
        # (c) a new allocated batch per step
        t0 = time.perf_counter()
        old = []
        for st in range(steps):
            m = members(st)
            b2 = inst.batch(q, m, [cur[s] for s in m])
            inst.run_layers(0, shape.L, b2, xs[st % 8], after_current_stream=False)
            for s in m:
                cur[s] += 1
            old.append(b2)                                # destroying it here would wait for the step
        host = time.perf_counter() - t0
        inst.sync()
        out["new_batch_per_step"] = {"ms_per_step": (time.perf_counter() - t0) / steps * 1e3,
                                     "host_enqueue_ms_per_step": host / steps * 1e3}
        for b2 in old:
            b2.close()
    head = out.get("rebuilt_in_place") or next(iter(out.values()))
    rec = base_record("decode tokens/s", B / (head["ms_per_step"] * 1e-3), "tokens/s", args,
                      head["ms_per_step"],
                      f"{shape.name}-shaped decoder, {shape.L} layers resident, continuous batching of {B} sequences out of a "
                      f"pool of {pool}: one leaves and one joins every step, the batch rebuilt in place",
                      {"shape": shape.name, "layers": shape.L, "sequences": B, "pool": pool})
    rec["modes"] = out
    inst.close()
    return rec


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
    stream, copy_stream = bench_streams(torch)
    inst = Instance(shape, max_seqs=B, max_seq_len=max(caps) + 1, max_tokens=T, kv_tokens=sum(caps) + 32 * B,
                    chunk_bytes=args.chunk_mib << 20, compute_stream=stream, copy_stream=copy_stream)
    lend_second_copy_stream(inst, torch)
    for i, c in enumerate(caps):
        inst.kv_reserve(i, c)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(base.seed)
    blobs = [gen_layer_blob_gpu(torch, inst, shape, gen) for _ in range(shape.L)]
    for i in range(16, B):
        fill_kv(torch, inst, shape, gen, i, befores[i])
    note(f"{shape.name}: {shape.L} pinned layer blobs and the caches of 48 decode sequences ready")
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
        inst.run_layers(0, shape.L, batch, x, after_current_stream=False)

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
    roof, all_tf = gemm_roofline(prof, shape.name, T)
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


def _release(torch):
    import gc
    gc.collect()
    torch.cuda.synchronize()
    torch.cuda.empty_cache()


def _leg_summary(rec, keys):
    out = {"workload": rec["config"]["workload"], "steps": rec["steps"], "warmup": rec["warmup"]}
    out.update({k: rec[k] for k in keys if k in rec})
    return out


def run_all(args, torch, Instance):
    """The default line: the 70B-shaped streamed prefill as the headline, the other configurations as extra
    keys.  --steps / --warmup apply to the headline leg; the secondary legs run their own, smaller counts."""
    import copy
    legs = {}
    a5 = copy.copy(args)
    a5.shape, a5.requests, a5.fixed_len, a5.distinct_blobs = "70b", 4, 2048, 4
    head, dec5 = run_prefill_stream(a5, torch, Instance, then_decode=dict(B=32, lo=512, hi=4096, steps=256, warmup=8))
    legs["cfg5_70b_decode"] = dec5
    _release(torch)
    note("headline leg and 70B decode leg done")

    small = min(args.steps, 5)
    a2 = copy.copy(args)
    a2.shape, a2.requests, a2.fixed_len, a2.distinct_blobs, a2.steps, a2.warmup, a2.no_cpu_baseline = "7b", 8, 0, 0, small, 2, True
    r2 = run_prefill_stream(a2, torch, Instance)
    legs["cfg2_7b_prefill_stream"] = _leg_summary(r2, ["value", "unit", "ms_per_step", "ttft_ms", "ingest_GBps",
                                                       "resident_prefill_tokens_per_s", "resident_ms",
                                                       "gemm_TFLOPs_all_classes", "kernel_ms_per_step", "roofline",
                                                       "roofline_back_to_back", "gemm_TFLOPs_all_classes_back_to_back"])
    legs["cfg2_7b_prefill_stream"]["ingest_streams"] = r2["config"]["ingest_streams"]
    _release(torch)
    note("7B streamed prefill leg done")

    a3 = copy.copy(args)
    a3.shape, a3.requests, a3.fixed_len, a3.steps, a3.warmup, a3.split, a3.no_cpu_baseline = "8b_gqa", 64, 0, 128, 8, 16, args.no_cpu_baseline
    r3 = run_decode(a3, torch, Instance)
    legs["cfg3_8b_gqa_decode"] = _leg_summary(r3, ["value", "unit", "ms_per_step", "weights_GB_per_step", "kv_GB_per_step",
                                                   "hbm_roofline_frac_whole_step", "kernel_ms_per_step", "roofline", "split",
                                                   "cpu_baseline"])
    _release(torch)
    note("8B-GQA decode leg done")

    a4 = copy.copy(args)
    a4.steps, a4.warmup, a4.no_cpu_baseline = small, 2, True
    r4 = run_mixed_ttft(a4, torch, Instance)
    legs["cfg4_13b_mixed_ttft"] = _leg_summary(r4, ["value", "unit", "ms_per_step", "ttft_ms", "ingest_ms", "ingest_GBps",
                                                    "kernel_ms_sum_per_step", "overlap_efficiency",
                                                    "gemm_TFLOPs_all_classes", "kernel_ms_per_step", "roofline"])
    legs["cfg4_13b_mixed_ttft"]["ingest_streams"] = r4["config"]["ingest_streams"]
    _release(torch)
    note("13B mixed-batch leg done")
    head["configs"] = legs
    return head


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
    ap.add_argument("--workload", default="all", choices=["all", "prefill_stream", "decode", "mixed_ttft", "zigzag", "continuous"])
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
    ap.add_argument("--continuous-modes", default="frozen,in_place,new",
                    help="continuous: which of the three ways to run (a trace of one way alone shows its host calls)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2
    if args.steps is None:
        args.steps = 128 if args.workload in ("decode", "continuous") else 5
    if args.warmup is None:
        args.warmup = 8 if args.workload == "decode" else 2

    import torch
    from paper_2412_17246_amd import Instance

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    fn = {"all": run_all, "prefill_stream": run_prefill_stream, "decode": run_decode, "mixed_ttft": run_mixed_ttft,
          "zigzag": run_zigzag, "continuous": run_continuous}[args.workload]
    print(json.dumps(fn(args, torch, Instance)))
    return 0


if __name__ == "__main__":
    sys.exit(main())
