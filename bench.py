#!/usr/bin/env python3
"""Benchmark of the hot path on one MI355X.

Default workload ("7b_prefill_stream"): a Llama-2-7B-shaped decoder (32 layers) whose weights
start in pinned host memory.  One step = scale start to first token: every layer is requested
with load_layer (chunked host->HBM copies on the copy stream) and, at the same moment, one packed
prefill batch of 8 requests (lognormal lengths) is sent through run_layers(0, 32), each layer
gated on its own ingest event, so resident layers execute while later ones are still arriving.
Hidden states, KV cache and workspaces are resident in HBM before the timed region; the weights'
trip over the host link is the method's own ingest step and is inside it.

Prints ONE JSON line (see the keys below).  `--gpus N` with N > 1 is refused: this build is
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


def gen_layer_blob_gpu(torch, inst, shape, layer, gen):
    """Draws one layer's nine tensors on the GPU (seeded) and returns a pinned host blob."""
    blob = torch.empty(inst.layer_bytes, dtype=torch.uint8, pin_memory=True)
    view = blob.view(torch.bfloat16)
    for name, shp in W.tensor_shapes(shape).items():
        n = int(np.prod(shp))
        t = torch.randn(n, generator=gen, device="cuda", dtype=torch.float32) * 0.02
        if name in ("g1", "g2"):
            t += 1.0
        off = getattr(inst.layout, name) // 2
        view[off:off + n].copy_(t.to(torch.bfloat16))
    return blob


def build_prefill_batch(shape, n_req, median, sigma, lo, hi):
    lens = W.lognormal_lengths(shape.seed, n_req, median, sigma, lo, hi)
    q_start = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    return lens, q_start


def cpu_baseline_prefill(shape, seconds_budget=20.0):
    """Times the CPU oracle (as it stands) on one layer of the real shape over a bounded sample:
    one request of `n` prompt tokens.  Reported in the metric's unit: tokens/s through all L
    layers = n / (L * seconds per layer)."""
    from oracle import decoder as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = os.cpu_count() or 1
    n = 256
    osh = O.OracleShape(L=shape.L, H=shape.H, Hq=shape.Hq, Hkv=shape.Hkv, d=shape.d, F=shape.F,
                        eps=shape.eps, rope_base=shape.rope_base)
    bits = W.layer_weights_bits(shape, 0)
    wts = {k: W.f32_from_bf16_bits(v).astype(np.float64) for k, v in bits.items()}
    x = W.f32_from_bf16_bits(W.hidden_bits(shape, n, step=0)).astype(np.float64)
    reps, t_used = 0, 0.0
    while reps < 1 or (t_used < seconds_budget / 2 and reps < 8):
        t0 = time.perf_counter()
        O.run_layers(osh, {0: wts}, 0, 1, x, O.OracleBatch([0, n], [0], [0]), O.OracleKV())
        t_used += time.perf_counter() - t0
        reps += 1
    per_layer = t_used / reps
    return {"value": n / (per_layer * shape.L), "unit": "tokens/s", "cores": int(cores), "kind": "oracle",
            "sample": f"float64 numpy oracle, 1 layer of the {shape.name} shape, one request of {n} prompt tokens, "
                      f"{reps} repetitions, scaled by 1/L to whole-model tokens/s"}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--shape", default="7b", choices=list(W.CONFIGS))
    ap.add_argument("--layers", type=int, default=0, help="use only the first N layers of the shape (debugging)")
    ap.add_argument("--chunk-mib", type=int, default=0, help="ingest chunk size in MiB (0 = library default)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no collectives, no sharding); "
              f"--gpus {args.gpus} is not supported", file=sys.stderr)
        return 2

    import torch
    from paper_2412_17246_amd import Instance

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 1
    base = W.CONFIGS[args.shape]
    shape = base if not args.layers else W.DecoderShape(base.name, args.layers, base.H, base.Hq, base.Hkv, base.d,
                                                        base.F, base.eps, base.rope_base, base.seed)
    lens, q_start = build_prefill_batch(shape, 8, 512.0, 0.6, 16, 2048)
    T = int(q_start[-1])
    B = len(lens)
    stream = torch.cuda.Stream()
    inst = Instance(shape, max_seqs=B, max_seq_len=int(lens.max()) + 1, max_tokens=T, kv_tokens=int(lens.sum()) + 32 * B,
                    chunk_bytes=args.chunk_mib << 20, compute_stream=stream)
    for i, n in enumerate(lens):
        inst.kv_reserve(i, int(n))
    gen = torch.Generator(device="cuda")
    gen.manual_seed(shape.seed)
    blobs = [gen_layer_blob_gpu(torch, inst, shape, l, gen) for l in range(shape.L)]
    x0 = torch.from_numpy(W.hidden_bits(shape, T, step=0).view(np.int16).copy()).view(torch.bfloat16).cuda()
    x = torch.empty_like(x0)
    batch = inst.batch(q_start, list(range(B)), [0] * B)
    torch.cuda.synchronize()

    def one_step():
        """Scale start -> first token.  Returns after everything has been enqueued."""
        inst.reset_clock()
        for l in range(shape.L):
            inst.load_layer(l, blobs[l])
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

    # ---- timed region: K steps, each bracketed by synchronisation; resets are outside the clock
    inst.profile_enable(True)
    inst.profile_read()
    total = 0.0
    ingest_ms = []
    for _ in range(args.steps):
        reset()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        one_step()
        inst.sync()
        torch.cuda.synchronize()
        total += time.perf_counter() - t0
        ingest_ms.append(inst.layer_ready_ms(shape.L - 1))
    prof = inst.profile_read()
    inst.profile_enable(False)
    ms_per_step = total / args.steps * 1e3
    value = T * args.steps / total

    # ---- all layers resident: compute-only rate of the same batch (context for the roofline)
    x.copy_(x0)
    torch.cuda.synchronize()
    reps = 3
    t0 = time.perf_counter()
    for _ in range(reps):
        inst.run_layers(0, shape.L, batch, x)
    inst.sync()
    resident_s = (time.perf_counter() - t0) / reps

    gemm_classes = [k for k in prof if k.startswith("gemm")]
    dom = max(gemm_classes, key=lambda k: prof[k]["ms"])
    d = prof[dom]
    achieved = d["flops"] / (d["ms"] * 1e-3) / 1e12 if d["ms"] > 0 else 0.0
    all_gemm_flops = sum(prof[k]["flops"] for k in gemm_classes)
    all_gemm_ms = sum(prof[k]["ms"] for k in gemm_classes)
    ingest_bytes = shape.L * inst.layer_bytes
    out = {
        "metric": "prefill tokens/s on partially loaded model",
        "value": value,
        "unit": "tokens/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "bf16",
        "data": "synthetic",
        "config": {
            "workload": f"{shape.name}-shaped decoder, {shape.L} layers streamed from pinned host memory while a "
                        f"packed prefill batch of {B} requests ({T} tokens, lognormal lengths) runs behind the frontier",
            "shape": shape.name, "layers": shape.L, "requests": B, "tokens": T,
            "lengths": [int(v) for v in lens],
        },
        "ttft_ms": ms_per_step,
        "ingest_GBps": ingest_bytes / (float(np.median(ingest_ms)) * 1e-3) / 1e9,
        "resident_prefill_tokens_per_s": T / resident_s,
        "resident_ms": resident_s * 1e3,
        "gemm_TFLOPs_all_classes": all_gemm_flops / (all_gemm_ms * 1e-3) / 1e12 if all_gemm_ms > 0 else 0.0,
        "kernel_ms_per_step": {k: v["ms"] / args.steps for k, v in prof.items() if v["launches"]},
        "roofline": {
            "bound": "mfma", "kernel": dom, "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
            "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None,
            "launches": d["launches"], "avg_ms": d["ms"] / max(d["launches"], 1),
        },
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline_prefill(base)
    inst.close()
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
