"""Shared helpers of the GPU parity tests: seeded inputs as both oracle (float64) and device
(bf16 / fp32) views, error metrics, instance set-up.  Uses the oracle and the binding side by side;
neither imports the other."""
import os

import numpy as np

import workloads as W
from oracle import decoder as O

BF16_TOL = 2e-2        # max-abs error over max-abs reference, bf16 product build
FP32_TOL = 1e-4        # same metric, fp32 debug build
# Second gate: rms(got - ref) / rms(ref).  The first gate follows the largest element; a mistake of a few per
# cent spread over every element (a dropped norm gain, a wrong constant) stays below it and shows here.  Values
# measured over the whole suite: single operations <= 1.8e-3, layers of the small shapes <= 3.9e-3, layers of the
# real shapes <= 9.5e-3 (70B: sums over 28672 terms), fp32 debug build <= 2.1e-6; the gates leave about a factor two.
RMS_BF16_OP = 4e-3
RMS_BF16 = 8e-3
RMS_BF16_FULLSIZE = 1.5e-2
RMS_FP32 = 5e-5


def oracle_shape(s: W.DecoderShape) -> O.OracleShape:
    return O.OracleShape(L=s.L, H=s.H, Hq=s.Hq, Hkv=s.Hkv, d=s.d, F=s.F, eps=s.eps, rope_base=s.rope_base)


def f64(bits: np.ndarray) -> np.ndarray:
    return W.f32_from_bf16_bits(bits).astype(np.float64)


def oracle_weights(bits: dict) -> dict:
    return {k: f64(v) for k, v in bits.items()}


def rel_err(got: np.ndarray, ref: np.ndarray) -> float:
    """max |got - ref| / max |ref| over the tensor."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    assert np.all(np.isfinite(got)), "non-finite values in the GPU result"
    err = float(np.max(np.abs(got - ref)) / max(float(np.max(np.abs(ref))), 1e-30))
    log = os.environ.get("BZ_TEST_ERR_LOG")              # opt-in: one line per comparison, for setting the gates
    if log:
        with open(log, "a") as f:
            f.write("%s max/max %.3e rms/rms %.3e shape %s\n" % (os.environ.get("PYTEST_CURRENT_TEST", "?"), err,
                                                               rms_err(got, ref), got.shape))
    return err


def rms_err(got: np.ndarray, ref: np.ndarray) -> float:
    """rms(got - ref) / rms(ref) over the tensor: a systematic few-per-cent mistake spread over every element
    (a dropped gain, a wrong constant) shows here although it stays far below the largest element."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    return float(np.sqrt(np.mean((got - ref) ** 2)) / max(float(np.sqrt(np.mean(ref * ref))), 1e-30))


def assert_rms(got: np.ndarray, ref: np.ndarray, tol: float) -> None:
    e = rms_err(got, ref)
    assert e <= tol, ("rms error", e, tol)


def mixed_err(got: np.ndarray, ref: np.ndarray, tol: float) -> float:
    """largest |got - ref| / (tol*|ref| + tol*rms(ref)); <= 1 passes the secondary criterion."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.max(np.abs(got - ref) / (tol * np.abs(ref) + tol * rms + 1e-300)))


def to_device(bits: np.ndarray, fp32: bool):
    """bf16 bit patterns -> device tensor in the library's activation type."""
    import torch
    t = torch.from_numpy(bits.view(np.int16).copy()).view(torch.bfloat16).cuda()
    return t.float().contiguous() if fp32 else t.contiguous()


def f64_to_device(x: np.ndarray, fp32: bool):
    """float64 values -> (device tensor, the exact float64 values it holds)."""
    import torch
    bits = W.bf16_bits_from_f32(np.asarray(x, dtype=np.float32))
    return to_device(bits, fp32), f64(bits)


def from_device(t) -> np.ndarray:
    import torch
    torch.cuda.synchronize()
    return t.detach().float().cpu().numpy().astype(np.float64)


def make_instance(shape, *, max_seqs, max_seq_len, max_tokens, kv_tokens, fp32=False, chunk_bytes=0):
    from paper_2412_17246_amd import Instance
    return Instance(shape, max_seqs=max_seqs, max_seq_len=max_seq_len, max_tokens=max_tokens,
                    kv_tokens=kv_tokens, fp32_debug=fp32, chunk_bytes=chunk_bytes)


def load_all_layers(inst, shape, layers=None):
    """Generates, packs, pins and loads the given layers; returns {layer: (bits, pinned tensor)}."""
    out = {}
    for l in (range(shape.L) if layers is None else layers):
        bits = W.layer_weights_bits(shape, l)
        pinned = inst.pinned_blob(inst.pack_layer(bits))
        inst.load_layer(l, pinned)
        out[l] = (bits, pinned)
    return out
