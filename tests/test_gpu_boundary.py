"""Boundary behaviour on the GPU: ingest byte-exactness for several chunk sizes and sources, KV
import/export round trips through the cache layout, slot reuse, error codes that need a device."""
import numpy as np
import pytest

import workloads as W
from paper_2412_17246_amd import binding as B
from tests import _util as U

pytestmark = pytest.mark.gpu

TINY = W.CONFIGS["tiny"]


@pytest.fixture(scope="module")
def torch():
    import torch
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return torch


@pytest.mark.parametrize("streams", [1, 2])
@pytest.mark.parametrize("chunk", [0, 4096, 1 << 20, 1000003])
def test_ingest_is_byte_exact_for_any_chunk_size(torch, chunk, streams):
    inst = U.make_instance(TINY, max_seqs=1, max_seq_len=32, max_tokens=8, kv_tokens=32, chunk_bytes=chunk)
    inst.set_ingest_streams(streams)
    with pytest.raises(Exception) as ei:
        inst.set_ingest_streams(3)
    assert "BZ_EINVAL" in str(ei.value)
    rng = np.random.default_rng(chunk + 1)
    blobs = [rng.integers(0, 256, inst.layer_bytes, dtype=np.uint8) for _ in range(TINY.L)]
    pinned = [inst.pinned_blob(b) for b in blobs]
    for l in (1, 0):                                   # out of order
        inst.load_layer(l, pinned[l])
    for l in range(TINY.L):
        assert np.array_equal(inst.readback_layer(l), blobs[l])
    st = inst.stats()
    assert st["bytes_ingested"] == TINY.L * inst.layer_bytes and st["frontier"] == TINY.L
    inst.close()


def test_device_resident_source_and_reload(torch):
    inst = U.make_instance(TINY, max_seqs=1, max_seq_len=32, max_tokens=8, kv_tokens=32)
    blob = np.random.default_rng(3).integers(0, 256, inst.layer_bytes, dtype=np.uint8)
    dev = torch.from_numpy(blob).cuda()
    torch.cuda.synchronize()
    inst.load_layer_from_device(0, dev)
    assert np.array_equal(inst.readback_layer(0), blob)
    inst.unload_layer(0)
    assert inst.frontier() == 0 and not inst.layer_ready(0)
    blob2 = blob[::-1].copy()
    inst.load_layer(0, inst.pinned_blob(blob2))        # the same slot can be loaded again after unload
    assert np.array_equal(inst.readback_layer(0), blob2)
    inst.close()


@pytest.mark.parametrize("streams", [1, 2])
def test_forwarding_chain_of_three_instances(torch, streams):
    """Section 5.1, serial forwarding chain S -> T1 -> T2 on one GPU: T1 receives every layer from page-locked host
    memory, T2 takes each layer from T1's copy as it lands, while T1 is receiving the next ones; nothing waits on
    the host while the chain is set up.  T2 executes a batch behind its own frontier; its weights are T1's bytes and
    its output is that of an instance loaded directly."""
    s = W.DecoderShape("chain", L=6, H=512, Hq=8, Hkv=2, d=64, F=1024, rope_base=10000.0, seed=88)
    mk = lambda: U.make_instance(s, max_seqs=1, max_seq_len=96, max_tokens=80, kv_tokens=96, chunk_bytes=256 << 10)
    t1, t2, ref = mk(), mk(), mk()
    other = U.make_instance(TINY, max_seqs=1, max_seq_len=32, max_tokens=8, kv_tokens=32)
    for inst in (t1, t2):
        inst.set_ingest_streams(streams)
    blobs = [t1.pack_layer(W.layer_weights_bits(s, l)) for l in range(s.L)]
    pinned = [t1.pinned_blob(b) for b in blobs]
    for bad, code in ((t2, "BZ_EINVAL"), (other, "BZ_EINVAL"), (t1, "BZ_ENOTLOADED")):   # itself; another shape; nothing requested yet
        with pytest.raises(Exception) as ei:
            t2.load_layer_from_peer(0, bad)
        assert code in str(ei.value)
    xbits = W.hidden_bits(s, 80, step=4, scale=1.0 / 16)
    x2, xr = U.to_device(xbits, False), U.to_device(xbits, False)
    for inst in (t2, ref):
        inst.kv_reserve(0, 80)
    torch.cuda.synchronize()
    for l in range(s.L):
        t1.load_layer(l, pinned[l])
        t2.load_layer_from_peer(l, t1)
    t2.run_layers(0, s.L, t2.batch([0, 80], [0], [0]), x2, after_current_stream=False)
    seen = []
    for _ in range(50):                                   # T2 never holds a layer T1 does not hold yet
        f2 = t2.frontier()
        f1 = t1.frontier()
        assert f2 <= f1
        seen.append((f1, f2))
        if f2 == s.L:
            break
    t2.sync()
    t1.sync()
    assert t1.frontier() == s.L and t2.frontier() == s.L
    for l in range(s.L):
        assert np.array_equal(t2.readback_layer(l), blobs[l])
    with pytest.raises(Exception) as ei:
        t2.load_layer_from_peer(0, t1)                      # already resident here
    assert "BZ_EBUSY" in str(ei.value)
    for l in range(s.L):
        ref.load_layer(l, pinned[l])
    ref.run_layers(0, s.L, ref.batch([0, 80], [0], [0]), xr, after_current_stream=False)
    ref.sync()
    assert torch.equal(x2.view(torch.int16), xr.view(torch.int16))
    for inst in (t2, t1, ref, other):
        inst.close()


@pytest.mark.parametrize("n_shards", [1, 3, 4, 16])
def test_sharded_ingest_is_byte_exact_and_ready_only_when_all_shards_landed(torch, n_shards):
    """Section 5.1, parallel sharded transfer: uneven shards, given out of order, from a mix of pinned
    host and device sources, on one stream each; the layer's bytes equal the whole blob; a following
    unsharded layer still completes; the frontier covers both."""
    inst = U.make_instance(TINY, max_seqs=1, max_seq_len=32, max_tokens=8, kv_tokens=32, chunk_bytes=64 << 10)
    n = inst.layer_bytes
    rng = np.random.default_rng(40 + n_shards)
    blob = rng.integers(0, 256, n, dtype=np.uint8)
    cuts = np.sort(rng.choice(np.arange(1, n), size=n_shards - 1, replace=False)) if n_shards > 1 else np.array([], int)
    edges = [0] + [int(c) for c in cuts] + [n]
    shards = []
    for j in range(n_shards):
        piece = blob[edges[j]:edges[j + 1]]
        src = torch.from_numpy(piece.copy()).cuda() if j % 2 else inst.pinned_blob(piece)
        shards.append((src, edges[j]))
    torch.cuda.synchronize()
    shards = shards[::-1]                                  # any order
    inst.load_layer_sharded(0, shards)
    blob1 = blob[::-1].copy()
    inst.load_layer(1, inst.pinned_blob(blob1))
    inst.wait_layer(1)
    assert inst.frontier() == 2
    assert np.array_equal(inst.readback_layer(0), blob)
    assert np.array_equal(inst.readback_layer(1), blob1)
    assert inst.stats()["bytes_ingested"] == 2 * n
    inst.close()


def test_sharded_ingest_rejects_gaps_overlaps_and_wrong_totals(torch):
    inst = U.make_instance(TINY, max_seqs=1, max_seq_len=32, max_tokens=8, kv_tokens=32)
    n = inst.layer_bytes
    half = inst.pinned_blob(np.zeros(n // 2, np.uint8))
    rest = inst.pinned_blob(np.zeros(n - n // 2, np.uint8))
    for bad in ([(half, 0)],                                # too short
                [(half, 0), (rest, n // 2 + 16)],           # gap (and runs past the end)
                [(half, 0), (rest, n // 2 - 16)],           # overlap
                [(half, 0), (rest, n // 2), (half, 0)],     # covered twice
                [(half, 16), (rest, n // 2 + 16)]):         # does not start at 0
        with pytest.raises(B.BzError) as e:
            inst.load_layer_sharded(0, bad)
        assert e.value.name == "BZ_EINVAL"
    with pytest.raises(B.BzError) as e:
        inst.load_layer_sharded(0, [(half, 0)] * (B.BZ_MAX_SHARDS + 1))
    assert e.value.name == "BZ_EINVAL"
    assert inst.frontier() == 0
    inst.load_layer_sharded(0, [(half, 0), (rest, n // 2)])
    with pytest.raises(B.BzError) as e:
        inst.load_layer_sharded(0, [(half, 0), (rest, n // 2)])
    assert e.value.name == "BZ_EBUSY"
    inst.wait_layer(0)
    inst.close()


@pytest.mark.parametrize("fp32", [False, True], ids=["bf16", "fp32dbg"])
@pytest.mark.parametrize("shape", [TINY, W.DecoderShape("g", L=2, H=256, Hq=8, Hkv=2, d=128, F=256, seed=51)],
                         ids=["d64", "d128"])
def test_kv_write_read_round_trip(torch, fp32, shape):
    """Token-major K/V in, cache layout inside (K in 32-position piece-major blocks), token-major out;
    partial ranges that straddle block boundaries; host and device buffers."""
    s = shape
    inst = U.make_instance(s, max_seqs=3, max_seq_len=200, max_tokens=8, kv_tokens=512, fp32=fp32)
    inst.kv_reserve(0, 100)
    inst.kv_reserve(2, 190)
    n = 150
    kb, vb = W.kv_prefill_bits(s, 1, 2, n)
    as_host = (lambda b: W.f32_from_bf16_bits(b)) if fp32 else (lambda b: b)
    inst.kv_write(1, 2, 0, 40, as_host(kb[:40]), as_host(vb[:40]))                 # host source
    kd, vd = U.to_device(kb[40:], fp32), U.to_device(vb[40:], fp32)
    torch.cuda.synchronize()
    inst.kv_write(1, 2, 40, n - 40, kd, vd)                                        # device source
    inst.sync()
    ko = np.empty((n - 7, s.Hkv, s.d), dtype=np.float32 if fp32 else np.uint16)
    vo = np.empty_like(ko)
    inst.kv_read(1, 2, 7, n - 7, ko, vo)
    assert np.array_equal(ko, as_host(kb[7:])) and np.array_equal(vo, as_host(vb[7:]))
    with pytest.raises(Exception) as ei:
        inst.kv_write(1, 2, 180, 20, as_host(kb[:20]), as_host(vb[:20]))
    assert "BZ_ECAPACITY" in str(ei.value)
    with pytest.raises(Exception) as ei:
        inst.kv_write(1, 1, 0, 4, as_host(kb[:4]), as_host(vb[:4]))                # slot 1 not reserved
    assert "BZ_ESTATE" in str(ei.value)
    # releasing and re-reserving hands the same room out again
    free_before = inst.kv_free_tokens()
    inst.kv_release(0)
    inst.kv_reserve(1, 64)
    assert inst.kv_free_tokens() <= free_before + 128
    inst.close()


def test_empty_ranges_and_single_token(torch):
    s = TINY
    inst = U.make_instance(s, max_seqs=2, max_seq_len=64, max_tokens=8, kv_tokens=128)
    U.load_all_layers(inst, s)
    inst.kv_reserve(0, 8)
    x = U.to_device(W.hidden_bits(s, 1), False)
    before = x.clone()
    torch.cuda.synchronize()
    batch = inst.batch([0, 1], [0], [0])
    inst.run_layers(1, 1, batch, x)                    # empty layer range: nothing happens
    inst.sync()
    assert torch.equal(x.view(torch.int16), before.view(torch.int16))
    inst.run_layers(0, 2, batch, x)                    # one token, empty cache
    inst.sync()
    assert torch.isfinite(x.float()).all() and not torch.equal(x.view(torch.int16), before.view(torch.int16))
    with pytest.raises(Exception) as ei:
        inst.run_layers(0, 3, batch, x)
    assert "BZ_EINVAL" in str(ei.value)
    with pytest.raises(Exception) as ei:
        inst.run_layers(0, 2, inst.batch([0, 1], [1], [0]), x)     # slot never reserved
    assert "BZ_ESTATE" in str(ei.value)
    inst.close()


def test_plain_c_program_streams_layers_and_runs_them(torch, tmp_path):
    """tests/c_abi/gpu_run.c, compiled with gcc as C99 against include/blitz_layer.h and the HIP runtime's C API: no
    Python and no PyTorch in its process, streams and arenas made by the library.  It streams the layers of a small
    GQA shape in, runs a prompt behind the frontier and one decode step, reads every layer back; its output file is
    compared with the oracle here."""
    import os
    import shutil
    import subprocess
    from oracle import decoder as O
    if shutil.which("gcc") is None:
        pytest.skip("no gcc")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    pkg = os.path.join(root, "paper_2412_17246_amd")
    exe = str(tmp_path / "gpu_run")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-D__HIP_PLATFORM_AMD__", "-I", os.path.join(root, "include"),
           "-isystem", "/opt/rocm/include", os.path.join(root, "tests", "c_abi", "gpu_run.c"), "-o", exe,
           "-L", pkg, "-l:libblitzlayer.so", "-L", "/opt/rocm/lib", "-lamdhip64",
           "-Wl,-rpath," + pkg, "-Wl,-rpath,/opt/rocm/lib"]
    res = subprocess.run(cmd, capture_output=True, text=True)
    assert res.returncode == 0, res.stderr

    s = W.DecoderShape("cprog", L=3, H=384, Hq=8, Hkv=2, d=64, F=520, rope_base=10000.0, seed=77)
    T = 150                                                    # two query tiles, the second ragged
    probe = B.Instance(s, max_seqs=1, max_seq_len=8, max_tokens=8, kv_tokens=32, dry_run=True)
    bits = {l: W.layer_weights_bits(s, l) for l in range(s.L)}
    blobs = [probe.pack_layer(bits[l]) for l in range(s.L)]
    probe.close()
    xbits = W.hidden_bits(s, T + 1, step=9, scale=1.0 / 16)    # rows 0..T-1: the prompt; row T: the decode step's input
    src, dst = tmp_path / "in.bin", tmp_path / "out.bin"
    with open(src, "wb") as f:
        f.write(np.array([s.L, s.H, s.Hq, s.Hkv, s.d, s.F, T], dtype=np.int32).tobytes())
        f.write(np.array([s.eps, s.rope_base], dtype=np.float32).tobytes())
        for b in blobs:
            f.write(b.tobytes())
        f.write(np.ascontiguousarray(xbits, dtype=np.uint16).tobytes())
    run = subprocess.run([exe, str(src), str(dst)], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0, run.stdout + run.stderr
    print(run.stdout)
    got = U.f64(np.fromfile(dst, dtype=np.uint16).reshape(T + 1, s.H))

    os_ = U.oracle_shape(s)
    wts = {l: U.oracle_weights(bits[l]) for l in range(s.L)}
    okv = O.OracleKV()
    x = U.f64(xbits)
    want_p = O.run_layers(os_, wts, 0, s.L, x[:T], O.OracleBatch([0, T], [0], [0]), okv)
    want_d = O.run_layers(os_, wts, 0, s.L, x[T:], O.OracleBatch([0, 1], [0], [T]), okv)
    assert U.rel_err(got[:T], want_p) <= U.BF16_TOL
    assert U.rel_err(got[T:], want_d) <= U.BF16_TOL
    U.assert_rms(got[:T], want_p, U.RMS_BF16)
