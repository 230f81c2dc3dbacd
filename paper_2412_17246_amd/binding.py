"""ctypes binding of include/blitz_layer.h: argument marshalling only.

Every step of the hot path runs inside the shared library; this module loads it, mirrors its
structs, turns negative status codes into exceptions, and uses PyTorch solely to own device
memory, pinned host memory and HIP streams.  There is no CPU fallback: if the library is not
built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libblitzlayer.so")
LIB_FP32_PATH = os.path.join(_PKG, "libblitzlayer_fp32dbg.so")

BZ_FLAG_DRY_RUN = 1
BZ_RUN_NOWAIT = 1
BZ_BUILD_FP32_DEBUG = 1
STATUS = {0: "BZ_OK", -1: "BZ_EINVAL", -2: "BZ_ENOMEM", -3: "BZ_EBUSY", -4: "BZ_ENOTLOADED",
          -5: "BZ_ENOTREADY", -6: "BZ_EHIP", -7: "BZ_ECAPACITY", -8: "BZ_ESTATE"}
KERNEL_CLASSES = ("rmsnorm", "gemm_qkv", "rope_append", "attn_prefill", "attn_decode", "attn_combine",
                  "gemm_o", "gemm_gateup", "gemm_down")
TENSOR_ORDER = ("g1", "wq", "wk", "wv", "wo", "g2", "wg", "wu", "wd")


class BzError(RuntimeError):
    def __init__(self, status: int, what: str, detail: str = ""):
        self.status = status
        self.name = STATUS.get(status, str(status))
        super().__init__(f"{what}: {self.name}" + (f" ({detail})" if detail else ""))


class bz_config(C.Structure):
    _fields_ = [
        ("n_layers", C.c_int32), ("hidden", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("ffn", C.c_int32), ("rms_eps", C.c_float), ("rope_base", C.c_float),
        ("max_seqs", C.c_int32), ("max_seq_len", C.c_int32), ("max_tokens", C.c_int32), ("flags", C.c_int32),
        ("kv_tokens", C.c_int64), ("chunk_bytes", C.c_int64),
        ("compute_stream", C.c_void_p), ("copy_stream", C.c_void_p),
        ("weights_arena", C.c_void_p), ("kv_arena", C.c_void_p), ("workspace", C.c_void_p),
        ("weights_arena_bytes", C.c_size_t), ("kv_arena_bytes", C.c_size_t), ("workspace_bytes", C.c_size_t),
    ]


class bz_sizes(C.Structure):
    _fields_ = [("layer_bytes", C.c_size_t), ("layer_stride", C.c_size_t), ("weights_arena_bytes", C.c_size_t),
                ("kv_arena_bytes", C.c_size_t), ("workspace_bytes", C.c_size_t), ("act_elem_bytes", C.c_size_t)]


class bz_layer_layout(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in TENSOR_ORDER] + [("total", C.c_size_t)]


class bz_batch_desc(C.Structure):
    _fields_ = [("n_seqs", C.c_int32), ("q_start", C.POINTER(C.c_int32)), ("seq_slot", C.POINTER(C.c_int32)),
                ("kv_len_before", C.POINTER(C.c_int32))]


class bz_stats(C.Structure):
    _fields_ = [("bytes_ingested", C.c_uint64), ("layers_requested", C.c_uint64), ("tokens_run", C.c_uint64),
                ("layer_launches", C.c_uint64), ("frontier", C.c_int32), ("reserved", C.c_int32)]


class bz_shard(C.Structure):
    _fields_ = [("src", C.c_void_p), ("offset", C.c_size_t), ("bytes", C.c_size_t), ("src_is_device", C.c_int32),
                ("reserved_", C.c_int32)]


BZ_MAX_SHARDS = 16


class bz_plan_node(C.Structure):
    _fields_ = [("id", C.c_int32), ("n_gpus", C.c_int32), ("leaf", C.c_int32), ("role", C.c_int32),
                ("out_busy", C.c_int32), ("reserved_", C.c_int32), ("gpu_bw", C.c_double)]


class bz_plan_hop(C.Structure):
    _fields_ = [("chain", C.c_int32), ("src", C.c_int32), ("dst", C.c_int32), ("is_tail", C.c_int32),
                ("bw", C.c_double), ("ready_s", C.c_double)]


BZ_PLAN_SOURCE, BZ_PLAN_SPARE, BZ_PLAN_OTHER = 0, 1, 2


class bz_zz_event(C.Structure):
    _fields_ = [("request", C.c_int32), ("instance", C.c_int32), ("layer_a", C.c_int32), ("layer_b", C.c_int32),
                ("frontier", C.c_int32), ("t_ms", C.c_float)]


BZ_ZZ_ZIGZAG = 0
BZ_ZZ_BEST_EFFORT = 1
_NK = len(KERNEL_CLASSES)


class bz_profile(C.Structure):
    _fields_ = [("launches", C.c_uint64 * _NK), ("ms", C.c_double * _NK), ("flops", C.c_double * _NK),
                ("bytes", C.c_double * _NK)]


# name -> (restype, argtypes); also the list of symbols the header declares
_P = C.c_void_p
SIGNATURES = {
    "bz_strerror": (C.c_char_p, [C.c_int]),
    "bz_build_info": (C.c_int, []),
    "bz_last_hip_error": (C.c_char_p, []),
    "bz_query_sizes": (C.c_int, [C.POINTER(bz_config), C.POINTER(bz_sizes)]),
    "bz_layer_layout_of": (C.c_int, [C.POINTER(bz_config), C.POINTER(bz_layer_layout)]),
    "bz_create": (C.c_int, [C.POINTER(bz_config), C.POINTER(_P)]),
    "bz_destroy": (C.c_int, [_P]),
    "bz_sync": (C.c_int, [_P]),
    "bz_load_layer": (C.c_int, [_P, C.c_int, _P, C.c_size_t]),
    "bz_load_layer_from_device": (C.c_int, [_P, C.c_int, _P, C.c_size_t]),
    "bz_load_layer_from_peer": (C.c_int, [_P, C.c_int, _P]),
    "bz_set_ingest_streams": (C.c_int, [_P, C.c_int]),
    "bz_lend_second_copy_stream": (C.c_int, [_P, _P]),
    "bz_load_layer_sharded": (C.c_int, [_P, C.c_int, C.POINTER(bz_shard), C.c_int]),
    "bz_plan_generate": (C.c_int, [C.POINTER(bz_plan_node), C.c_int, C.c_int, C.c_double, C.c_int, C.c_double,
                                   C.POINTER(bz_plan_hop), C.c_int, C.POINTER(C.c_int), C.POINTER(C.c_int),
                                   C.POINTER(C.c_int)]),
    "bz_unload_layer": (C.c_int, [_P, C.c_int]),
    "bz_frontier": (C.c_int, [_P]),
    "bz_layer_ready": (C.c_int, [_P, C.c_int]),
    "bz_wait_layer": (C.c_int, [_P, C.c_int]),
    "bz_layer_ready_ms": (C.c_int, [_P, C.c_int, C.POINTER(C.c_float)]),
    "bz_reset_clock": (C.c_int, [_P]),
    "bz_readback_layer": (C.c_int, [_P, C.c_int, _P]),
    "bz_kv_reserve": (C.c_int, [_P, C.c_int, C.c_int]),
    "bz_kv_release": (C.c_int, [_P, C.c_int]),
    "bz_kv_free_tokens": (C.c_int64, [_P]),
    "bz_kv_write": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_int, _P, _P, C.c_int]),
    "bz_kv_read": (C.c_int, [_P, C.c_int, C.c_int, C.c_int, C.c_int, _P, _P, C.c_int]),
    "bz_batch_create": (C.c_int, [C.POINTER(bz_batch_desc), C.POINTER(_P)]),
    "bz_batch_storage_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int]),
    "bz_batch_create_in": (C.c_int, [C.POINTER(bz_batch_desc), _P, C.c_size_t, _P, C.c_size_t, _P, C.POINTER(_P)]),
    "bz_batch_rebuild": (C.c_int, [_P, C.POINTER(bz_batch_desc), _P]),
    "bz_batch_destroy": (C.c_int, [_P]),
    "bz_batch_tokens": (C.c_int, [_P]),
    "bz_batch_advance": (C.c_int, [_P, _P]),
    "bz_run_layers": (C.c_int, [_P, C.c_int, C.c_int, _P, _P, C.c_int]),
    "bz_export_boundary": (C.c_int, [_P, _P, C.c_size_t, _P, C.c_int]),
    "bz_import_boundary": (C.c_int, [_P, _P, C.c_size_t, _P, C.c_int]),
    "bz_wait_stream": (C.c_int, [_P, _P]),
    "bz_signal_stream": (C.c_int, [_P, _P]),
    "bz_stats_read": (C.c_int, [_P, C.POINTER(bz_stats)]),
    "bz_profile_enable": (C.c_int, [_P, C.c_int]),
    "bz_profile_read": (C.c_int, [_P, C.POINTER(bz_profile)]),
    "bz_zz_simulate": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_double, C.c_double, C.POINTER(C.c_int32),
                                 C.POINTER(C.c_double)]),
    "bz_zz_simulate_weighted": (C.c_int, [C.c_int, C.c_int, C.c_int, C.c_double, C.c_double, C.POINTER(C.c_double),
                                          C.POINTER(C.c_int32), C.POINTER(C.c_double)]),
    "bz_zz_create": (C.c_int, [_P, _P, C.c_int, C.POINTER(_P)]),
    "bz_zz_destroy": (C.c_int, [_P]),
    "bz_zz_submit": (C.c_int, [_P, _P, _P, _P]),
    "bz_zz_run": (C.c_int, [_P]),
    "bz_zz_layers_on_target": (C.c_int, [_P, C.c_int]),
    "bz_zz_trace": (C.c_int, [_P, C.POINTER(bz_zz_event), C.c_int]),
    "bz_op_rmsnorm": (C.c_int, [_P, _P, _P, C.c_int, C.c_int, C.c_float, _P]),
    "bz_op_gemm_workspace_bytes": (C.c_size_t, [C.c_int, C.c_int, C.c_int, C.c_int]),
    "bz_op_gemm": (C.c_int, [C.c_int, _P, _P, _P, _P, C.c_int, C.c_int, C.c_int, _P, C.c_size_t, _P]),
    "bz_op_gemm_static": (C.c_int, [C.c_int, _P, _P, _P, _P, C.c_int, C.c_int, C.c_int, _P]),
}

_libs: Dict[str, C.CDLL] = {}


def load_library(fp32_debug: bool = False) -> C.CDLL:
    path = LIB_FP32_PATH if fp32_debug else LIB_PATH
    if path in _libs:
        return _libs[path]
    if not os.path.exists(path):
        raise RuntimeError(f"{path} is not built: run `python -m paper_2412_17246_amd.build` "
                           "(there is no fallback path)")
    lib = C.CDLL(path)
    for name, (res, args) in SIGNATURES.items():
        fn = getattr(lib, name)
        fn.restype = res
        fn.argtypes = args
    _libs[path] = lib
    return lib


def make_config(shape, *, max_seqs: int, max_seq_len: int, max_tokens: int, kv_tokens: int,
                chunk_bytes: int = 0, flags: int = 0) -> bz_config:
    """`shape` is any object with L, H, Hq, Hkv, d, F, eps, rope_base attributes."""
    c = bz_config()
    c.n_layers, c.hidden, c.n_q_heads, c.n_kv_heads = shape.L, shape.H, shape.Hq, shape.Hkv
    c.head_dim, c.ffn, c.rms_eps, c.rope_base = shape.d, shape.F, shape.eps, shape.rope_base
    c.max_seqs, c.max_seq_len, c.max_tokens, c.flags = max_seqs, max_seq_len, max_tokens, flags
    c.kv_tokens, c.chunk_bytes = kv_tokens, chunk_bytes
    return c


def _ptr(x) -> int:
    """Address of a torch tensor, numpy array or raw integer."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    if isinstance(x, np.ndarray):
        return x.ctypes.data
    return x.data_ptr()


def _i32(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _desc(q_start, seq_slot, kv_len_before):
    qs, sl, kb = _i32(q_start), _i32(seq_slot), _i32(kv_len_before)
    if qs.size != sl.size + 1 or kb.size != sl.size:
        raise ValueError("q_start must have one more entry than seq_slot / kv_len_before")
    d = bz_batch_desc(int(sl.size), qs.ctypes.data_as(C.POINTER(C.c_int32)), sl.ctypes.data_as(C.POINTER(C.c_int32)),
                      kb.ctypes.data_as(C.POINTER(C.c_int32)))
    return d, (qs, sl, kb)


class Batch:
    """A packed batch.  With `storage` = (device uint8 tensor, pinned uint8 tensor of twice its size, stream)
    the batch lives in that memory, is uploaded asynchronously and can be rebuilt in place; without, the
    library allocates and uploads synchronously."""

    def __init__(self, lib: C.CDLL, q_start: Sequence[int], seq_slot: Sequence[int], kv_len_before: Sequence[int],
                 storage=None):
        self._lib = lib
        d, keep = _desc(q_start, seq_slot, kv_len_before)
        h = _P()
        self._storage = storage
        if storage is None:
            rc = lib.bz_batch_create(C.byref(d), C.byref(h))
        else:
            dev, pinned, stream = storage
            rc = lib.bz_batch_create_in(C.byref(d), dev.data_ptr(), dev.numel(), pinned.data_ptr(), pinned.numel(),
                                        stream.cuda_stream if stream is not None else 0, C.byref(h))
        if rc:
            raise BzError(rc, "bz_batch_create", lib.bz_last_hip_error().decode())
        self.handle = h
        self.T = int(keep[0][-1])
        self.B = int(keep[1].size)

    def rebuild(self, q_start, seq_slot, kv_len_before, stream=None) -> None:
        d, keep = _desc(q_start, seq_slot, kv_len_before)
        if stream is None and self._storage is not None:
            stream = self._storage[2]
        rc = self._lib.bz_batch_rebuild(self.handle, C.byref(d), stream.cuda_stream if stream is not None else 0)
        if rc:
            raise BzError(rc, "bz_batch_rebuild", self._lib.bz_last_hip_error().decode())
        self.T = int(keep[0][-1])
        self.B = int(keep[1].size)

    def close(self):
        if self.handle:
            self._lib.bz_batch_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Instance:
    """One serving instance on the current GPU.  Arenas are torch tensors, streams are torch streams."""

    def __init__(self, shape, *, max_seqs: int, max_seq_len: int, max_tokens: int, kv_tokens: int,
                 chunk_bytes: int = 0, fp32_debug: bool = False, dry_run: bool = False,
                 compute_stream=None, copy_stream=None, device: str = "cuda:0"):
        self.lib = load_library(fp32_debug)
        self.shape = shape
        self.fp32_debug = fp32_debug
        cfg = make_config(shape, max_seqs=max_seqs, max_seq_len=max_seq_len, max_tokens=max_tokens,
                          kv_tokens=kv_tokens, chunk_bytes=chunk_bytes, flags=BZ_FLAG_DRY_RUN if dry_run else 0)
        self.sizes = bz_sizes()
        self._check(self.lib.bz_query_sizes(C.byref(cfg), C.byref(self.sizes)), "bz_query_sizes")
        self.layout = bz_layer_layout()
        self._check(self.lib.bz_layer_layout_of(C.byref(cfg), C.byref(self.layout)), "bz_layer_layout_of")
        self.dry_run = dry_run
        self._keep = {}               # layer -> source buffers borrowed by the library while the layer is loaded
        if not dry_run:
            import torch
            self.torch = torch
            self.device = torch.device(device)
            self.compute_stream = compute_stream or torch.cuda.Stream(device=self.device)
            self.copy_stream = copy_stream or torch.cuda.Stream(device=self.device)
            self.weights_arena = torch.empty(self.sizes.weights_arena_bytes, dtype=torch.uint8, device=self.device)
            self.kv_arena = torch.zeros(self.sizes.kv_arena_bytes, dtype=torch.uint8, device=self.device)
            self.workspace = torch.empty(self.sizes.workspace_bytes, dtype=torch.uint8, device=self.device)
            cfg.compute_stream = self.compute_stream.cuda_stream
            cfg.copy_stream = self.copy_stream.cuda_stream
            cfg.weights_arena, cfg.weights_arena_bytes = self.weights_arena.data_ptr(), self.weights_arena.numel()
            cfg.kv_arena, cfg.kv_arena_bytes = self.kv_arena.data_ptr(), self.kv_arena.numel()
            cfg.workspace, cfg.workspace_bytes = self.workspace.data_ptr(), self.workspace.numel()
            torch.cuda.synchronize(self.device)
        self.cfg = cfg
        h = _P()
        self._check(self.lib.bz_create(C.byref(cfg), C.byref(h)), "bz_create")
        self.handle = h

    # -- helpers
    def _check(self, rc: int, what: str) -> int:
        if rc < 0:
            raise BzError(rc, what, self.lib.bz_last_hip_error().decode() if rc == -6 else "")
        return rc

    @property
    def layer_bytes(self) -> int:
        return int(self.sizes.layer_bytes)

    @property
    def act_dtype(self):
        return self.torch.float32 if self.fp32_debug else self.torch.bfloat16

    def close(self):
        if getattr(self, "handle", None):
            self.lib.bz_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    # -- layer blobs
    def pack_layer(self, tensors: Dict[str, np.ndarray]) -> np.ndarray:
        """Lays the nine tensors (uint16 bf16 bit patterns) out as one layer blob (uint8)."""
        blob = np.empty(self.layer_bytes, dtype=np.uint8)
        for name in TENSOR_ORDER:
            t = np.ascontiguousarray(tensors[name], dtype=np.uint16).reshape(-1).view(np.uint8)
            off = getattr(self.layout, name)
            blob[off:off + t.size] = t
        return blob

    def pinned_blob(self, blob: np.ndarray):
        """Copies a blob into a new pinned host tensor."""
        t = self.torch.empty(blob.size, dtype=self.torch.uint8, pin_memory=True)
        t.numpy()[:] = blob
        return t

    # -- ingest
    def set_ingest_streams(self, n: int) -> None:
        self._check(self.lib.bz_set_ingest_streams(self.handle, n), "bz_set_ingest_streams")

    def lend_second_copy_stream(self, stream) -> None:
        """A torch stream of the caller's as the second ingest stream (kept alive by this object)."""
        self._check(self.lib.bz_lend_second_copy_stream(self.handle, stream.cuda_stream), "bz_lend_second_copy_stream")
        self.copy_stream2 = stream

    def load_layer(self, layer: int, pinned) -> None:
        self._check(self.lib.bz_load_layer(self.handle, layer, _ptr(pinned), pinned.numel()), "bz_load_layer")
        self._keep[layer] = [pinned]

    def load_layer_from_peer(self, layer: int, peer: "Instance") -> None:
        """One hop of a forwarding chain: the layer comes from `peer`'s copy as soon as that has landed."""
        self._check(self.lib.bz_load_layer_from_peer(self.handle, layer, peer.handle), "bz_load_layer_from_peer")
        self._keep[layer] = [peer]

    def load_layer_from_device(self, layer: int, dev) -> None:
        self._check(self.lib.bz_load_layer_from_device(self.handle, layer, _ptr(dev), dev.numel()),
                    "bz_load_layer_from_device")
        self._keep[layer] = [dev]

    def drop_sources(self) -> None:
        """Lets go of the source buffers of layers that are resident by now (the library borrows a source
        only until its layer has landed)."""
        for layer in list(self._keep):
            if self.layer_ready(layer):
                del self._keep[layer]

    def load_layer_sharded(self, layer: int, shards) -> None:
        """shards: sequence of (source tensor, byte offset in the layer); each source supplies its
        whole length.  Host tensors must be pinned."""
        arr = (bz_shard * len(shards))()
        for j, (t, off) in enumerate(shards):
            arr[j] = bz_shard(_ptr(t), int(off), t.numel() * t.element_size(), 1 if t.is_cuda else 0, 0)
        self._check(self.lib.bz_load_layer_sharded(self.handle, layer, arr, len(shards)), "bz_load_layer_sharded")
        self._keep[layer] = [t for t, _ in shards]

    def unload_layer(self, layer: int) -> None:
        self._check(self.lib.bz_unload_layer(self.handle, layer), "bz_unload_layer")
        self._keep.pop(layer, None)

    def frontier(self) -> int:
        return self._check(self.lib.bz_frontier(self.handle), "bz_frontier")

    def layer_ready(self, layer: int) -> bool:
        return bool(self._check(self.lib.bz_layer_ready(self.handle, layer), "bz_layer_ready"))

    def wait_layer(self, layer: int) -> None:
        self._check(self.lib.bz_wait_layer(self.handle, layer), "bz_wait_layer")

    def layer_ready_ms(self, layer: int) -> float:
        v = C.c_float()
        self._check(self.lib.bz_layer_ready_ms(self.handle, layer, C.byref(v)), "bz_layer_ready_ms")
        return float(v.value)

    def reset_clock(self) -> None:
        self._check(self.lib.bz_reset_clock(self.handle), "bz_reset_clock")

    def readback_layer(self, layer: int) -> np.ndarray:
        out = np.empty(self.layer_bytes, dtype=np.uint8)
        self._check(self.lib.bz_readback_layer(self.handle, layer, out.ctypes.data), "bz_readback_layer")
        return out

    def sync(self) -> None:
        self._check(self.lib.bz_sync(self.handle), "bz_sync")

    # -- KV
    def kv_reserve(self, slot: int, capacity: int) -> None:
        self._check(self.lib.bz_kv_reserve(self.handle, slot, capacity), "bz_kv_reserve")

    def kv_release(self, slot: int) -> None:
        self._check(self.lib.bz_kv_release(self.handle, slot), "bz_kv_release")

    def kv_free_tokens(self) -> int:
        return int(self._check(self.lib.bz_kv_free_tokens(self.handle), "bz_kv_free_tokens"))

    def kv_write(self, layer: int, slot: int, pos0: int, n: int, k, v) -> None:
        is_host = int(isinstance(k, np.ndarray))
        self._check(self.lib.bz_kv_write(self.handle, layer, slot, pos0, n, _ptr(k), _ptr(v), is_host), "bz_kv_write")

    def kv_read(self, layer: int, slot: int, pos0: int, n: int, k, v) -> None:
        is_host = int(isinstance(k, np.ndarray))
        self._check(self.lib.bz_kv_read(self.handle, layer, slot, pos0, n, _ptr(k), _ptr(v), is_host), "bz_kv_read")

    # -- batches and execution
    def batch(self, q_start, seq_slot, kv_len_before, storage=None) -> Batch:
        return Batch(self.lib, q_start, seq_slot, kv_len_before, storage)

    def batch_storage(self, max_seqs: int, max_tokens: int, max_seq_len: int):
        """Memory for a batch that is built and rebuilt without allocation: (device tensor, pinned tensor of
        twice the size, this instance's compute stream) for `batch(..., storage=...)`."""
        n = int(self.lib.bz_batch_storage_bytes(max_seqs, max_tokens, max_seq_len))
        dev = self.torch.empty(n, dtype=self.torch.uint8, device=self.device)
        pinned = self.torch.empty(2 * n, dtype=self.torch.uint8, pin_memory=True)
        return dev, pinned, self.compute_stream

    def batch_advance(self, batch: Batch) -> None:
        self._check(self.lib.bz_batch_advance(self.handle, batch.handle), "bz_batch_advance")

    def run_layers(self, a: int, b: int, batch: Batch, hidden, flags: int = 0, after_current_stream: bool = True) -> None:
        """`hidden` is normally produced on torch's current stream, the layers run on the instance's compute
        stream: unless told otherwise the compute stream is first made to wait (on the device) for the work
        enqueued so far on the current stream.  Reading the result needs sync() or signal_stream()."""
        if after_current_stream:
            cur = self.torch.cuda.current_stream(self.device)
            if cur.cuda_stream != self.compute_stream.cuda_stream:
                self._check(self.lib.bz_wait_stream(self.handle, cur.cuda_stream), "bz_wait_stream")
        self._check(self.lib.bz_run_layers(self.handle, a, b, batch.handle, _ptr(hidden), flags), "bz_run_layers")

    def wait_stream(self, stream) -> None:
        self._check(self.lib.bz_wait_stream(self.handle, stream.cuda_stream), "bz_wait_stream")

    def signal_stream(self, stream=None) -> None:
        """Makes `stream` (default: torch's current stream) wait for the compute stream's work so far."""
        stream = stream or self.torch.cuda.current_stream(self.device)
        self._check(self.lib.bz_signal_stream(self.handle, stream.cuda_stream), "bz_signal_stream")

    def export_boundary(self, hidden, T: int, buf) -> None:
        is_host = int(isinstance(buf, np.ndarray) or (hasattr(buf, "is_cuda") and not buf.is_cuda))
        self._check(self.lib.bz_export_boundary(self.handle, _ptr(hidden), T, _ptr(buf), is_host), "bz_export_boundary")

    def import_boundary(self, hidden, T: int, buf) -> None:
        is_host = int(isinstance(buf, np.ndarray) or (hasattr(buf, "is_cuda") and not buf.is_cuda))
        self._check(self.lib.bz_import_boundary(self.handle, _ptr(hidden), T, _ptr(buf), is_host), "bz_import_boundary")

    # -- counters
    def stats(self) -> dict:
        s = bz_stats()
        self._check(self.lib.bz_stats_read(self.handle, C.byref(s)), "bz_stats_read")
        return {n: int(getattr(s, n)) for n, _ in bz_stats._fields_ if n != "reserved"}

    def profile_enable(self, on: bool) -> None:
        self._check(self.lib.bz_profile_enable(self.handle, int(on)), "bz_profile_enable")

    def profile_read(self) -> dict:
        p = bz_profile()
        self._check(self.lib.bz_profile_read(self.handle, C.byref(p)), "bz_profile_read")
        return {name: {"launches": int(p.launches[i]), "ms": float(p.ms[i]), "flops": float(p.flops[i]),
                       "bytes": float(p.bytes[i])} for i, name in enumerate(KERNEL_CLASSES)}


def zz_simulate(policy: int, n_layers: int, n_requests: int, load_time: float, source_free_at: float = 0.0,
                fp32_debug: bool = False, layer_time: Optional[Sequence[float]] = None):
    """Virtual-time run of the scheduler's decision code: (layers on target, finish time) per request.
    layer_time: time of one layer of each request (default: 1 for all)."""
    lib = load_library(fp32_debug)
    T = (C.c_int32 * n_requests)()
    fin = (C.c_double * n_requests)()
    if layer_time is None:
        rc = lib.bz_zz_simulate(policy, n_layers, n_requests, load_time, source_free_at, T, fin)
    else:
        if len(layer_time) != n_requests:
            raise ValueError("layer_time needs one entry per request")
        w = (C.c_double * n_requests)(*[float(x) for x in layer_time])
        rc = lib.bz_zz_simulate_weighted(policy, n_layers, n_requests, load_time, source_free_at, w, T, fin)
    if rc:
        raise BzError(rc, "bz_zz_simulate")
    return list(T), list(fin)


def plan_generate(nodes, n_targets: int, oversub: float, n_layers: int, layer_bytes: float,
                  fp32_debug: bool = False) -> dict:
    """Scale-plan generation.  nodes: sequence of (id, n_gpus, gpu_bw, leaf, role, out_busy).
    Returns chains (node ids, root first), per-hop bandwidths, per-target ready times, chain tails and
    whether a source with a busy outgoing link had to be used."""
    lib = load_library(fp32_debug)
    arr = (bz_plan_node * max(1, len(nodes)))()
    for i, (nid, gpus, bw, leaf, role, busy) in enumerate(nodes):
        arr[i] = bz_plan_node(int(nid), int(gpus), int(leaf), int(role), 1 if busy else 0, 0, float(bw))
    hops = (bz_plan_hop * max(1, n_targets))()
    n_hops, n_chains, interferes = C.c_int(), C.c_int(), C.c_int()
    rc = lib.bz_plan_generate(arr, len(nodes), n_targets, oversub, n_layers, layer_bytes, hops, max(1, n_targets),
                              C.byref(n_hops), C.byref(n_chains), C.byref(interferes))
    if rc:
        raise BzError(rc, "bz_plan_generate")
    chains = [[] for _ in range(n_chains.value)]
    hop_bw = [[] for _ in range(n_chains.value)]
    ready, tails = {}, []
    for h in hops[:n_hops.value]:
        if not chains[h.chain]:
            chains[h.chain].append(h.src)
        chains[h.chain].append(h.dst)
        hop_bw[h.chain].append(h.bw)
        ready[h.dst] = h.ready_s
        if h.is_tail:
            tails.append(h.dst)
    return {"chains": chains, "hop_bw": hop_bw, "ready": ready, "tails": tails, "interferes": bool(interferes.value)}


class Scheduler:
    """Two-instance request scheduler (best-effort or ZigZag) over one target and one source."""

    def __init__(self, target: "Instance", source: "Instance", policy: int = BZ_ZZ_ZIGZAG):
        self.lib = target.lib
        h = _P()
        rc = self.lib.bz_zz_create(target.handle, source.handle, policy, C.byref(h))
        if rc:
            raise BzError(rc, "bz_zz_create")
        self.handle = h
        self._keep = []

    def submit(self, batch: Batch, hidden_target, hidden_source) -> int:
        self._keep.append((batch, hidden_target, hidden_source))
        rc = self.lib.bz_zz_submit(self.handle, batch.handle, _ptr(hidden_target), _ptr(hidden_source))
        if rc < 0:
            raise BzError(rc, "bz_zz_submit")
        return rc

    def run(self) -> None:
        rc = self.lib.bz_zz_run(self.handle)
        if rc:
            raise BzError(rc, "bz_zz_run", self.lib.bz_last_hip_error().decode() if rc == -6 else "")

    def layers_on_target(self, request: int) -> int:
        rc = self.lib.bz_zz_layers_on_target(self.handle, request)
        if rc < 0:
            raise BzError(rc, "bz_zz_layers_on_target")
        return rc

    def trace(self):
        n = self.lib.bz_zz_trace(self.handle, None, 0)
        buf = (bz_zz_event * max(n, 1))()
        self.lib.bz_zz_trace(self.handle, buf, n)
        return [dict(request=e.request, instance=e.instance, layer_a=e.layer_a, layer_b=e.layer_b,
                     frontier=e.frontier, t_ms=e.t_ms) for e in buf[:n]]

    def close(self):
        if self.handle:
            self.lib.bz_zz_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def op_rmsnorm(x, gain, y, eps: float, stream=None, fp32_debug: bool = False) -> None:
    lib = load_library(fp32_debug)
    rc = lib.bz_op_rmsnorm(_ptr(x), _ptr(gain), _ptr(y), x.shape[0], x.shape[1], eps, stream.cuda_stream if stream else 0)
    if rc:
        raise BzError(rc, "bz_op_rmsnorm")


def op_gemm_workspace_bytes(mode: int, M: int, N: int, K: int, fp32_debug: bool = False) -> int:
    return int(load_library(fp32_debug).bz_op_gemm_workspace_bytes(mode, M, N, K))


def op_gemm(mode: int, a, w, r, c, M: int, N: int, K: int, stream=None, fp32_debug: bool = False,
            workspace=None) -> None:
    lib = load_library(fp32_debug)
    rc = lib.bz_op_gemm(mode, _ptr(a), _ptr(w), _ptr(r), _ptr(c), M, N, K, _ptr(workspace),
                        workspace.numel() * workspace.element_size() if workspace is not None else 0,
                        stream.cuda_stream if stream else 0)
    if rc:
        raise BzError(rc, "bz_op_gemm")


BZ_STATIC_SCRATCH_BYTES = 64 << 20


def op_gemm_static(mode: int, a, w, r, c, M: int, N: int, K: int, stream=None, fp32_debug: bool = False) -> None:
    """bz_op_gemm with the library's static scratch: allocates nothing."""
    lib = load_library(fp32_debug)
    rc = lib.bz_op_gemm_static(mode, _ptr(a), _ptr(w), _ptr(r), _ptr(c), M, N, K, stream.cuda_stream if stream else 0)
    if rc:
        raise BzError(rc, "bz_op_gemm_static", lib.bz_last_hip_error().decode() if rc == -6 else "")
