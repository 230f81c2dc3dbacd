/*
 * blitz_layer.h — C ABI of the single-GPU share of live, layer-level model scaling.
 *
 * The paper scales a serving instance by sending it the model one layer at a time and lets the
 * instance execute whatever prefix of layers it already holds, handing the activation to a fully
 * loaded instance at a layer boundary (section 4, the part on making autoscaling live; section 5.2,
 * the three-step protocol between a paired new and old instance).  On one MI355X that becomes:
 *
 *   - an *instance*: a weight arena for L decoder layers, a KV cache, two HIP streams;
 *   - *layer ingest*: copy layer i's parameter blob from pinned host memory into HBM in chunks
 *     on the copy stream, mark completion with a per-layer event (the host-memory source of
 *     section 1 / section 5.3's parameter pool, overlapped with execution as in section 4);
 *   - the *frontier*: how many leading layers are resident (section 1, challenges: a scaling instance
 *     can execute only the layers whose parameters it already holds, and that set keeps growing);
 *   - *run layers [a,b)* on a packed batch of hidden states with prefill and/or decode sequences
 *     (section 2.1, layer-by-layer execution with a KV cache held in GPU memory), each layer
 *     gated on its own ingest event;
 *   - *boundary export / import*: the activation hand-off between instances (section 4).
 *
 * The arithmetic of a layer is the Llama-family decoder layer (RMSNorm, QKV projection, rotary
 * embedding, causal attention with grouped KV heads, output projection, SwiGLU MLP, pre-norm
 * residuals, no biases); the paper leaves it to its kernel library.
 *
 * Conventions
 *   - All functions return 0 (BZ_OK) or a negative bz_status; none throws, none aborts.
 *   - "device" pointers are HIP device addresses on the current device; "host" pointers are
 *     ordinary host addresses; "pinned" means page-locked host memory (hipHostMalloc).
 *   - Activations are bf16 (2 bytes, row-major).  In the fp32 debug build of the library
 *     (bz_build_info() & BZ_BUILD_FP32_DEBUG) activations and the KV cache are float32; weights
 *     stay bf16 in both builds.
 *   - Work is enqueued on the instance's streams and completes asynchronously; bz_sync() or the
 *     caller's own stream synchronisation makes results visible.
 *   - An instance is not thread-safe: call it from one host thread at a time.
 */
#ifndef BLITZ_LAYER_H
#define BLITZ_LAYER_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum bz_status {
    BZ_OK = 0,
    BZ_EINVAL = -1,      /* bad argument (null, out of range, wrong size, misaligned) */
    BZ_ENOMEM = -2,      /* allocation failed or a caller-provided arena is too small */
    BZ_EBUSY = -3,       /* layer already loading or resident */
    BZ_ENOTLOADED = -4,  /* a layer in [a,b) was never requested with bz_load_layer */
    BZ_ENOTREADY = -5,   /* BZ_RUN_NOWAIT and a layer in [a,b) has not finished loading */
    BZ_EHIP = -6,        /* a HIP runtime call failed; see bz_last_hip_error() */
    BZ_ECAPACITY = -7,   /* KV arena / slot capacity / max_tokens / max_seq_len exceeded */
    BZ_ESTATE = -8,      /* call not valid in this state (e.g. dry-run instance, slot not reserved) */
} bz_status;

enum {
    BZ_FLAG_DRY_RUN = 1,        /* bz_create: build host-side state only, touch no GPU.  Calls that
                                   would enqueue GPU work validate their arguments and then return
                                   BZ_ESTATE. */
};
enum {
    BZ_RUN_NOWAIT = 1,          /* bz_run_layers: fail with BZ_ENOTREADY instead of waiting on ingest */
};
enum {
    BZ_BUILD_FP32_DEBUG = 1,
};

typedef struct bz_instance bz_instance;
typedef struct bz_batch bz_batch;

/* Model shape, capacities and (optionally) caller-owned resources.  Plain data. */
typedef struct bz_config {
    int32_t n_layers;        /* L >= 1 */
    int32_t hidden;          /* H, multiple of 8 */
    int32_t n_q_heads;       /* Hq */
    int32_t n_kv_heads;      /* Hkv, divides Hq; Hq/Hkv in {1,2,4,8} */
    int32_t head_dim;        /* d: 64 or 128 */
    int32_t ffn;             /* F, multiple of 8 */
    float   rms_eps;
    float   rope_base;
    int32_t max_seqs;        /* number of KV slots */
    int32_t max_seq_len;     /* largest sequence length (positions 0..max_seq_len-1) */
    int32_t max_tokens;      /* largest number of packed rows T in one bz_run_layers call */
    int32_t flags;           /* BZ_FLAG_* */
    int64_t kv_tokens;       /* KV arena capacity, in tokens per layer, shared by all slots */
    int64_t chunk_bytes;     /* ingest chunk size; 0 selects the default (32 MiB) */
    void*   compute_stream;  /* hipStream_t for kernels, or NULL: the library creates one */
    void*   copy_stream;     /* hipStream_t for ingest, or NULL: the library creates one */
    void*   weights_arena;   /* device, >= bz_sizes.weights_arena_bytes, 256-byte aligned; NULL: library allocates */
    void*   kv_arena;        /* device, >= bz_sizes.kv_arena_bytes; NULL: library allocates; cleared by bz_create */
    void*   workspace;       /* device, >= bz_sizes.workspace_bytes; NULL: library allocates */
    size_t  weights_arena_bytes;
    size_t  kv_arena_bytes;
    size_t  workspace_bytes;
} bz_config;

typedef struct bz_sizes {
    size_t layer_bytes;          /* exact size of one layer blob */
    size_t layer_stride;         /* distance between layers in the weight arena (256-byte multiple) */
    size_t weights_arena_bytes;
    size_t kv_arena_bytes;
    size_t workspace_bytes;
    size_t act_elem_bytes;       /* 2 (bf16) or 4 (fp32 debug build) */
} bz_sizes;

/* Byte offsets of the nine tensors inside a layer blob.  Every tensor is bf16, row-major;
 * projection matrices are [out_features, in_features].  Order in the blob:
 *   g1[H]  wq[Hq*d,H]  wk[Hkv*d,H]  wv[Hkv*d,H]  wo[H,Hq*d]  g2[H]  wg[F,H]  wu[F,H]  wd[H,F]
 * (wq,wk,wv are adjacent and form one [(Hq+2Hkv)*d, H] matrix; wg,wu likewise [2F, H]). */
typedef struct bz_layer_layout {
    size_t g1, wq, wk, wv, wo, g2, wg, wu, wd;
    size_t total;                /* == bz_sizes.layer_bytes */
} bz_layer_layout;

/* One packed ragged batch.  Sequence s owns rows q_start[s] .. q_start[s+1]-1 of the [T,H] hidden
 * states, lives in KV slot seq_slot[s], and already has kv_len_before[s] cached positions; its new
 * tokens take positions kv_len_before[s] + 0, 1, ...  A sequence with exactly one new token is
 * served by the decode-attention kernel, one with more by the prefill kernel; both may be mixed
 * in one batch (section 5.4, PD colocation).  All three arrays are host memory, read during the
 * call only. */
typedef struct bz_batch_desc {
    int32_t        n_seqs;          /* B >= 1 */
    const int32_t* q_start;         /* [B+1], q_start[0] == 0, non-decreasing; T = q_start[B] */
    const int32_t* seq_slot;        /* [B], distinct, each in [0, max_seqs) */
    const int32_t* kv_len_before;   /* [B], >= 0 */
} bz_batch_desc;

typedef struct bz_stats {
    uint64_t bytes_ingested;     /* sum of layer bytes whose copies were enqueued */
    uint64_t layers_requested;
    uint64_t tokens_run;         /* sum over bz_run_layers calls of T * (b - a) */
    uint64_t layer_launches;     /* layers enqueued by bz_run_layers */
    int32_t  frontier;
    int32_t  reserved;
} bz_stats;

/* Kernel classes for bz_profile_read. */
enum {
    BZ_K_RMSNORM = 0, BZ_K_GEMM_QKV, BZ_K_ROPE_APPEND, BZ_K_ATTN_PREFILL, BZ_K_ATTN_DECODE,
    BZ_K_ATTN_COMBINE, BZ_K_GEMM_O, BZ_K_GEMM_GATEUP, BZ_K_GEMM_DOWN, BZ_K_COUNT
};
typedef struct bz_profile {
    uint64_t launches[BZ_K_COUNT];
    double   ms[BZ_K_COUNT];        /* summed HIP-event time of those launches */
    double   flops[BZ_K_COUNT];     /* summed algorithmic flops (2*M*N*K for GEMMs, causal half for attention) */
    double   bytes[BZ_K_COUNT];     /* summed algorithmic HBM bytes (decode attention: K and V read once) */
} bz_profile;

/* ---- pure helpers (no GPU, no instance) ------------------------------------------------ */

const char* bz_strerror(int status);
int         bz_build_info(void);                  /* BZ_BUILD_* bits */
const char* bz_last_hip_error(void);              /* text of the last failed HIP call on this thread */

/* Validates `cfg` (shape limits above) and reports blob, arena and workspace sizes. */
int bz_query_sizes(const bz_config* cfg, bz_sizes* out);
int bz_layer_layout_of(const bz_config* cfg, bz_layer_layout* out);

/* ---- instance ---------------------------------------------------------------------------- */

/* Creates an instance: allocates (or adopts) arenas, creates streams and per-layer events, builds
 * the rotary table (angles in float64 on the host).  This is control-plane work the paper keeps
 * off the scaling path (appendix A.1, pre-created contexts), so it is outside any TTFT figure.
 * Adopted arenas and streams stay owned by the caller and must outlive the instance. */
int bz_create(const bz_config* cfg, bz_instance** out);
int bz_destroy(bz_instance* inst);               /* waits for the instance's streams, frees what the library allocated */
int bz_sync(bz_instance* inst);                  /* waits for the copy streams, then for the compute stream */

/* Layer ingest (section 4: load the next layers while loaded ones execute; section 5.1: layers
 * arrive one by one).  Enqueues chunked async copies of `n` == layer_bytes bytes from pinned host
 * memory `host` into layer i's slot of the weight arena on the copy stream, records the layer's
 * event and returns at once.  `host` is borrowed until the layer is resident.  Layers may be
 * requested in any order.  BZ_EBUSY if layer i is loading or resident.  BZ_EINVAL if `host` is not
 * page-locked memory known to the runtime (from pageable memory every copy would block the caller and
 * nothing would overlap).  If a HIP call fails while the copies are being enqueued the call returns
 * BZ_EHIP and the layer is left in a failed state: it cannot run (BZ_ESTATE) or be requested again
 * (BZ_EBUSY) until bz_unload_layer, which waits for the copies already in flight, has cleared it.
 * The bytes go over in blob order, which is the order the layer reads them (attention weights
 * first, down projection last), and an event is also recorded behind each group of tensors that one
 * stage of the layer needs; bz_run_layers uses them (see there).  See bz_set_ingest_streams for
 * the number of streams the bytes travel on.  The layer counts as resident, for
 * the frontier and every query below, only when all of it has landed. */
int bz_load_layer(bz_instance* inst, int layer, const void* host, size_t n);
/* Number of streams (1, the default, or 2) that later bz_load_layer / bz_load_layer_from_device calls
 * spread a layer over.  With 2, each tensor group is cut in two halves that travel concurrently, one
 * on the copy stream and one on a second stream the library owns; the layer's event, on the copy
 * stream, follows both.  Two transfers in flight keep a host link busier than one (57.1 against
 * 55.8 GB/s measured), but not from every host buffer: from some pinned allocations of a virtualised
 * host two concurrent transfers ran at 46 GB/s where one kept 55.8.  A caller that cares measures
 * both on its own buffers (bench.py does, during warm-up).  BZ_EINVAL for any other n. */
int bz_set_ingest_streams(bz_instance* inst, int n);
/* Makes `stream` (a hipStream_t of the caller's, distinct from the instance's compute and copy streams) the
 * second ingest stream, in place of one the library would create; the caller keeps it alive until
 * bz_destroy and owns it afterwards.  For processes that run several instances: a process has few hardware
 * queues, streams are dealt onto them in creation order, and an ingest stream that lands on the compute
 * stream's queue serialises copies and kernels; a caller that creates its streams once, early, and lends
 * them to every instance keeps the assignment it has measured.  Waits for transfers still on a stream it
 * replaces.  Does not change the number of streams in use (bz_set_ingest_streams).  BZ_ESTATE on a dry-run
 * instance. */
int bz_lend_second_copy_stream(bz_instance* inst, void* stream);
/* Same, from a device buffer (a resident peer's copy: one hop of section 5.1's forwarding chain). */
int bz_load_layer_from_device(bz_instance* inst, int layer, const void* dev, size_t n);
/* Serial forwarding chain (section 5.1: a node passes layer k on while it receives layer k + 1): loads layer
 * `layer` from the copy that `peer`, an instance of the same shape on the same GPU, holds or is still receiving.
 * Returns at once; on the device the transfer starts when the peer's layer has landed, so a chain
 * S -> T1 -> T2 is set up by requesting every layer on T1 and then on T2 without waiting in between.  The peer
 * must keep the layer (no bz_unload_layer, no bz_destroy) until it is resident here.  BZ_ENOTLOADED if the
 * peer's layer was never requested, BZ_ESTATE if it is in the failed state or either instance is a dry run,
 * BZ_EINVAL for peer == inst or another shape; otherwise as bz_load_layer. */
int bz_load_layer_from_peer(bz_instance* inst, int layer, bz_instance* peer);
/* Parallel sharded transfer (section 5.1, the optimisation that sends the shards of a layer from
 * several sources at once): the layer's bytes arrive as n_shards <= BZ_MAX_SHARDS contiguous pieces, each from its
 * own source buffer, spread over two extra copy streams so that transfers from different sources
 * overlap; the layer's event fires when all of them have landed (the point at which the paper's
 * all-gather has finished).
 * Shard j copies `bytes` bytes from `src` (pinned host memory, or device memory if src_is_device) to
 * byte `offset` of the layer; the shards, in any order, must cover [0, layer_bytes) exactly once
 * (BZ_EINVAL otherwise).  Sources are borrowed until the layer is resident.  BZ_EBUSY as above. */
#define BZ_MAX_SHARDS 16
typedef struct bz_shard {
    const void* src;
    size_t      offset;
    size_t      bytes;
    int32_t     src_is_device;
    int32_t     reserved_;
} bz_shard;
int bz_load_layer_sharded(bz_instance* inst, int layer, const bz_shard* shards, int n_shards);
/* Forgets layer i (waits for the instance's streams first); it must be loaded again before it can run.
 * Also the only way out of the failed state a broken-off load leaves. */
int bz_unload_layer(bz_instance* inst, int layer);

/* Number k of leading layers [0,k) that are resident now.  Never blocks. */
int bz_frontier(bz_instance* inst);
/* 1 if layer i is resident, 0 if requested but still in flight or never requested.  Never blocks. */
int bz_layer_ready(bz_instance* inst, int layer);
/* Blocks the host until layer i is resident.  BZ_ENOTLOADED if it was never requested. */
int bz_wait_layer(bz_instance* inst, int layer);
/* Milliseconds from the first bz_load_layer (since creation or the last bz_reset_clock) to layer
 * i's residency, from HIP events on the copy stream.  Layer must be resident. */
int bz_layer_ready_ms(bz_instance* inst, int layer, float* ms);
int bz_reset_clock(bz_instance* inst);
/* Debug: copies layer i's device bytes to host memory `host` (layer_bytes) and waits. */
int bz_readback_layer(bz_instance* inst, int layer, void* host);

/* ---- KV slots ------------------------------------------------------------------------------ */

/* Reserves room for `capacity_tokens` positions (in every layer) for slot `slot`; the arena hands
 * out multiples of 32 positions, so the request is rounded up.  BZ_ECAPACITY if the arena has no
 * contiguous room or capacity_tokens > max_seq_len, BZ_EBUSY if the slot is reserved already. */
int bz_kv_reserve(bz_instance* inst, int slot, int capacity_tokens);
int bz_kv_release(bz_instance* inst, int slot);
int64_t bz_kv_free_tokens(bz_instance* inst);    /* largest reservable capacity right now */
/* Writes / reads n positions starting at pos0 of (layer, slot): k and v are [n, Hkv, d] activation
 * elements, token-major, in host (is_host != 0) or device memory.  Ordered on the compute stream;
 * host transfers complete before return and are staged through the instance's workspace (nothing is
 * allocated), so they must not be issued from another thread while bz_run_layers is being called. */
int bz_kv_write(bz_instance* inst, int layer, int slot, int pos0, int n, const void* k, const void* v, int is_host);
int bz_kv_read(bz_instance* inst, int layer, int slot, int pos0, int n, void* k, void* v, int is_host);

/* ---- batches ------------------------------------------------------------------------------- */

/* Builds the device-side description of a packed batch (offsets, per-token sequence ids, attention
 * work lists).  A batch is independent of any instance and can be run by several (the two
 * instances of a split run share one).  This form allocates device memory and uploads synchronously:
 * for set-up code.  A serving loop whose batch changes every step (section 6, continuous batching)
 * uses bz_batch_create_in / bz_batch_rebuild below. */
int bz_batch_create(const bz_batch_desc* desc, bz_batch** out);
/* The same without allocation and without a blocking copy.  The caller lends `device_mem` (device,
 * 32-byte aligned, device_bytes >= bz_batch_storage_bytes(...) of the largest batch it will hold) and
 * `pinned_mem` (page-locked host memory, pinned_bytes >= 2 * device_bytes: two staging halves used in
 * turn), both until bz_batch_destroy.  The description is laid out in the staging and uploaded with one
 * asynchronous copy on `stream` (a hipStream_t, normally the compute stream of the instance that runs
 * the batch next); the call returns at once.  bz_run_layers on an instance whose compute stream is a
 * different one waits, on the device, for the upload.  BZ_ECAPACITY if the batch does not fit. */
size_t bz_batch_storage_bytes(int max_seqs, int max_tokens, int max_seq_len);
int bz_batch_create_in(const bz_batch_desc* desc, void* device_mem, size_t device_bytes, void* pinned_mem,
                       size_t pinned_bytes, void* stream, bz_batch** out);
/* Replaces the description of a batch made by bz_batch_create_in (sequences joined or left, new
 * lengths) in the same storage, asynchronously on `stream`.  Runs already enqueued keep the old
 * description: the upload is ordered behind them (behind runs on other streams through events).  The
 * host blocks only if the upload of the last-but-one build has not started yet (two builds ahead of
 * the device).  A refused description (BZ_EINVAL, BZ_ECAPACITY) leaves the batch as it was;
 * BZ_ESTATE for a batch that was made by bz_batch_create. */
int bz_batch_rebuild(bz_batch* batch, const bz_batch_desc* desc, void* stream);
int bz_batch_destroy(bz_batch* batch);
int bz_batch_tokens(const bz_batch* batch);
/* For a batch in which every sequence has exactly one new token: enqueue, on `inst`'s compute
 * stream, kv_len_before[s] += 1 for all s — the next decode step of the same sequences.  The
 * batch's list of cache chunks is rebuilt on the device in the same step; it has room for 16384
 * positions of growth per sequence since the batch was built (less if lent storage is smaller),
 * beyond which the call returns BZ_ECAPACITY and changes nothing (build a new batch).
 * A batch shared by two instances with different compute streams needs no host synchronisation:
 * the update waits, on the device, for runs of the batch enqueued earlier on the other stream, and
 * runs enqueued later on the other stream wait for the update. */
int bz_batch_advance(bz_instance* inst, bz_batch* batch);

/* ---- execution ------------------------------------------------------------------------------ */

/* Runs decoder layers [a,b) in order on the compute stream over `hidden` — device, [T,H]
 * activation elements, updated in place — appending the new tokens' K/V of those layers to the
 * instance's cache.  The compute stream waits on layer i's ingest before it runs layer i, so the
 * call may be issued while later layers are still arriving (section 5.2, step 2 of the protocol).
 * The paper gates at layer granularity, and so does this call for every layer but the last of
 * the range: if layer b-1 is still in flight and was requested with bz_load_layer or
 * bz_load_layer_from_device, each of its stages waits only for the tensors it reads (QKV group
 * before the first norm, wo and the second norm's gain before the output projection, gate/up
 * before the MLP, the whole layer before the down projection), so its attention runs while its
 * MLP weights arrive.  A sharded layer is waited for as a whole.  With BZ_RUN_NOWAIT the call
 * returns BZ_ENOTREADY instead if any layer of [a,b) is not resident yet.  Results do not depend on
 * a, b, the frontier or timing: running [a,k) then [k,b) (on this or another instance holding the
 * same weights) is bit-identical to running [a,b).
 * BZ_ENOTLOADED if a layer of [a,b) was never requested, BZ_ECAPACITY if the batch has more rows than
 * max_tokens or a sequence outgrows its slot, BZ_ESTATE if a slot of the batch is not reserved. */
int bz_run_layers(bz_instance* inst, int a, int b, const bz_batch* batch, void* hidden, int flags);

/* Activation hand-off at a layer boundary (section 4, cooperative execution: the scaled instance
 * passes the activation of its last resident layer on to the loaded one).  Bit-preserving copy of T rows of H activation elements between
 * `hidden` (device) and `buf` (device, or pinned/ordinary host when is_host != 0), ordered on the
 * compute stream.  Host copies complete before return. */
int bz_export_boundary(bz_instance* inst, const void* hidden, size_t T, void* buf, int is_host);
int bz_import_boundary(bz_instance* inst, void* hidden, size_t T, const void* buf, int is_host);

/* Ordering against a stream the library does not own.  bz_wait_stream: the compute stream waits for
 * everything enqueued so far on `stream` (a caller that prepared `hidden` on its own stream calls this
 * before bz_run_layers).  bz_signal_stream: `stream` waits for everything enqueued so far on the compute
 * stream (before the caller reads the result on its own stream).  Both are device-side waits and return
 * at once; a no-op when `stream` is the compute stream. */
int bz_wait_stream(bz_instance* inst, void* stream);
int bz_signal_stream(bz_instance* inst, void* stream);

/* ---- counters -------------------------------------------------------------------------------- */

int bz_stats_read(bz_instance* inst, bz_stats* out);
/* Per-kernel-class HIP-event timing of bz_run_layers.  While enabled every kernel launch is
 * bracketed by two events on the compute stream; bz_profile_read waits for the stream, sums the
 * intervals recorded since the last read and clears them. */
int bz_profile_enable(bz_instance* inst, int on);
int bz_profile_read(bz_instance* inst, bz_profile* out);

/* ---- request scheduling during live scaling ------------------------------------------------- */
/* Section 5.2: while the target instance is still loading, request batches are split between the
 * target (the layers it has) and the source (the rest).  Two policies:
 *   BZ_ZZ_BEST_EFFORT  each batch runs as many layers as are resident on the target when it is
 *                      dispatched there (at most half of the model), the rest on the source, in
 *                      arrival order;
 *   BZ_ZZ_ZIGZAG       the ILP-free ZigZag policy: the target runs ONE layer of the first batch (in
 *                      arrival order) whose next layer is resident and keeps the batch queued; the
 *                      source, whenever it is idle, takes the first unfinished batch and runs all of
 *                      its remaining layers.  When both are free at once the source chooses first;
 *                      the source never takes a batch whose layer the target is executing.
 * Results do not depend on the schedule: every batch's output equals the unsplit run bit for bit. */
enum { BZ_ZZ_ZIGZAG = 0, BZ_ZZ_BEST_EFFORT = 1 };
typedef struct bz_zz bz_zz;
typedef struct bz_zz_event {
    int32_t request;     /* index returned by bz_zz_submit */
    int32_t instance;    /* 0 = target, 1 = source */
    int32_t layer_a;     /* layers [layer_a, layer_b) were enqueued */
    int32_t layer_b;
    int32_t frontier;    /* the target's frontier when the decision was taken */
    float   t_ms;        /* host time since bz_zz_run started */
} bz_zz_event;

/* Decision logic alone, in virtual time (no GPU): one layer of one batch takes one time unit on
 * either instance, layer k of the target is resident from k * load_time on, the source is busy
 * until source_free_at.  Writes, per request, the layers run on the target and the time it left
 * the source.  Same decision code as bz_zz_run. */
int bz_zz_simulate(int policy, int n_layers, int n_requests, double load_time, double source_free_at,
                   int32_t* layers_on_target, double* finish_time);
/* The same with a time per layer for every request (section 5.4: the time of a layer grows with the
 * number of batched tokens, so the formulation gets one factor per request batch, found by profiling):
 * one layer of request r takes layer_time[r] (host, [n_requests], each > 0 and finite) on either
 * instance, in the unit load_time and source_free_at are given in.  The decision rules are those of
 * bz_zz_simulate; NULL means 1 for every request.  BZ_EINVAL for a factor that is not positive. */
int bz_zz_simulate_weighted(int policy, int n_layers, int n_requests, double load_time, double source_free_at,
                            const double* layer_time, int32_t* layers_on_target, double* finish_time);

/* A scheduler over two instances holding the same model (the source fully resident; the target
 * loading: the caller issues bz_load_layer on it before or while bz_zz_run runs).  Both instances
 * must have KV slots reserved for every submitted batch. */
int bz_zz_create(bz_instance* target, bz_instance* source, int policy, bz_zz** out);
int bz_zz_destroy(bz_zz* zz);
/* Queues a batch (arrival order = submission order).  `hidden_target` (device, [T,H]) holds the
 * input and is the buffer the target works in; `hidden_source` (device, [T,H], distinct) receives
 * the activation at the hand-off and holds the final output.  Returns the request index (>= 0). */
int bz_zz_submit(bz_zz* zz, const bz_batch* batch, void* hidden_target, void* hidden_source);
/* Runs every submitted batch to completion under the policy, polling the target's frontier and the
 * two compute streams; returns when all outputs are complete. */
int bz_zz_run(bz_zz* zz);
int bz_zz_layers_on_target(const bz_zz* zz, int request);
/* Copies up to max_events decision records; returns the total number recorded. */
int bz_zz_trace(const bz_zz* zz, bz_zz_event* out, int max_events);

/* ---- single operations (the layer's steps, exposed for tests and micro-benchmarks) ---------- */
/* All pointers are device memory; work is enqueued on `stream` (a hipStream_t, NULL = default).
 * Activations are activation elements (bf16, or float in the fp32 debug build); weights bf16. */

/* y[T,H] = x / sqrt(mean(x^2) + eps) * gain */
int bz_op_rmsnorm(const void* x, const void* gain, void* y, int T, int H, float eps, void* stream);
/* mode 0: c[M,N] = a[M,K] * w[N,K]^T
 * mode 1: c[M,N] = r[M,N] + a * w^T          (r may alias c)
 * mode 2: w is [2N,K] (gate rows then up rows): c[M,N] = silu(a*wg^T) .* (a*wu^T)
 * `workspace`: device scratch of at least bz_op_gemm_workspace_bytes(mode, M, N, K) bytes, 16-byte
 * aligned.  Problems of up to 256 rows split K over workgroups and keep partial sums there;
 * larger ones whose tile count is below the number of compute units, or leaves a small last
 * round, split those tiles over K and keep partial tiles there.  With NULL or too small a workspace
 * a schedule that needs none is used (same result up to fp32 summation order); bz_run_layers always
 * provides one. */
size_t bz_op_gemm_workspace_bytes(int mode, int M, int N, int K);
int bz_op_gemm(int mode, const void* a, const void* w, const void* r, void* c, int M, int N, int K, void* workspace,
               size_t workspace_bytes, void* stream);

/* bz_op_gemm for callers that cannot allocate device memory and have no workspace to hand over: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, kernels,
 * schedules and results (bit for bit) as bz_op_gemm called with a sufficient workspace; the scratch comes
 * from a static device array of BZ_STATIC_SCRATCH_BYTES that each GPU the library runs on holds until
 * the process ends.  The call allocates and frees nothing.  BZ_ECAPACITY, before any GPU work, if
 * bz_op_gemm_workspace_bytes(mode, M, N, K) exceeds BZ_STATIC_SCRATCH_BYTES (a problem of up to 256
 * rows whose split-K partial sums are larger; every larger problem fits).  All calls on one GPU share
 * the one array: calls that overlap in time on the same GPU (two streams, two threads) race; issue
 * them on one stream or order them with events.  Nothing in the array has to be cleared between calls. */
#define BZ_STATIC_SCRATCH_BYTES (64u << 20)
int bz_op_gemm_static(int mode, const void* a, const void* w, const void* r, void* c, int M, int N, int K,
                      void* stream);

#ifdef __cplusplus
}
#endif
#endif /* BLITZ_LAYER_H */
