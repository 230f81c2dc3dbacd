// Host side of the C ABI: instance state, layer ingest with per-layer events, the frontier,
// KV slots, batches, the per-layer kernel sequence, boundary hand-off, counters.
#include <algorithm>
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <new>
#include <string>
#include <vector>

#include "instance.h"

using namespace bz;

namespace {

thread_local std::string g_hip_err;

}  // namespace

namespace bz {
int hip_fail(hipError_t e, const char* what) {
    char buf[256];
    snprintf(buf, sizeof buf, "%s: %s", what, hipGetErrorString(e));
    g_hip_err = buf;
    return BZ_EHIP;
}
}  // namespace bz

namespace {

#define HIP_TRY(call)                                   \
    do {                                                \
        hipError_t e__ = (call);                        \
        if (e__ != hipSuccess) return hip_fail(e__, #call); \
    } while (0)

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }


int validate(const bz_config* c) {
    if (!c) return BZ_EINVAL;
    if (c->n_layers < 1 || c->hidden < 8 || c->hidden % 8) return BZ_EINVAL;
    if (c->head_dim != 64 && c->head_dim != 128) return BZ_EINVAL;
    if (c->n_kv_heads < 1 || c->n_q_heads < c->n_kv_heads || c->n_q_heads % c->n_kv_heads) return BZ_EINVAL;
    const int g = c->n_q_heads / c->n_kv_heads;
    if (g != 1 && g != 2 && g != 4 && g != 8) return BZ_EINVAL;
    if (c->ffn < 8 || c->ffn % 8) return BZ_EINVAL;
    if (!(c->rms_eps > 0.f) || !(c->rope_base > 1.f)) return BZ_EINVAL;
    if (c->max_seqs < 1 || c->max_seq_len < 1 || c->max_tokens < 1) return BZ_EINVAL;
#ifdef BZ_FP32_DEBUG
    if (c->max_seq_len > 16384) return BZ_EINVAL;       // the debug attention keeps a row of scores in LDS
#endif
    if (c->kv_tokens < 1 || c->kv_tokens > 0x7fffffffLL) return BZ_EINVAL;
    if (c->chunk_bytes < 0) return BZ_EINVAL;
    return BZ_OK;
}

void layout_of(const bz_config* c, bz_layer_layout* o) {
    const size_t H = c->hidden, d = c->head_dim, Hq = c->n_q_heads, Hkv = c->n_kv_heads, F = c->ffn;
    size_t p = 0;
    o->g1 = p; p += H * 2;
    o->wq = p; p += Hq * d * H * 2;
    o->wk = p; p += Hkv * d * H * 2;
    o->wv = p; p += Hkv * d * H * 2;
    o->wo = p; p += H * Hq * d * 2;
    o->g2 = p; p += H * 2;
    o->wg = p; p += F * H * 2;
    o->wu = p; p += F * H * 2;
    o->wd = p; p += H * F * 2;
    o->total = p;
}


void ws_layout(const bz_config* c, WsLayout* w) {
    const size_t T = c->max_tokens, e = sizeof(act_t);
    const size_t nqkv = (size_t)(c->n_q_heads + 2 * c->n_kv_heads) * c->head_dim;
    size_t p = 0;
    auto take = [&](size_t bytes) { size_t at = p; p = align_up(p + bytes, 256); return at; };
    w->normed = take(T * c->hidden * e);
    w->qkv = take(T * nqkv * e);
    w->attn = take(T * (size_t)c->n_q_heads * c->head_dim * e);
    w->act = take(T * c->ffn * e);
    const size_t chunks = (c->max_seq_len + kDecodeChunk - 1) / kDecodeChunk;
    w->partial = take((size_t)c->max_seqs * c->n_q_heads * chunks * decode_partial_stride(c->head_dim) * sizeof(float));
    {   // fp32 scratch of the GEMMs: the largest need of the four projections over every row count a
        // call may bring (up to 256 rows: split-K partial sums, a plan per number of 64-row blocks and linear
        // in the rows; beyond: partial tiles of split tiles, which depend on the number of 256-row tiles only)
        const int qd = c->n_q_heads * c->head_dim;
        size_t g = 0;
        auto need = [&](int M) {
            size_t t = gemm_workspace_bytes(0, M, (int)nqkv, c->hidden); if (t > g) g = t;
            t = gemm_workspace_bytes(1, M, c->hidden, qd); if (t > g) g = t;
            t = gemm_workspace_bytes(2, M, c->ffn, c->hidden); if (t > g) g = t;
            t = gemm_workspace_bytes(1, M, c->hidden, c->ffn); if (t > g) g = t;
        };
        for (int M = 64; M <= 256; M += 64) need(M < c->max_tokens ? M : c->max_tokens);   // split-K kernel: per 64-row block
        for (int M = 256; M < c->max_tokens + 256; M += 256) need(M < c->max_tokens ? M : c->max_tokens);
        w->gemm_ws_bytes = g;
        w->gemm_ws = take(g);
    }
    w->rope = take((size_t)c->max_seq_len * c->head_dim * sizeof(float));
    w->slot_off = take((size_t)c->max_seqs * sizeof(int32_t));
    w->slot_cap = take((size_t)c->max_seqs * sizeof(int32_t));
    w->total = p;
}



}  // namespace



namespace {

unsigned char* layer_ptr(bz_instance* I, int l) { return I->weights + (size_t)l * I->sz.layer_stride; }

KvView kv_view(bz_instance* I, int layer) {
    const size_t part = (size_t)I->cfg.kv_tokens * I->sh.Hkv * I->sh.d;     // elements in a K or V part
    act_t* base = reinterpret_cast<act_t*>(I->kv) + (size_t)layer * 2 * part;
    KvView v;
    v.k = base;
    v.v = base + part;
    v.slot_off = reinterpret_cast<const int32_t*>(I->wsp + I->ws.slot_off);
    v.slot_cap = reinterpret_cast<const int32_t*>(I->wsp + I->ws.slot_cap);
    v.Hkv = I->sh.Hkv;
    v.d = I->sh.d;
    return v;
}

BatchView batch_view(const bz_batch* b) {
    BatchView v;
    v.B = b->B;
    v.T = b->T;
    v.q_start = b->d_q_start;
    v.seq_slot = b->d_seq_slot;
    v.kv_before = b->d_kv_before;
    v.token_seq = b->d_token_seq;
    v.prefill_items = b->d_items;
    v.n_prefill_items = b->n_prefill_items;
    v.decode_seqs = b->d_decode;
    v.n_decode = b->n_decode;
    int mx = 0, work = 0;
    for (int s : b->decode_seqs) {
        mx = mx > b->kv_before[s] + 1 ? mx : b->kv_before[s] + 1;
        work += (b->kv_before[s] + 1 + kDecodeChunk - 1) / kDecodeChunk;
    }
    v.decode_chunks = (mx + kDecodeChunk - 1) / kDecodeChunk;
    v.decode_work = b->d_work;
    v.n_decode_work = work;             // the device list was built for these same lengths
    return v;
}

int poll_layer(bz_instance* I, int l) {
    if (I->state[l] == kLoading) {
        hipError_t e = hipEventQuery(I->ev[l]);
        if (e == hipSuccess) I->state[l] = kResident;
        else if (e != hipErrorNotReady) return hip_fail(e, "hipEventQuery");
    }
    return BZ_OK;
}

hipEvent_t take_event(bz_instance* I) {
    if (!I->ev_pool.empty()) {
        hipEvent_t e = I->ev_pool.back();
        I->ev_pool.pop_back();
        return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
}

struct ProfScope {
    bz_instance* I;
    ProfRec rec;
    bool on;
    ProfScope(bz_instance* inst, int cls, double flops, double bytes) : I(inst), on(inst->prof_on) {
        if (!on) return;
        rec.cls = cls;
        rec.flops = flops;
        rec.bytes = bytes;
        rec.e0 = take_event(I);
        rec.e1 = take_event(I);
        if (!rec.e0 || !rec.e1) { on = false; return; }
        (void)hipEventRecord(rec.e0, I->compute);
    }
    ~ProfScope() {
        if (!on) return;
        (void)hipEventRecord(rec.e1, I->compute);
        I->prof.push_back(rec);
    }
};

// Is `p` page-locked host memory the runtime knows (hipHostMalloc, or registered)?  Pageable memory makes
// hipMemcpyAsync stage the bytes through a bounce buffer and block the calling thread: the copies would no
// longer overlap with anything.
bool is_pinned_host(const void* p) {
    hipPointerAttribute_t a;
    memset(&a, 0, sizeof a);
    if (hipPointerGetAttributes(&a, p) != hipSuccess) {
        (void)hipGetLastError();             // ordinary malloc memory: the query itself fails
        return false;
    }
    return a.type == hipMemoryTypeHost;
}

// `after` (optional): an event of another stream that must have completed before the first byte is read
int enqueue_copy(bz_instance* I, int layer, const void* src, size_t n, hipMemcpyKind kind, hipEvent_t after = nullptr) {
    if (!I || !src) return BZ_EINVAL;
    if (layer < 0 || layer >= I->sh.L || n != I->sz.layer_bytes) return BZ_EINVAL;
    if (I->state[layer] != kNone) return BZ_EBUSY;
    if (I->dry) return BZ_ESTATE;
    if (kind == hipMemcpyHostToDevice && !is_pinned_host(src)) return BZ_EINVAL;
    if (!I->clock_started) {
        HIP_TRY(hipEventRecord(I->t0, I->copy));
        I->clock_started = true;
    }
    const size_t chunk = I->cfg.chunk_bytes > 0 ? (size_t)I->cfg.chunk_bytes : ((size_t)32 << 20);
    unsigned char* dst = layer_ptr(I, layer);
    const unsigned char* s = static_cast<const unsigned char*>(src);
    // The blob goes over in the order the layer consumes it, with an event behind each group of
    // tensors, so that the layer's first stages can run while its MLP weights are still arriving.
    // With two ingest streams each group's bytes are cut in two halves, one per copy stream; the streams
    // never wait for each other inside a layer (a stage of the layer waits for both halves of its group),
    // only at its end, where the layer's own event is recorded behind both.
    const bool two = I->ingest_streams == 2;
    const size_t ends[4] = {I->lay.wo, I->lay.wg, I->lay.wd, n};
    auto enqueue = [&]() -> hipError_t {
        hipError_t e = hipSuccess;
        if (after) {
            if ((e = hipStreamWaitEvent(I->copy, after, 0)) != hipSuccess) return e;
            if (two && (e = hipStreamWaitEvent(I->copy2, after, 0)) != hipSuccess) return e;
        }
        size_t start = 0;
        for (int part = 0; part < 4; ++part) {
            const size_t mid = start + ((ends[part] - start) / 2 + 255) / 256 * 256;
            const size_t cut = (two && mid < ends[part]) ? mid : ends[part];
            for (size_t off = start; off < cut;) {
                const size_t m = cut - off < chunk ? cut - off : chunk;
                if ((e = hipMemcpyAsync(dst + off, s + off, m, kind, I->copy)) != hipSuccess) return e;
                off += m;
            }
            for (size_t off = cut; off < ends[part];) {
                const size_t m = ends[part] - off < chunk ? ends[part] - off : chunk;
                if ((e = hipMemcpyAsync(dst + off, s + off, m, kind, I->copy2)) != hipSuccess) return e;
                off += m;
            }
            if (two && (e = hipEventRecord(I->ev_part2[4 * layer + part], I->copy2)) != hipSuccess) return e;
            if (part < 3) {
                if ((e = hipEventRecord(I->ev_part[3 * layer + part], I->copy)) != hipSuccess) return e;
            } else {
                if (two && (e = hipStreamWaitEvent(I->copy, I->ev_part2[4 * layer + part], 0)) != hipSuccess) return e;
                if ((e = hipEventRecord(I->ev[layer], I->copy)) != hipSuccess) return e;
            }
            start = ends[part];
        }
        return hipSuccess;
    };
    const hipError_t e = enqueue();
    if (e != hipSuccess) {
        // some chunks may be on their way: the layer can neither run nor be requested again until
        // bz_unload_layer has waited for the streams
        I->state[layer] = kFailed;
        I->parts_valid[layer] = 0;
        return hip_fail(e, "layer ingest");
    }
    I->parts_valid[layer] = (char)I->ingest_streams;     // 1: group events on the copy stream only; 2: on both streams
    I->state[layer] = kLoading;
    I->stats.bytes_ingested += n;
    I->stats.layers_requested += 1;
    return BZ_OK;
}

}  // namespace

extern "C" {

const char* bz_strerror(int st) {
    switch (st) {
        case BZ_OK: return "ok";
        case BZ_EINVAL: return "invalid argument";
        case BZ_ENOMEM: return "out of memory or arena too small";
        case BZ_EBUSY: return "layer or slot already in use";
        case BZ_ENOTLOADED: return "layer was never requested";
        case BZ_ENOTREADY: return "layer not resident yet";
        case BZ_EHIP: return "HIP runtime error";
        case BZ_ECAPACITY: return "capacity exceeded";
        case BZ_ESTATE: return "call not valid in this state";
        default: return "unknown status";
    }
}

int bz_build_info(void) {
#ifdef BZ_FP32_DEBUG
    return BZ_BUILD_FP32_DEBUG;
#else
    return 0;
#endif
}

const char* bz_last_hip_error(void) { return g_hip_err.c_str(); }

int bz_layer_layout_of(const bz_config* cfg, bz_layer_layout* out) {
    if (!out) return BZ_EINVAL;
    int rc = validate(cfg);
    if (rc) return rc;
    layout_of(cfg, out);
    return BZ_OK;
}

int bz_query_sizes(const bz_config* cfg, bz_sizes* out) {
    if (!out) return BZ_EINVAL;
    int rc = validate(cfg);
    if (rc) return rc;
    bz_layer_layout lay;
    layout_of(cfg, &lay);
    WsLayout ws;
    ws_layout(cfg, &ws);
    out->layer_bytes = lay.total;
    out->layer_stride = align_up(lay.total, 256);
    out->weights_arena_bytes = out->layer_stride * (size_t)cfg->n_layers;
    out->kv_arena_bytes = (size_t)cfg->n_layers * 2 * (size_t)cfg->kv_tokens * cfg->n_kv_heads * cfg->head_dim * sizeof(act_t);
    out->workspace_bytes = ws.total;
    out->act_elem_bytes = sizeof(act_t);
    return BZ_OK;
}

int bz_destroy(bz_instance* I) {
    if (!I) return BZ_EINVAL;
    if (!I->dry) {
        if (I->compute) (void)hipStreamSynchronize(I->compute);
        if (I->copy) (void)hipStreamSynchronize(I->copy);
        if (I->copy2) { (void)hipStreamSynchronize(I->copy2); if (I->own_copy2) (void)hipStreamDestroy(I->copy2); }
        for (hipEvent_t e : I->ev) if (e) (void)hipEventDestroy(e);
        for (hipEvent_t e : I->ev_part) if (e) (void)hipEventDestroy(e);
        for (hipEvent_t e : I->ev_part2) if (e) (void)hipEventDestroy(e);
        for (hipEvent_t e : I->ev_pool) (void)hipEventDestroy(e);
        for (hipStream_t q : I->shard_streams) { (void)hipStreamSynchronize(q); (void)hipStreamDestroy(q); }
        for (hipEvent_t e : I->shard_events) (void)hipEventDestroy(e);
        for (auto& r : I->prof) { (void)hipEventDestroy(r.e0); (void)hipEventDestroy(r.e1); }
        if (I->t0) (void)hipEventDestroy(I->t0);
        if (I->own_weights && I->weights) (void)hipFree(I->weights);
        if (I->order_ev) (void)hipEventDestroy(I->order_ev);
        if (I->own_kv && I->kv) (void)hipFree(I->kv);
        if (I->own_ws && I->wsp) (void)hipFree(I->wsp);
        if (I->own_compute && I->compute) (void)hipStreamDestroy(I->compute);
        if (I->own_copy && I->copy) (void)hipStreamDestroy(I->copy);
    }
    delete I->slots;
    delete I;
    return BZ_OK;
}

int bz_create(const bz_config* cfg, bz_instance** out) try {
    if (!out) return BZ_EINVAL;
    *out = nullptr;
    int rc = validate(cfg);
    if (rc) return rc;
    bz_instance* I = new (std::nothrow) bz_instance();
    if (!I) return BZ_ENOMEM;
    I->cfg = *cfg;
    I->sh = Shape{cfg->n_layers, cfg->hidden, cfg->n_q_heads, cfg->n_kv_heads, cfg->head_dim, cfg->ffn};
    bz_query_sizes(cfg, &I->sz);
    layout_of(cfg, &I->lay);
    ws_layout(cfg, &I->ws);
    I->dry = (cfg->flags & BZ_FLAG_DRY_RUN) != 0;
    I->state.assign(cfg->n_layers, kNone);
    I->parts_valid.assign(cfg->n_layers, 0);
    I->slots = new KvSlots(cfg->max_seqs, cfg->kv_tokens);
    memset(&I->stats, 0, sizeof I->stats);
    if (I->dry) {
        *out = I;
        return BZ_OK;
    }
    auto fail = [&](int code) { bz_destroy(I); return code; };
#define HIP_TRY_C(call)                                                       \
    do {                                                                      \
        hipError_t e__ = (call);                                              \
        if (e__ != hipSuccess) { hip_fail(e__, #call); return fail(BZ_EHIP); } \
    } while (0)
    if (cfg->compute_stream) I->compute = (hipStream_t)cfg->compute_stream;
    else { HIP_TRY_C(hipStreamCreateWithFlags(&I->compute, hipStreamNonBlocking)); I->own_compute = true; }
    if (cfg->copy_stream) I->copy = (hipStream_t)cfg->copy_stream;
    else { HIP_TRY_C(hipStreamCreateWithFlags(&I->copy, hipStreamNonBlocking)); I->own_copy = true; }
    if (cfg->weights_arena) {
        if (cfg->weights_arena_bytes < I->sz.weights_arena_bytes || ((uintptr_t)cfg->weights_arena & 255)) return fail(BZ_ENOMEM);
        I->weights = (unsigned char*)cfg->weights_arena;
    } else { HIP_TRY_C(hipMalloc((void**)&I->weights, I->sz.weights_arena_bytes)); I->own_weights = true; }
    if (cfg->kv_arena) {
        if (cfg->kv_arena_bytes < I->sz.kv_arena_bytes || ((uintptr_t)cfg->kv_arena & 255)) return fail(BZ_ENOMEM);
        I->kv = (unsigned char*)cfg->kv_arena;
    } else { HIP_TRY_C(hipMalloc((void**)&I->kv, I->sz.kv_arena_bytes)); I->own_kv = true; }
    if (cfg->workspace) {
        if (cfg->workspace_bytes < I->sz.workspace_bytes || ((uintptr_t)cfg->workspace & 255)) return fail(BZ_ENOMEM);
        I->wsp = (unsigned char*)cfg->workspace;
    } else { HIP_TRY_C(hipMalloc((void**)&I->wsp, I->sz.workspace_bytes)); I->own_ws = true; }
    I->ev.assign(cfg->n_layers, nullptr);
    for (int l = 0; l < cfg->n_layers; ++l) HIP_TRY_C(hipEventCreate(&I->ev[l]));
    I->ev_part.assign((size_t)3 * cfg->n_layers, nullptr);
    for (size_t k = 0; k < I->ev_part.size(); ++k) HIP_TRY_C(hipEventCreateWithFlags(&I->ev_part[k], hipEventDisableTiming));
    I->ev_part2.assign((size_t)4 * cfg->n_layers, nullptr);
    for (size_t k = 0; k < I->ev_part2.size(); ++k) HIP_TRY_C(hipEventCreateWithFlags(&I->ev_part2[k], hipEventDisableTiming));
    HIP_TRY_C(hipEventCreate(&I->t0));
    {   // rotary table: angle = pos * base^(-2j/d) in float64, stored as (cos, sin) floats
        const int d = cfg->head_dim, half = d / 2;
        std::vector<float> tab((size_t)cfg->max_seq_len * d);
        std::vector<double> theta(half);
        for (int j = 0; j < half; ++j) theta[j] = pow((double)cfg->rope_base, -2.0 * j / d);
        for (int p = 0; p < cfg->max_seq_len; ++p)
            for (int j = 0; j < half; ++j) {
                const double a = (double)p * theta[j];
                tab[((size_t)p * half + j) * 2] = (float)cos(a);
                tab[((size_t)p * half + j) * 2 + 1] = (float)sin(a);
            }
        HIP_TRY_C(hipMemcpy(I->wsp + I->ws.rope, tab.data(), tab.size() * sizeof(float), hipMemcpyHostToDevice));
    }
    // attention multiplies V of masked positions by zero instead of skipping it: the cache must never
    // hold non-finite bit patterns, so it starts out cleared (also when the caller brought the arena)
    HIP_TRY_C(hipMemset(I->kv, 0, I->sz.kv_arena_bytes));
    HIP_TRY_C(hipMemset(I->wsp + I->ws.slot_off, 0, (size_t)cfg->max_seqs * sizeof(int32_t)));
    HIP_TRY_C(hipMemset(I->wsp + I->ws.slot_cap, 0, (size_t)cfg->max_seqs * sizeof(int32_t)));
    HIP_TRY_C(hipDeviceSynchronize());
#undef HIP_TRY_C
    *out = I;
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int bz_sync(bz_instance* I) {
    if (!I) return BZ_EINVAL;
    if (I->dry) return BZ_OK;
    // shard streams feed the copy stream through events, so they need no wait of their own
    HIP_TRY(hipStreamSynchronize(I->copy));
    if (I->copy2) HIP_TRY(hipStreamSynchronize(I->copy2));
    HIP_TRY(hipStreamSynchronize(I->compute));
    return BZ_OK;
}

int bz_set_ingest_streams(bz_instance* I, int n) {
    if (!I || (n != 1 && n != 2)) return BZ_EINVAL;
    // the second stream exists only for instances that ask for it: a process has few hardware queues, and a
    // split pair of instances would otherwise hold eight streams between them
    if (n == 2 && !I->dry && !I->copy2) {
        HIP_TRY(hipStreamCreateWithFlags(&I->copy2, hipStreamNonBlocking));
        I->own_copy2 = true;
    }
    I->ingest_streams = n;
    return BZ_OK;
}

int bz_lend_second_copy_stream(bz_instance* I, void* stream) {
    if (!I || !stream) return BZ_EINVAL;
    if (I->dry) return BZ_ESTATE;
    const hipStream_t st = (hipStream_t)stream;
    if (st == I->copy || st == I->compute) return BZ_EINVAL;
    if (I->copy2 == st) return BZ_OK;
    if (I->copy2) {                     // halves of earlier layers may still travel on the stream being replaced
        HIP_TRY(hipStreamSynchronize(I->copy2));
        if (I->own_copy2) HIP_TRY(hipStreamDestroy(I->copy2));
    }
    I->copy2 = st;
    I->own_copy2 = false;
    return BZ_OK;
}

int bz_load_layer(bz_instance* I, int layer, const void* host, size_t n) {
    return enqueue_copy(I, layer, host, n, hipMemcpyHostToDevice);
}

int bz_load_layer_from_device(bz_instance* I, int layer, const void* dev, size_t n) {
    return enqueue_copy(I, layer, dev, n, hipMemcpyDeviceToDevice);
}

int bz_load_layer_from_peer(bz_instance* I, int layer, bz_instance* peer) {
    if (!I || !peer || I == peer) return BZ_EINVAL;
    if (layer < 0 || layer >= I->sh.L || layer >= peer->sh.L) return BZ_EINVAL;
    if (I->sz.layer_bytes != peer->sz.layer_bytes || I->sh.H != peer->sh.H || I->sh.F != peer->sh.F ||
        I->sh.Hq != peer->sh.Hq || I->sh.Hkv != peer->sh.Hkv || I->sh.d != peer->sh.d)
        return BZ_EINVAL;
    if (I->dry || peer->dry) return BZ_ESTATE;
    if (peer->state[layer] == kNone) return BZ_ENOTLOADED;
    if (peer->state[layer] == kFailed) return BZ_ESTATE;
    // the peer's layer event lies behind all of the layer's bytes, on whichever streams they travelled
    return enqueue_copy(I, layer, layer_ptr(peer, layer), I->sz.layer_bytes, hipMemcpyDeviceToDevice, peer->ev[layer]);
}

int bz_load_layer_sharded(bz_instance* I, int layer, const bz_shard* shards, int n_shards) try {
    if (!I || !shards || n_shards < 1 || n_shards > BZ_MAX_SHARDS) return BZ_EINVAL;
    if (layer < 0 || layer >= I->sh.L) return BZ_EINVAL;
    // the shards must tile [0, layer_bytes) exactly: sort indices by offset, then walk
    int order[BZ_MAX_SHARDS];
    for (int j = 0; j < n_shards; ++j) order[j] = j;
    std::sort(order, order + n_shards, [&](int a, int b) { return shards[a].offset < shards[b].offset; });
    size_t at = 0;
    for (int k = 0; k < n_shards; ++k) {
        const bz_shard& sh = shards[order[k]];
        if (!sh.src || sh.bytes == 0 || sh.offset != at) return BZ_EINVAL;
        at += sh.bytes;
        if (at > I->sz.layer_bytes) return BZ_EINVAL;
    }
    if (at != I->sz.layer_bytes) return BZ_EINVAL;
    if (I->state[layer] != kNone) return BZ_EBUSY;
    if (I->dry) return BZ_ESTATE;
    // Shards alternate over a small fixed set of extra streams: a process has few hardware queues
    // (four here), and a stream beyond them shares a queue with the compute stream, whose kernels
    // then wait behind copies.
    constexpr int kShardStreams = 2;
    const int n_streams = n_shards < kShardStreams ? n_shards : kShardStreams;
    while ((int)I->shard_streams.size() < n_streams) {
        hipStream_t q = nullptr;
        hipEvent_t e = nullptr;
        HIP_TRY(hipStreamCreateWithFlags(&q, hipStreamNonBlocking));
        I->shard_streams.push_back(q);
        HIP_TRY(hipEventCreateWithFlags(&e, hipEventDisableTiming));
        I->shard_events.push_back(e);
    }
    for (int j = 0; j < n_shards; ++j)
        if (!shards[j].src_is_device && !is_pinned_host(shards[j].src)) return BZ_EINVAL;
    if (!I->clock_started) {
        HIP_TRY(hipEventRecord(I->t0, I->copy));
        I->clock_started = true;
    }
    const size_t chunk = I->cfg.chunk_bytes > 0 ? (size_t)I->cfg.chunk_bytes : ((size_t)32 << 20);
    unsigned char* dst = layer_ptr(I, layer);
    auto enqueue = [&]() -> hipError_t {
        hipError_t e = hipSuccess;
        for (int j = 0; j < n_shards; ++j) {
            const bz_shard& sh = shards[j];
            const unsigned char* s = static_cast<const unsigned char*>(sh.src);
            const hipMemcpyKind kind = sh.src_is_device ? hipMemcpyDeviceToDevice : hipMemcpyHostToDevice;
            for (size_t off = 0; off < sh.bytes; off += chunk) {
                const size_t m = sh.bytes - off < chunk ? sh.bytes - off : chunk;
                e = hipMemcpyAsync(dst + sh.offset + off, s + off, m, kind, I->shard_streams[j % n_streams]);
                if (e != hipSuccess) return e;
            }
        }
        for (int q = 0; q < n_streams; ++q) {
            if ((e = hipEventRecord(I->shard_events[q], I->shard_streams[q])) != hipSuccess) return e;
            if ((e = hipStreamWaitEvent(I->copy, I->shard_events[q], 0)) != hipSuccess) return e;
        }
        return hipEventRecord(I->ev[layer], I->copy);        // fires when every shard has landed
    };
    const hipError_t e = enqueue();
    if (e != hipSuccess) {
        I->state[layer] = kFailed;                           // see enqueue_copy
        I->parts_valid[layer] = 0;
        return hip_fail(e, "sharded layer ingest");
    }
    I->parts_valid[layer] = 0;                            // shards land in no particular order
    I->state[layer] = kLoading;
    I->stats.bytes_ingested += I->sz.layer_bytes;
    I->stats.layers_requested += 1;
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int bz_unload_layer(bz_instance* I, int layer) {
    if (!I || layer < 0 || layer >= I->sh.L) return BZ_EINVAL;
    int rc = I->dry ? BZ_OK : bz_sync(I);
    if (rc) return rc;
    if (I->state[layer] == kFailed)                    // a load that broke off may have left shards in flight that
        for (hipStream_t q : I->shard_streams) HIP_TRY(hipStreamSynchronize(q));      // nothing on the copy stream waits for
    I->state[layer] = kNone;
    I->parts_valid[layer] = 0;
    return BZ_OK;
}

int bz_frontier(bz_instance* I) {
    if (!I) return BZ_EINVAL;
    int k = 0;
    for (; k < I->sh.L; ++k) {
        if (I->state[k] == kNone) break;
        if (!I->dry) {
            int rc = poll_layer(I, k);
            if (rc) return rc;
        }
        if (I->state[k] != kResident) break;
    }
    return k;
}

int bz_layer_ready(bz_instance* I, int layer) {
    if (!I || layer < 0 || layer >= I->sh.L) return BZ_EINVAL;
    if (I->state[layer] == kNone) return 0;
    if (!I->dry) {
        int rc = poll_layer(I, layer);
        if (rc) return rc;
    }
    return I->state[layer] == kResident ? 1 : 0;
}

int bz_wait_layer(bz_instance* I, int layer) {
    if (!I || layer < 0 || layer >= I->sh.L) return BZ_EINVAL;
    if (I->state[layer] == kNone) return BZ_ENOTLOADED;
    if (I->dry || I->state[layer] == kFailed) return BZ_ESTATE;
    HIP_TRY(hipEventSynchronize(I->ev[layer]));
    I->state[layer] = kResident;
    return BZ_OK;
}

int bz_layer_ready_ms(bz_instance* I, int layer, float* ms) {
    if (!I || !ms || layer < 0 || layer >= I->sh.L) return BZ_EINVAL;
    if (I->dry || !I->clock_started) return BZ_ESTATE;
    int r = bz_layer_ready(I, layer);
    if (r < 0) return r;
    if (r == 0) return BZ_ENOTREADY;
    HIP_TRY(hipEventElapsedTime(ms, I->t0, I->ev[layer]));
    return BZ_OK;
}

int bz_reset_clock(bz_instance* I) {
    if (!I) return BZ_EINVAL;
    I->clock_started = false;
    return BZ_OK;
}

int bz_readback_layer(bz_instance* I, int layer, void* host) {
    if (!I || !host || layer < 0 || layer >= I->sh.L) return BZ_EINVAL;
    if (I->state[layer] == kNone) return BZ_ENOTLOADED;
    if (I->dry) return BZ_ESTATE;
    int rc = bz_wait_layer(I, layer);
    if (rc) return rc;
    HIP_TRY(hipMemcpy(host, layer_ptr(I, layer), I->sz.layer_bytes, hipMemcpyDeviceToHost));
    return BZ_OK;
}

// ---- KV slots -----------------------------------------------------------------------------

static int push_slot(bz_instance* I, int slot) {
    if (I->dry) return BZ_OK;
    const int32_t off = I->slots->reserved(slot) ? (int32_t)I->slots->offset(slot) : 0;
    const int32_t cap = I->slots->reserved(slot) ? (int32_t)I->slots->capacity(slot) : 0;
    // in stream order on the compute stream, where every kernel that reads the table runs
    launch_set_slot(reinterpret_cast<int32_t*>(I->wsp + I->ws.slot_off) + slot,
                    reinterpret_cast<int32_t*>(I->wsp + I->ws.slot_cap) + slot, off, cap, I->compute);
    HIP_TRY(hipGetLastError());
    return BZ_OK;
}

int bz_kv_reserve(bz_instance* I, int slot, int capacity_tokens) try {
    if (!I || slot < 0 || slot >= I->cfg.max_seqs || capacity_tokens < 1) return BZ_EINVAL;
    if (capacity_tokens > I->cfg.max_seq_len) return BZ_ECAPACITY;
    if (I->slots->reserved(slot)) return BZ_EBUSY;
    // the K cache is stored in blocks of 32 positions
    if (!I->slots->reserve(slot, ((int64_t)capacity_tokens + 31) / 32 * 32)) return BZ_ECAPACITY;
    return push_slot(I, slot);
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int bz_kv_release(bz_instance* I, int slot) try {
    if (!I || slot < 0 || slot >= I->cfg.max_seqs) return BZ_EINVAL;
    if (!I->slots->reserved(slot)) return BZ_ESTATE;
    if (!I->dry) {
        int rc = bz_sync(I);      // no kernel may still be reading the slot
        if (rc) return rc;
    }
    I->slots->release(slot);
    return push_slot(I, slot);
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int64_t bz_kv_free_tokens(bz_instance* I) {
    if (!I) return BZ_EINVAL;
    return I->slots->largest_free() / 32 * 32;
}

static int kv_xfer(bz_instance* I, int layer, int slot, int pos0, int n, const void* k, const void* v, void* ko,
                   void* vo, int is_host, bool to_cache) {
    if (!I || layer < 0 || layer >= I->sh.L || slot < 0 || slot >= I->cfg.max_seqs || pos0 < 0 || n < 0) return BZ_EINVAL;
    if (to_cache ? (!k || !v) : (!ko || !vo)) return BZ_EINVAL;
    if (!I->slots->reserved(slot)) return BZ_ESTATE;
    if ((int64_t)pos0 + n > I->slots->capacity(slot) || (int64_t)pos0 + n > I->cfg.max_seq_len) return BZ_ECAPACITY;
    if (I->dry) return BZ_ESTATE;
    if (n == 0) return BZ_OK;
    const KvView view = kv_view(I, layer);
    if (!is_host) {
        launch_kv_scatter((const act_t*)k, (const act_t*)v, view, slot, pos0, n, to_cache, (act_t*)ko, (act_t*)vo, I->compute);
        HIP_TRY(hipGetLastError());
        return BZ_OK;
    }
    // Host side: staged through the activation buffers of the workspace (free between bz_run_layers calls, and
    // every use here is in stream order on the compute stream), as many positions at a time as fit.
    unsigned char* stage = I->wsp + I->ws.normed;
    const size_t span = I->ws.partial - I->ws.normed;
    const size_t per_tok = (size_t)I->sh.Hkv * I->sh.d * sizeof(act_t);
    const int step = (int)std::min<size_t>((size_t)n, span / (2 * per_tok));
    if (step < 1) return BZ_ECAPACITY;
    hipError_t e = hipSuccess;
    for (int at = 0; at < n && e == hipSuccess; at += step) {
        const int m = n - at < step ? n - at : step;
        const size_t mb = (size_t)m * per_tok;
        act_t* sk = reinterpret_cast<act_t*>(stage);
        act_t* sv = reinterpret_cast<act_t*>(stage + (size_t)step * per_tok);
        if (to_cache) {
            e = hipMemcpyAsync(sk, static_cast<const unsigned char*>(k) + (size_t)at * per_tok, mb, hipMemcpyHostToDevice, I->compute);
            if (e == hipSuccess)
                e = hipMemcpyAsync(sv, static_cast<const unsigned char*>(v) + (size_t)at * per_tok, mb, hipMemcpyHostToDevice, I->compute);
            if (e == hipSuccess) {
                launch_kv_scatter(sk, sv, view, slot, pos0 + at, m, true, nullptr, nullptr, I->compute);
                e = hipGetLastError();
            }
        } else {
            launch_kv_scatter(nullptr, nullptr, view, slot, pos0 + at, m, false, sk, sv, I->compute);
            e = hipGetLastError();
            if (e == hipSuccess)
                e = hipMemcpyAsync(static_cast<unsigned char*>(ko) + (size_t)at * per_tok, sk, mb, hipMemcpyDeviceToHost, I->compute);
            if (e == hipSuccess)
                e = hipMemcpyAsync(static_cast<unsigned char*>(vo) + (size_t)at * per_tok, sv, mb, hipMemcpyDeviceToHost, I->compute);
        }
    }
    if (e == hipSuccess) e = hipStreamSynchronize(I->compute);
    if (e != hipSuccess) return hip_fail(e, "kv transfer");
    return BZ_OK;
}

int bz_kv_write(bz_instance* I, int layer, int slot, int pos0, int n, const void* k, const void* v, int is_host) {
    return kv_xfer(I, layer, slot, pos0, n, k, v, nullptr, nullptr, is_host, true);
}

int bz_kv_read(bz_instance* I, int layer, int slot, int pos0, int n, void* k, void* v, int is_host) {
    return kv_xfer(I, layer, slot, pos0, n, nullptr, nullptr, k, v, is_host, false);
}

// ---- batches ------------------------------------------------------------------------------

namespace {

constexpr int kWorkGrowth = 64;          // chunks per decode sequence the work list can grow by before a rebuild

size_t align32(size_t v) { return (v + 31) / 32 * 32; }

// Fills the host side of `b` from a validated description and lays the device image out in `image`
// (32-bit words; the decode work list starts at byte *work_at).  `max_bytes` (0: no limit) bounds the
// image: the work list's room for growth shrinks to what fits, and BZ_ECAPACITY is returned if even the
// present entries do not.
int describe_batch(const bz_batch_desc* d, bz_batch* b, std::vector<int32_t>& image, size_t max_bytes) {
    size_t* work_at = &b->work_at;
    if (!d || d->n_seqs < 1 || !d->q_start || !d->seq_slot || !d->kv_len_before) return BZ_EINVAL;
    const int B = d->n_seqs;
    if (d->q_start[0] != 0) return BZ_EINVAL;
    for (int s = 0; s < B; ++s)
        if (d->q_start[s + 1] < d->q_start[s] || d->kv_len_before[s] < 0 || d->seq_slot[s] < 0) return BZ_EINVAL;
    {   // every sequence in a slot of its own
        std::vector<int32_t> sorted(d->seq_slot, d->seq_slot + B);
        std::sort(sorted.begin(), sorted.end());
        if (std::adjacent_find(sorted.begin(), sorted.end()) != sorted.end()) return BZ_EINVAL;
    }
    const int T = d->q_start[B];
    if (T < 1) return BZ_EINVAL;
    b->B = B;
    b->T = T;
    b->q_start.assign(d->q_start, d->q_start + B + 1);
    b->seq_slot.assign(d->seq_slot, d->seq_slot + B);
    b->kv_before.assign(d->kv_len_before, d->kv_len_before + B);
    b->decode_seqs.clear();
    b->prefill_sq = 0;
    std::vector<int32_t> token_seq(T), items;
    b->all_decode = true;
    struct Item { int s, qt; long long extent; };
    std::vector<Item> its;
    for (int s = 0; s < B; ++s) {
        const int qlen = b->q_start[s + 1] - b->q_start[s];
        for (int t = b->q_start[s]; t < b->q_start[s + 1]; ++t) token_seq[t] = s;
        if (qlen == 1) b->decode_seqs.push_back(s);
        if (qlen != 1) b->all_decode = false;
        if (qlen > 1) {
            const int tiles = (qlen + kPrefillTileQ - 1) / kPrefillTileQ;
            for (int qt = 0; qt < tiles; ++qt) {
                const int last = (qt * kPrefillTileQ + kPrefillTileQ < qlen ? qt * kPrefillTileQ + kPrefillTileQ : qlen);
                its.push_back({s, qt, (long long)b->kv_before[s] + last});
            }
            b->prefill_sq += (double)qlen * b->kv_before[s] + 0.5 * (double)qlen * (qlen + 1);
        }
    }
    // longest key range first, so the tail of the grid is made of short tiles
    std::stable_sort(its.begin(), its.end(), [](const Item& a, const Item& c) { return a.extent > c.extent; });
    for (const Item& it : its) { items.push_back(it.s); items.push_back(it.qt); }
    b->n_prefill_items = (int)its.size();
    b->n_decode = (int)b->decode_seqs.size();

    // decode work list: one entry per chunk of every decode sequence's cache (the new token included), with
    // room for kWorkGrowth more chunks per sequence as bz_batch_advance lengthens the caches.  The room is
    // zero-filled, so that a kernel that ran ahead of an update would read a harmless entry, never garbage.
    std::vector<int32_t> work;
    for (int di = 0; di < b->n_decode; ++di) {
        const int s = b->decode_seqs[di];
        const int n = (b->kv_before[s] + 1 + kDecodeChunk - 1) / kDecodeChunk;
        const int first = (int)(work.size() / 8);
        for (int c = 0; c < n; ++c) {
            const int32_t entry[8] = {s, b->seq_slot[s], di, n, first, 0, 0, 0};
            work.insert(work.end(), entry, entry + 8);
        }
    }
    const size_t n_i32 = (size_t)(B + 1) + B + B + T + items.size() + b->decode_seqs.size();
    *work_at = align32(n_i32 * 4);
    const size_t present = work.size() / 8;
    size_t capacity = present + (size_t)kWorkGrowth * b->n_decode;
    if (max_bytes) {
        if (*work_at + present * 32 + 64 > max_bytes) return BZ_ECAPACITY;
        const size_t fits = (max_bytes - *work_at - 64) / 32;
        if (capacity > fits) capacity = fits;
    }
    b->work_capacity = (int)capacity;
    image.clear();
    image.reserve((*work_at + capacity * 32 + 64) / 4);
    auto put = [&](const std::vector<int32_t>& v) { const size_t at = image.size(); image.insert(image.end(), v.begin(), v.end()); return at; };
    b->off_words[0] = put(b->q_start);
    b->off_words[1] = put(b->seq_slot);
    b->off_words[2] = put(b->kv_before);
    b->off_words[3] = put(token_seq);
    b->off_words[4] = put(items);
    b->off_words[5] = put(b->decode_seqs);
    image.resize(*work_at / 4, 0);
    image.insert(image.end(), work.begin(), work.end());
    image.resize((*work_at + capacity * 32 + 64) / 4, 0);
    return BZ_OK;
}

// Device addresses of the arrays, once b->dev is known.
void bind_batch(bz_batch* b) {
    int32_t* base = static_cast<int32_t*>(b->dev);
    b->d_q_start = base + b->off_words[0];
    b->d_seq_slot = base + b->off_words[1];
    b->d_kv_before = base + b->off_words[2];
    b->d_token_seq = base + b->off_words[3];
    b->d_items = base + b->off_words[4];
    b->d_decode = base + b->off_words[5];
    b->d_work = reinterpret_cast<int4*>(static_cast<unsigned char*>(b->dev) + b->work_at);
}

// Orders stream `st` behind every run of the batch that was enqueued on another stream.
int wait_for_runs_elsewhere(const bz_batch* b, hipStream_t st) {
    for (const bz_batch::Use& u : b->runs)
        if (u.st != st) HIP_TRY(hipStreamWaitEvent(st, u.ev, 0));
    return BZ_OK;
}

int mark_changed(bz_batch* b, hipStream_t st) {
    if (!b->changed_ev) HIP_TRY(hipEventCreateWithFlags(&b->changed_ev, hipEventDisableTiming));
    HIP_TRY(hipEventRecord(b->changed_ev, st));
    b->changed_on = st;
    b->changed_valid = true;
    return BZ_OK;
}

}  // namespace

int bz_batch_destroy(bz_batch* b) {
    if (!b) return BZ_EINVAL;
    // an upload still reading the caller's staging, or a kernel still reading the device arrays, must not outlive them
    for (int h = 0; h < 2; ++h) {
        if (b->staged_valid[h]) (void)hipEventSynchronize(b->staged_ev[h]);
        if (b->staged_ev[h]) (void)hipEventDestroy(b->staged_ev[h]);
    }
    if (b->changed_valid) (void)hipEventSynchronize(b->changed_ev);
    for (const bz_batch::Use& u : b->runs) { (void)hipEventSynchronize(u.ev); (void)hipEventDestroy(u.ev); }
    if (b->changed_ev) (void)hipEventDestroy(b->changed_ev);
    if (b->own_dev && b->dev) (void)hipFree(b->dev);
    delete b;
    return BZ_OK;
}

int bz_batch_create(const bz_batch_desc* d, bz_batch** out) try {
    if (!out) return BZ_EINVAL;
    *out = nullptr;
    bz_batch* b = new (std::nothrow) bz_batch();
    if (!b) return BZ_ENOMEM;
    std::vector<int32_t> image;
    const int rc = describe_batch(d, b, image, 0);
    if (rc) { delete b; return rc; }
    hipError_t e = hipMalloc(&b->dev, image.size() * 4);
    if (e != hipSuccess) { hip_fail(e, "hipMalloc(batch)"); delete b; return BZ_EHIP; }
    b->own_dev = true;
    b->dev_bytes = image.size() * 4;
    bind_batch(b);
    e = hipMemcpy(b->dev, image.data(), image.size() * 4, hipMemcpyHostToDevice);
    if (e != hipSuccess) { hip_fail(e, "hipMemcpy(batch)"); bz_batch_destroy(b); return BZ_EHIP; }
    *out = b;
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

size_t bz_batch_storage_bytes(int max_seqs, int max_tokens, int max_seq_len) {
    if (max_seqs < 1 || max_tokens < 1 || max_seq_len < 1) return 0;
    const size_t B = (size_t)max_seqs, T = (size_t)max_tokens;
    const size_t items = 2 * (T / kPrefillTileQ + B);                        // (sequence, query tile) pairs
    const size_t words = (B + 1) + B + B + T + items + B;
    const size_t chunks = ((size_t)max_seq_len + kDecodeChunk) / kDecodeChunk;  // of a cache of max_seq_len positions
    return align32(words * 4) + B * (chunks + kWorkGrowth) * 32 + 64;
}

static int build_in_place(bz_batch* b, const bz_batch_desc* d, hipStream_t st) {
    const int h = b->staging_next;
    // the upload that last used this half of the staging (two builds ago) must have left it ...
    if (b->staged_valid[h]) HIP_TRY(hipEventSynchronize(b->staged_ev[h]));
    // ... and runs enqueued on other streams must have read the device arrays before the new ones land
    int rc = wait_for_runs_elsewhere(b, st);
    if (rc) return rc;
    if (b->changed_valid && b->changed_on != st) HIP_TRY(hipStreamWaitEvent(st, b->changed_ev, 0));
    std::vector<int32_t> image;
    rc = describe_batch(d, b, image, b->dev_bytes);
    if (rc) return rc;
    bind_batch(b);
    unsigned char* half = static_cast<unsigned char*>(b->staging) + (size_t)h * b->dev_bytes;
    memcpy(half, image.data(), image.size() * 4);
    HIP_TRY(hipMemcpyAsync(b->dev, half, image.size() * 4, hipMemcpyHostToDevice, st));
    if (!b->staged_ev[h]) HIP_TRY(hipEventCreateWithFlags(&b->staged_ev[h], hipEventDisableTiming));
    HIP_TRY(hipEventRecord(b->staged_ev[h], st));
    b->staged_valid[h] = true;
    b->staging_next = h ^ 1;
    return mark_changed(b, st);
}

int bz_batch_create_in(const bz_batch_desc* d, void* device_mem, size_t device_bytes, void* pinned_mem, size_t pinned_bytes,
                       void* stream, bz_batch** out) try {
    if (!out) return BZ_EINVAL;
    *out = nullptr;
    if (!device_mem || !pinned_mem || ((uintptr_t)device_mem & 31) || ((uintptr_t)pinned_mem & 3)) return BZ_EINVAL;
    if (device_bytes < 128 || pinned_bytes < 2 * device_bytes) return BZ_EINVAL;
    if (!d || d->n_seqs < 1) return BZ_EINVAL;
    if (!is_pinned_host(pinned_mem)) return BZ_EINVAL;
    bz_batch* b = new (std::nothrow) bz_batch();
    if (!b) return BZ_ENOMEM;
    b->dev = device_mem;
    b->dev_bytes = device_bytes;
    b->staging = pinned_mem;
    const int rc = build_in_place(b, d, (hipStream_t)stream);
    if (rc) { bz_batch_destroy(b); return rc; }
    *out = b;
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int bz_batch_rebuild(bz_batch* b, const bz_batch_desc* d, void* stream) try {
    if (!b || !d) return BZ_EINVAL;
    if (!b->staging) return BZ_ESTATE;                 // only batches that live in caller memory can be rebuilt
    {   // validate first: a refused description must leave the batch as it was
        bz_batch probe;
        std::vector<int32_t> image;
        const int rc = describe_batch(d, &probe, image, b->dev_bytes);
        if (rc) return rc;
    }
    return build_in_place(b, d, (hipStream_t)stream);
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int bz_batch_tokens(const bz_batch* b) { return b ? b->T : BZ_EINVAL; }

int bz_batch_advance(bz_instance* I, bz_batch* b) {
    if (!I || !b) return BZ_EINVAL;
    if (!b->all_decode) return BZ_ESTATE;
    if (I->dry) return BZ_ESTATE;
    long long work = 0;                  // entries of the work list after this step
    for (int s : b->decode_seqs) work += (b->kv_before[s] + 2 + kDecodeChunk - 1) / kDecodeChunk;
    if (work > b->work_capacity) return BZ_ECAPACITY;
    // runs of this batch enqueued on another instance's stream still read the lengths and the work list
    int rc = wait_for_runs_elsewhere(b, I->compute);
    if (rc) return rc;
    if (b->changed_valid && b->changed_on != I->compute) HIP_TRY(hipStreamWaitEvent(I->compute, b->changed_ev, 0));
    launch_batch_advance(b->d_kv_before, b->B, b->d_decode, b->d_seq_slot, b->n_decode, b->d_work, b->work_capacity,
                         I->compute);
    HIP_TRY(hipGetLastError());
    rc = mark_changed(b, I->compute);
    if (rc) return rc;
    for (auto& v : b->kv_before) v += 1;
    return BZ_OK;
}

// ---- execution ----------------------------------------------------------------------------

int bz_run_layers(bz_instance* I, int a, int b, const bz_batch* batch, void* hidden, int flags) try {
    if (!I || !batch || !hidden) return BZ_EINVAL;
    if (a < 0 || b > I->sh.L || a > b) return BZ_EINVAL;
    if (batch->T > I->cfg.max_tokens) return BZ_ECAPACITY;
    for (int s = 0; s < batch->B; ++s) {
        const int slot = batch->seq_slot[s];
        if (slot >= I->cfg.max_seqs) return BZ_EINVAL;
        if (!I->slots->reserved(slot)) return BZ_ESTATE;
        const int qlen = batch->q_start[s + 1] - batch->q_start[s];
        if ((int64_t)batch->kv_before[s] + qlen > I->slots->capacity(slot)) return BZ_ECAPACITY;
        if ((int64_t)batch->kv_before[s] + qlen > I->cfg.max_seq_len) return BZ_ECAPACITY;
    }
    for (int l = a; l < b; ++l) {
        if (I->state[l] == kNone) return BZ_ENOTLOADED;
        if (I->state[l] == kFailed) return BZ_ESTATE;
    }
    if (I->dry) return BZ_ESTATE;
    if (flags & BZ_RUN_NOWAIT) {
        for (int l = a; l < b; ++l) {
            int rc = poll_layer(I, l);
            if (rc) return rc;
            if (I->state[l] != kResident) return BZ_ENOTREADY;
        }
    }
    const Shape& sh = I->sh;
    const int T = batch->T;
    // the batch's device arrays may have been uploaded, or advanced, on another instance's stream
    if (batch->changed_valid && batch->changed_on != I->compute) HIP_TRY(hipStreamWaitEvent(I->compute, batch->changed_ev, 0));
    const BatchView bv = batch_view(batch);
    act_t* x = static_cast<act_t*>(hidden);
    act_t* normed = reinterpret_cast<act_t*>(I->wsp + I->ws.normed);
    act_t* qkv = reinterpret_cast<act_t*>(I->wsp + I->ws.qkv);
    act_t* attn = reinterpret_cast<act_t*>(I->wsp + I->ws.attn);
    act_t* act = reinterpret_cast<act_t*>(I->wsp + I->ws.act);
    float* partial = reinterpret_cast<float*>(I->wsp + I->ws.partial);
    float* gws = reinterpret_cast<float*>(I->wsp + I->ws.gemm_ws);
    const size_t gwsb = I->ws.gemm_ws_bytes;
    const float* rope = reinterpret_cast<const float*>(I->wsp + I->ws.rope);
    hipStream_t st = I->compute;
    const double e = sizeof(act_t);
    double decode_kv = 0;
    for (int s : batch->decode_seqs) decode_kv += (double)(batch->kv_before[s] + 1);

    int pending_down = 0;        // split-K slices of the previous layer's down projection still to be folded into x
    for (int l = a; l < b; ++l) {
        // A layer still on its way is waited for as a whole, except the last one of the range: there each
        // stage waits only for the tensors it reads, so the range ends one down projection, not one whole
        // layer, behind the last byte.  (Finer gating of the layers before it would not end the range any
        // sooner, and every wait on another stream's event costs the compute stream some tens of
        // microseconds.)
        if (I->state[l] == kLoading) {                   // may have landed since it was last looked at: then no wait at all
            int rc = poll_layer(I, l);
            if (rc) return rc;
        }
        const bool gated = I->state[l] != kResident;
        const bool by_part = gated && I->parts_valid[l] && l == b - 1;
        if (gated) HIP_TRY(hipStreamWaitEvent(st, by_part ? I->ev_part[3 * l] : I->ev[l], 0));
        const bool two = by_part && I->parts_valid[l] == 2;
        if (two) HIP_TRY(hipStreamWaitEvent(st, I->ev_part2[4 * l], 0));
        const unsigned char* wl = layer_ptr(I, l);
        const bf16* g1 = (const bf16*)(wl + I->lay.g1);
        const bf16* wqkv = (const bf16*)(wl + I->lay.wq);
        const bf16* wo = (const bf16*)(wl + I->lay.wo);
        const bf16* g2 = (const bf16*)(wl + I->lay.g2);
        const bf16* wgu = (const bf16*)(wl + I->lay.wg);
        const bf16* wd = (const bf16*)(wl + I->lay.wd);
        const KvView kvv = kv_view(I, l);
        const int nqkv = sh.nqkv(), qd = sh.Hq * sh.d;
        // Decode-sized batches: the projections leave split-K partial sums in `gws` and the kernel that
        // consumes the projection folds them (QKV -> rotary/append; O and down -> residual + next norm).
        // The stored values are the same bits the unfused kernels produce.
        { ProfScope p(I, BZ_K_RMSNORM, 4.0 * T * sh.H, 2.0 * T * sh.H * e);
          if (pending_down > 0) launch_reduce_residual_rmsnorm(x, gws, pending_down, g1, normed, T, sh.H, I->cfg.rms_eps, st);
          else launch_rmsnorm(x, g1, normed, T, sh.H, I->cfg.rms_eps, st);
          pending_down = 0; }
        int ks_qkv = 0;
        { ProfScope p(I, BZ_K_GEMM_QKV, 2.0 * T * nqkv * sh.H, ((double)T * sh.H + (double)T * nqkv) * e + 2.0 * nqkv * sh.H);
          ks_qkv = launch_gemm_partial(0, normed, wqkv, T, nqkv, sh.H, gws, gwsb, st);
          if (ks_qkv == 0) launch_gemm(0, normed, wqkv, nullptr, qkv, T, nqkv, sh.H, gws, gwsb, st); }
        { ProfScope p(I, BZ_K_ROPE_APPEND, 3.0 * T * (sh.Hq + sh.Hkv) * sh.d, (double)T * (2.0 * sh.Hq + 4.0 * sh.Hkv) * sh.d * e);
          if (ks_qkv > 0) launch_rope_append_reduce(qkv, gws, ks_qkv, rope, bv, kvv, sh.Hq, st);
          else launch_rope_append(qkv, rope, bv, kvv, sh.Hq, st); }
        if (bv.n_prefill_items > 0) {
            ProfScope p(I, BZ_K_ATTN_PREFILL, 4.0 * sh.Hq * sh.d * batch->prefill_sq, 0.0);
            launch_attn_prefill(qkv, attn, bv, kvv, sh.Hq, st);
        }
        if (bv.n_decode > 0) {
            ProfScope p(I, BZ_K_ATTN_DECODE, 4.0 * sh.Hq * sh.d * decode_kv, decode_kv * 2.0 * sh.Hkv * sh.d * e);
            launch_attn_decode(qkv, attn, partial, bv, kvv, sh.Hq, st);
        }
        int ks_o = 0;
        if (by_part) {
            HIP_TRY(hipStreamWaitEvent(st, I->ev_part[3 * l + 1], 0));
            if (two) HIP_TRY(hipStreamWaitEvent(st, I->ev_part2[4 * l + 1], 0));
        }
        { ProfScope p(I, BZ_K_GEMM_O, 2.0 * T * sh.H * qd, (2.0 * T * sh.H + (double)T * qd) * e + 2.0 * sh.H * qd);
          ks_o = launch_gemm_partial(1, attn, wo, T, sh.H, qd, gws, gwsb, st);
          if (ks_o == 0) launch_gemm(1, attn, wo, x, x, T, sh.H, qd, gws, gwsb, st); }
        { ProfScope p(I, BZ_K_RMSNORM, 4.0 * T * sh.H, 2.0 * T * sh.H * e);
          if (ks_o > 0) launch_reduce_residual_rmsnorm(x, gws, ks_o, g2, normed, T, sh.H, I->cfg.rms_eps, st);
          else launch_rmsnorm(x, g2, normed, T, sh.H, I->cfg.rms_eps, st); }
        if (by_part) {
            HIP_TRY(hipStreamWaitEvent(st, I->ev_part[3 * l + 2], 0));
            if (two) HIP_TRY(hipStreamWaitEvent(st, I->ev_part2[4 * l + 2], 0));
        }
        { ProfScope p(I, BZ_K_GEMM_GATEUP, 4.0 * T * sh.F * sh.H, ((double)T * sh.H + (double)T * sh.F) * e + 4.0 * sh.F * sh.H);
          launch_gemm(2, normed, wgu, nullptr, act, T, sh.F, sh.H, gws, gwsb, st); }
        if (by_part) HIP_TRY(hipStreamWaitEvent(st, I->ev[l], 0));
        { ProfScope p(I, BZ_K_GEMM_DOWN, 2.0 * T * sh.H * sh.F, (2.0 * T * sh.H + (double)T * sh.F) * e + 2.0 * sh.H * sh.F);
          pending_down = launch_gemm_partial(1, act, wd, T, sh.H, sh.F, gws, gwsb, st);
          if (pending_down == 0) launch_gemm(1, act, wd, x, x, T, sh.H, sh.F, gws, gwsb, st); }
        HIP_TRY(hipGetLastError());
    }
    if (pending_down > 0) {      // last layer of the range: finish the residual stream without a norm
        ProfScope p(I, BZ_K_RMSNORM, 1.0 * T * sh.H, 2.0 * T * sh.H * e);
        launch_reduce_residual_rmsnorm(x, gws, pending_down, nullptr, normed, T, sh.H, I->cfg.rms_eps, st);
        HIP_TRY(hipGetLastError());
    }
    if (batch->all_decode || batch->staging) {
        // this batch can change on the device later (advance, rebuild), possibly on another stream: leave a
        // marker behind the kernels that read it (one event per stream that ever ran it, re-recorded)
        bz_batch::Use* use = nullptr;
        for (bz_batch::Use& u : batch->runs)
            if (u.st == st) use = &u;
        if (!use) {
            hipEvent_t ev = nullptr;
            HIP_TRY(hipEventCreateWithFlags(&ev, hipEventDisableTiming));
            batch->runs.push_back(bz_batch::Use{st, ev});
            use = &batch->runs.back();
        }
        HIP_TRY(hipEventRecord(use->ev, st));
    }
    I->stats.tokens_run += (uint64_t)T * (uint64_t)(b - a);
    I->stats.layer_launches += (uint64_t)(b - a);
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int bz_export_boundary(bz_instance* I, const void* hidden, size_t T, void* buf, int is_host) {
    if (!I || !hidden || !buf) return BZ_EINVAL;
    if (T > (size_t)I->cfg.max_tokens) return BZ_ECAPACITY;
    if (I->dry) return BZ_ESTATE;
    const size_t bytes = T * I->sh.H * sizeof(act_t);
    if (bytes == 0) return BZ_OK;
    HIP_TRY(hipMemcpyAsync(buf, hidden, bytes, is_host ? hipMemcpyDeviceToHost : hipMemcpyDeviceToDevice, I->compute));
    if (is_host) HIP_TRY(hipStreamSynchronize(I->compute));
    return BZ_OK;
}

int bz_import_boundary(bz_instance* I, void* hidden, size_t T, const void* buf, int is_host) {
    if (!I || !hidden || !buf) return BZ_EINVAL;
    if (T > (size_t)I->cfg.max_tokens) return BZ_ECAPACITY;
    if (I->dry) return BZ_ESTATE;
    const size_t bytes = T * I->sh.H * sizeof(act_t);
    if (bytes == 0) return BZ_OK;
    HIP_TRY(hipMemcpyAsync(hidden, buf, bytes, is_host ? hipMemcpyHostToDevice : hipMemcpyDeviceToDevice, I->compute));
    if (is_host) HIP_TRY(hipStreamSynchronize(I->compute));
    return BZ_OK;
}

int bz_wait_stream(bz_instance* I, void* stream) {
    if (!I) return BZ_EINVAL;
    if (I->dry) return BZ_ESTATE;
    if ((hipStream_t)stream == I->compute) return BZ_OK;
    if (!I->order_ev) HIP_TRY(hipEventCreateWithFlags(&I->order_ev, hipEventDisableTiming));
    HIP_TRY(hipEventRecord(I->order_ev, (hipStream_t)stream));
    HIP_TRY(hipStreamWaitEvent(I->compute, I->order_ev, 0));
    return BZ_OK;
}

int bz_signal_stream(bz_instance* I, void* stream) {
    if (!I) return BZ_EINVAL;
    if (I->dry) return BZ_ESTATE;
    if ((hipStream_t)stream == I->compute) return BZ_OK;
    if (!I->order_ev) HIP_TRY(hipEventCreateWithFlags(&I->order_ev, hipEventDisableTiming));
    HIP_TRY(hipEventRecord(I->order_ev, I->compute));
    HIP_TRY(hipStreamWaitEvent((hipStream_t)stream, I->order_ev, 0));
    return BZ_OK;
}

// ---- counters -----------------------------------------------------------------------------

int bz_stats_read(bz_instance* I, bz_stats* out) {
    if (!I || !out) return BZ_EINVAL;
    I->stats.frontier = bz_frontier(I);
    *out = I->stats;
    return BZ_OK;
}

int bz_profile_enable(bz_instance* I, int on) try {
    if (!I) return BZ_EINVAL;
    if (I->dry) return BZ_ESTATE;
    I->prof_on = on != 0;
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int bz_profile_read(bz_instance* I, bz_profile* out) try {
    if (!I || !out) return BZ_EINVAL;
    if (I->dry) return BZ_ESTATE;
    memset(out, 0, sizeof *out);
    HIP_TRY(hipStreamSynchronize(I->compute));
    for (auto& r : I->prof) {
        float ms = 0.f;
        HIP_TRY(hipEventElapsedTime(&ms, r.e0, r.e1));
        out->launches[r.cls] += 1;
        out->ms[r.cls] += ms;
        out->flops[r.cls] += r.flops;
        out->bytes[r.cls] += r.bytes;
        I->ev_pool.push_back(r.e0);
        I->ev_pool.push_back(r.e1);
    }
    I->prof.clear();
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

// ---- single operations -----------------------------------------------------------------------

int bz_op_rmsnorm(const void* x, const void* gain, void* y, int T, int H, float eps, void* stream) {
    if (!x || !gain || !y || T < 0 || H < 8 || H % 8) return BZ_EINVAL;
    launch_rmsnorm((const act_t*)x, (const bf16*)gain, (act_t*)y, T, H, eps, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return BZ_OK;
}

size_t bz_op_gemm_workspace_bytes(int mode, int M, int N, int K) {
    if (mode < 0 || mode > 2 || M < 0 || N < 1 || K < 8 || K % 8) return 0;
    return gemm_workspace_bytes(mode, M, N, K);
}

int bz_op_gemm(int mode, const void* a, const void* w, const void* r, void* c, int M, int N, int K, void* workspace,
               size_t workspace_bytes, void* stream) {
    if (mode < 0 || mode > 2 || !a || !w || !c || (mode == 1 && !r)) return BZ_EINVAL;
    if (M < 0 || N < 1 || K < 8 || K % 8) return BZ_EINVAL;
    if (workspace && ((uintptr_t)workspace & 15)) return BZ_EINVAL;
    launch_gemm(mode, (const act_t*)a, (const bf16*)w, (const act_t*)r, (act_t*)c, M, N, K, (float*)workspace,
                workspace_bytes, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return BZ_OK;
}

// ---- bz_op_gemm for callers that cannot allocate ----------------------------------------------
// Same kernels and schedules as bz_op_gemm; the scratch the schedules need (split-K partial sums,
// partial tiles) lives in a file-scope device array instead of a caller's workspace.  In host code the
// array's name is only a handle for hipGetSymbolAddress: the address that kernels and copies use is
// looked up once per device, with that device current, and kept.

}  // extern "C"

static __device__ __align__(256) unsigned char scratch[BZ_STATIC_SCRATCH_BYTES];

namespace {

std::atomic<void*> g_scratch_ptr[64];        // per device ordinal; nullptr until looked up

int static_scratch_of_current_device(void** out) {
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    if (dev < 0 || dev >= 64) return BZ_EINVAL;
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        HIP_TRY(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return BZ_EHIP;
        g_scratch_ptr[dev].store(p, std::memory_order_release);     // racing threads store the same address
    }
    *out = p;
    return BZ_OK;
}

}  // namespace

extern "C" {

int bz_op_gemm_static(int mode, const void* a, const void* w, const void* r, void* c, int M, int N, int K,
                      void* stream) {
    if (mode < 0 || mode > 2 || !a || !w || !c || (mode == 1 && !r)) return BZ_EINVAL;
    if (M < 0 || N < 1 || K < 8 || K % 8) return BZ_EINVAL;
    const size_t need = gemm_workspace_bytes(mode, M, N, K);
    if (need > (size_t)BZ_STATIC_SCRATCH_BYTES) return BZ_ECAPACITY;      // before anything touches the GPU
    void* ws = nullptr;
    int rc = static_scratch_of_current_device(&ws);
    if (rc) return rc;
    // nothing in the scratch has to start at zero: every schedule writes each partial sum it later reads
    launch_gemm(mode, (const act_t*)a, (const bf16*)w, (const act_t*)r, (act_t*)c, M, N, K, (float*)ws,
                (size_t)BZ_STATIC_SCRATCH_BYTES, (hipStream_t)stream);
    HIP_TRY(hipGetLastError());
    return BZ_OK;
}

}  // extern "C"
