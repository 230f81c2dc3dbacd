// Internal definitions of the instance and batch objects, shared by the translation units that
// implement the C ABI.
#pragma once

#include <string>
#include <vector>

#include "common.h"
#include "kv_slots.h"

namespace bz {

struct Shape {
    int L, H, Hq, Hkv, d, F;
    int nqkv() const { return (Hq + 2 * Hkv) * d; }
};

struct WsLayout {
    size_t normed, qkv, attn, act, partial, gemm_ws, gemm_ws_bytes, rope, slot_off, slot_cap, total;
};

// kFailed: a HIP call failed while the layer's copies were being enqueued; some of them may be in flight.
// Only bz_unload_layer, which waits for the streams, clears it.
enum LayerState { kNone = 0, kLoading = 1, kResident = 2, kFailed = 3 };

struct ProfRec {
    int cls;
    hipEvent_t e0, e1;
    double flops, bytes;
};

// records a failed HIP call for bz_last_hip_error() and returns BZ_EHIP
int hip_fail(hipError_t e, const char* what);

}  // namespace bz

struct bz_batch {
    int B = 0, T = 0;
    bool all_decode = false;
    std::vector<int32_t> q_start, seq_slot, kv_before;
    int n_prefill_items = 0, n_decode = 0;
    std::vector<int32_t> decode_seqs;
    double prefill_sq = 0;            // sum over prefill sequences of visible (query, key) pairs
    void* dev = nullptr;              // one allocation holding all device arrays
    int32_t *d_q_start = nullptr, *d_seq_slot = nullptr, *d_kv_before = nullptr, *d_token_seq = nullptr,
            *d_items = nullptr, *d_decode = nullptr;
    int4* d_work = nullptr;           // decode work list (see BatchView), room for work_capacity entries
    int work_capacity = 0;
    // storage: either one hipMalloc of the library's (own_dev) or memory the caller lent (bz_batch_create_in)
    bool own_dev = false;
    size_t dev_bytes = 0;
    // caller's pinned host memory the description is laid out in before the upload: two halves of dev_bytes
    // used in turn, so that the host can lay out the next description while the last upload is still queued
    void* staging = nullptr;
    hipEvent_t staged_ev[2] = {nullptr, nullptr};   // upload out of half h has completed
    bool staged_valid[2] = {false, false};
    int staging_next = 0;
    size_t off_words[6] = {0, 0, 0, 0, 0, 0};       // q_start, seq_slot, kv_before, token_seq, items, decode (32-bit words from dev)
    size_t work_at = 0;                             // byte offset of the work list
    // Ordering between streams.  A batch may be run by two instances with different compute streams (a split
    // pair).  Runs that must be ordered against a later device-side change of the batch (advance, rebuild)
    // leave an event per stream; the change leaves one that later runs on other streams wait for.
    struct Use { hipStream_t st; hipEvent_t ev; };
    mutable std::vector<Use> runs;
    hipStream_t changed_on = nullptr;
    hipEvent_t changed_ev = nullptr;
    bool changed_valid = false;
};

struct bz_instance {
    bz_config cfg;
    bz::Shape sh;
    bz_sizes sz;
    bz_layer_layout lay;
    bz::WsLayout ws;
    bool dry = false;
    hipStream_t compute = nullptr, copy = nullptr;
    bool own_compute = false, own_copy = false;
    // second copy stream (always the library's own, created by the first bz_set_ingest_streams(2)): a layer's
    // tensor groups are then cut in two halves, one per stream
    hipStream_t copy2 = nullptr;
    bool own_copy2 = false;
    int ingest_streams = 1;
    unsigned char* weights = nullptr;
    unsigned char* kv = nullptr;
    unsigned char* wsp = nullptr;
    bool own_weights = false, own_kv = false, own_ws = false;
    std::vector<int> state;
    std::vector<hipEvent_t> ev;                  // layer l is complete
    // A layer copied in blob order also records an event when each group of tensors that one stage of
    // the layer needs has landed: [3l] QKV group (g1, wq, wk, wv), [3l+1] wo and g2, [3l+2] wg and wu;
    // the down projection waits for ev[l].  parts_valid[l] says whether the current load recorded them.
    std::vector<hipEvent_t> ev_part;
    std::vector<hipEvent_t> ev_part2;            // [4l + p]: the second stream's half of tensor group p of layer l
    std::vector<char> parts_valid;               // 0: no group events for the current load; 1 / 2: recorded on one / two streams
    hipEvent_t t0 = nullptr;
    bool clock_started = false;
    bz::KvSlots* slots = nullptr;
    bz_stats stats;
    bool prof_on = false;
    std::vector<bz::ProfRec> prof;
    std::vector<hipEvent_t> ev_pool;
    std::vector<hipStream_t> shard_streams;      // created on first sharded load
    std::vector<hipEvent_t> shard_events;
    hipEvent_t order_ev = nullptr;               // scratch event of bz_wait_stream / bz_signal_stream
};
