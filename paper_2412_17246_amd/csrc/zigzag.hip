// Request scheduling between a loading (target) and a loaded (source) instance while layers are
// still arriving: the best-effort policy and the ILP-free ZigZag policy of the paper's section 5.2.
//
// The decisions live in one small class (ZzCore) that knows nothing about time or GPUs.  Two
// drivers use it: a virtual-time simulation in units of one layer execution (bz_zz_simulate, used
// to check the decisions against the CPU oracle and the paper's worked example) and the real
// driver (bz_zz_run), which polls the target's frontier and the two compute streams and issues
// bz_run_layers / hand-offs accordingly.
#include <chrono>
#include <new>
#include <thread>
#include <vector>

#include "instance.h"

using namespace bz;

namespace {

#define HIP_TRY(call)                                       \
    do {                                                    \
        hipError_t e__ = (call);                            \
        if (e__ != hipSuccess) return hip_fail(e__, #call); \
    } while (0)

// Queue state and the two choices of the ILP-free ZigZag policy.  Requests are numbered in
// arrival order (FCFS).
class ZzCore {
  public:
    ZzCore(int n_layers, int n_requests)
        : L(n_layers), done(n_requests, 0), with_source(n_requests, 0) {}
    int n() const { return (int)done.size(); }
    bool finished_or_taken(int r) const { return with_source[r] || done[r] >= L; }
    bool all_placed() const {
        for (int r = 0; r < n(); ++r)
            if (!finished_or_taken(r)) return false;
        return true;
    }
    // Source, when idle: the first request that is neither finished nor taken.  If the target is in
    // the middle of a layer of exactly that request, the source waits (returns -1): no skipping ahead.
    int pick_source(int target_running) const {
        for (int r = 0; r < n(); ++r)
            if (!finished_or_taken(r)) return r == target_running ? -1 : r;
        return -1;
    }
    // Target, when idle: the first request, in arrival order, whose next layer is resident.
    int pick_target(int resident_layers) const {
        for (int r = 0; r < n(); ++r)
            if (!finished_or_taken(r) && done[r] < resident_layers) return r;
        return -1;
    }
    const int L;
    std::vector<int> done;          // layers executed so far (all on the target until the source takes over)
    std::vector<char> with_source;  // the source has taken the request and runs the rest
};

// Layers resident at time t (layer k from k * load_time on).  Settled against the products k * load_time
// themselves: event times are such products, and the quotient t / load_time may round to just below k for them.
int resident_at(double t, double load_time, int L) {
    if (load_time <= 0) return L;
    const double q = t / load_time;
    int k = q >= (double)L ? L : (int)q + 1;
    if (k < 1) k = 1;
    if (k > L) k = L;
    while (k < L && (double)k * load_time <= t) ++k;
    while (k > 1 && (double)(k - 1) * load_time > t) --k;
    return k;
}

}  // namespace

struct bz_zz_trace_rec {
    int32_t request, instance, layer_a, layer_b, frontier;
    float t_ms;
};

struct bz_zz {
    bz_instance* target = nullptr;
    bz_instance* source = nullptr;
    int policy = 0;
    std::vector<const bz_batch*> batch;
    std::vector<void*> hid_t, hid_s;
    std::vector<int> T;
    std::vector<bz_zz_trace_rec> trace;
    hipEvent_t ev_t = nullptr, ev_s = nullptr, ev_hand = nullptr;
};

extern "C" {

int bz_zz_simulate(int policy, int n_layers, int n_requests, double load_time, double source_free_at,
                   int32_t* T_out, double* finish_out) {
    return bz_zz_simulate_weighted(policy, n_layers, n_requests, load_time, source_free_at, nullptr, T_out, finish_out);
}

int bz_zz_simulate_weighted(int policy, int n_layers, int n_requests, double load_time, double source_free_at,
                            const double* layer_time, int32_t* T_out, double* finish_out) try {
    if (n_layers < 1 || n_requests < 1 || !T_out || !finish_out || load_time < 0 || source_free_at < 0) return BZ_EINVAL;
    if (policy != BZ_ZZ_ZIGZAG && policy != BZ_ZZ_BEST_EFFORT) return BZ_EINVAL;
    const int L = n_layers, N = n_requests;
    std::vector<double> w(N, 1.0);                 // time of one layer of request r
    if (layer_time)
        for (int r = 0; r < N; ++r) {
            if (!(layer_time[r] > 0) || layer_time[r] > 1e300) return BZ_EINVAL;      // also refuses NaN
            w[r] = layer_time[r];
        }
    if (policy == BZ_ZZ_BEST_EFFORT) {
        const int half = L / 2 > 1 ? L / 2 : 1;
        double t_target = 0, t_source = source_free_at;
        for (int r = 0; r < N; ++r) {
            int k = resident_at(t_target, load_time, L);
            if (k > half) k = half;
            if (k < 1) k = 1;
            const double handed = t_target + k * w[r];
            t_target = handed;
            T_out[r] = k;
            if (k == L) {                        // a one-layer model: nothing is left for the source
                finish_out[r] = handed;
                continue;
            }
            const double start = t_source > handed ? t_source : handed;
            t_source = start + (L - k) * w[r];
            finish_out[r] = t_source;
        }
        return BZ_OK;
    }
    ZzCore core(L, N);
    std::vector<double> fin(N, -1.0);
    double t = 0, source_free = source_free_at;
    int target_req = -1;
    double target_end = 0;
    for (int guard = 0; guard < 10000000; ++guard) {
        bool open = false;
        for (int r = 0; r < N; ++r) open = open || fin[r] < 0;
        if (!open) break;
        if (target_req >= 0 && target_end <= t) {              // the target's layer ends now
            core.done[target_req] += 1;
            if (core.done[target_req] == L && !core.with_source[target_req]) fin[target_req] = target_end;
            target_req = -1;
        }
        if (source_free <= t) {                                // the source chooses first
            const int r = core.pick_source(target_req);
            if (r >= 0) {
                core.with_source[r] = 1;
                T_out[r] = core.done[r];
                source_free = t + (L - core.done[r]) * w[r];
                fin[r] = source_free;
            }
        }
        if (target_req < 0) {
            const int r = core.pick_target(resident_at(t, load_time, L));
            if (r >= 0) {
                target_req = r;
                target_end = t + w[r];
            }
        }
        double nxt = -1;
        auto consider = [&](double v) { if (v > t && (nxt < 0 || v < nxt)) nxt = v; };
        if (target_req >= 0) consider(target_end);
        consider(source_free);
        if (load_time > 0) {
            const int k = resident_at(t, load_time, L);      // layer k is the next to arrive
            if (k < L) consider((double)k * load_time);
        }
        consider(source_free_at);
        if (nxt < 0) break;
        t = nxt;
    }
    for (int r = 0; r < N; ++r) {
        if (!core.with_source[r]) T_out[r] = core.done[r];
        finish_out[r] = fin[r];
    }
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int bz_zz_create(bz_instance* target, bz_instance* source, int policy, bz_zz** out) try {
    if (!out) return BZ_EINVAL;
    *out = nullptr;
    if (!target || !source || target == source) return BZ_EINVAL;
    if (policy != BZ_ZZ_ZIGZAG && policy != BZ_ZZ_BEST_EFFORT) return BZ_EINVAL;
    if (target->sh.L != source->sh.L || target->sh.H != source->sh.H) return BZ_EINVAL;
    if (target->dry || source->dry) return BZ_ESTATE;
    bz_zz* z = new (std::nothrow) bz_zz();
    if (!z) return BZ_ENOMEM;
    z->target = target;
    z->source = source;
    z->policy = policy;
    if (hipEventCreateWithFlags(&z->ev_t, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&z->ev_s, hipEventDisableTiming) != hipSuccess ||
        hipEventCreateWithFlags(&z->ev_hand, hipEventDisableTiming) != hipSuccess) {
        delete z;
        return BZ_EHIP;
    }
    *out = z;
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int bz_zz_destroy(bz_zz* z) {
    if (!z) return BZ_EINVAL;
    if (z->ev_t) (void)hipEventDestroy(z->ev_t);
    if (z->ev_s) (void)hipEventDestroy(z->ev_s);
    if (z->ev_hand) (void)hipEventDestroy(z->ev_hand);
    delete z;
    return BZ_OK;
}

int bz_zz_submit(bz_zz* z, const bz_batch* batch, void* hidden_target, void* hidden_source) try {
    if (!z || !batch || !hidden_target || !hidden_source || hidden_target == hidden_source) return BZ_EINVAL;
    z->batch.push_back(batch);
    z->hid_t.push_back(hidden_target);
    z->hid_s.push_back(hidden_source);
    z->T.push_back(0);
    return (int)z->batch.size() - 1;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

// Hand-off of request r after `done` layers: copy the activation on the target's stream, then make
// the source's stream wait for that copy.
static int handoff(bz_zz* z, int r) {
    const size_t bytes = (size_t)z->batch[r]->T * z->target->sh.H * sizeof(act_t);
    HIP_TRY(hipMemcpyAsync(z->hid_s[r], z->hid_t[r], bytes, hipMemcpyDeviceToDevice, z->target->compute));
    HIP_TRY(hipEventRecord(z->ev_hand, z->target->compute));
    HIP_TRY(hipStreamWaitEvent(z->source->compute, z->ev_hand, 0));
    return BZ_OK;
}

int bz_zz_run(bz_zz* z) try {
    if (!z) return BZ_EINVAL;
    const int N = (int)z->batch.size();
    if (N == 0) return BZ_OK;
    bz_instance* tg = z->target;
    bz_instance* sr = z->source;
    const int L = tg->sh.L;
    const auto t0 = std::chrono::steady_clock::now();
    auto now_ms = [&]() { return std::chrono::duration<float, std::milli>(std::chrono::steady_clock::now() - t0).count(); };
    auto log = [&](int r, int inst, int a, int b, int f) { z->trace.push_back({r, inst, a, b, f, now_ms()}); };

    if (z->policy == BZ_ZZ_BEST_EFFORT) {
        const int half = L / 2 > 1 ? L / 2 : 1;
        for (int r = 0; r < N; ++r) {
            int f = bz_frontier(tg);
            if (f < 0) return f;
            if (f < 1) {                                   // nothing resident yet: wait for the first layer
                int rc = bz_wait_layer(tg, 0);
                if (rc) return rc;
                f = bz_frontier(tg);
            }
            const int k = f < half ? f : half;
            int rc = bz_run_layers(tg, 0, k, z->batch[r], z->hid_t[r], 0);
            if (rc) return rc;
            log(r, 0, 0, k, f);
            rc = handoff(z, r);
            if (rc) return rc;
            rc = bz_run_layers(sr, k, L, z->batch[r], z->hid_s[r], 0);    // waits for any layer not resident yet
            if (rc) return rc;
            log(r, 1, k, L, f);
            z->T[r] = k;
        }
        HIP_TRY(hipStreamSynchronize(tg->compute));
        HIP_TRY(hipStreamSynchronize(sr->compute));
        return BZ_OK;
    }

    ZzCore core(L, N);
    int target_req = -1;
    bool source_busy = false;
    while (!core.all_placed() || target_req >= 0) {
        bool progressed = false;
        if (target_req >= 0) {
            const hipError_t e = hipEventQuery(z->ev_t);
            if (e == hipSuccess) {
                core.done[target_req] += 1;
                target_req = -1;
                progressed = true;
            } else if (e != hipErrorNotReady) {
                return hip_fail(e, "hipEventQuery(target)");
            }
        }
        if (source_busy) {
            const hipError_t e = hipEventQuery(z->ev_s);
            if (e == hipSuccess) {
                source_busy = false;
                progressed = true;
            } else if (e != hipErrorNotReady) {
                return hip_fail(e, "hipEventQuery(source)");
            }
        }
        if (!source_busy) {                                // the source chooses first
            const int r = core.pick_source(target_req);
            if (r >= 0) {
                const int k = core.done[r];
                int rc = handoff(z, r);
                if (rc) return rc;
                if (k < L) {
                    rc = bz_run_layers(sr, k, L, z->batch[r], z->hid_s[r], 0);
                    if (rc) return rc;
                }
                HIP_TRY(hipEventRecord(z->ev_s, sr->compute));
                log(r, 1, k, L, bz_frontier(tg));
                core.with_source[r] = 1;
                z->T[r] = k;
                source_busy = true;
                progressed = true;
            }
        }
        if (target_req < 0) {
            const int f = bz_frontier(tg);
            if (f < 0) return f;
            const int r = core.pick_target(f);
            if (r >= 0) {
                const int k = core.done[r];
                int rc = bz_run_layers(tg, k, k + 1, z->batch[r], z->hid_t[r], BZ_RUN_NOWAIT);
                if (rc) return rc;
                HIP_TRY(hipEventRecord(z->ev_t, tg->compute));
                log(r, 0, k, k + 1, f);
                target_req = r;
                progressed = true;
            }
        }
        if (!progressed) std::this_thread::sleep_for(std::chrono::microseconds(20));
    }
    for (int r = 0; r < N; ++r)
        if (!core.with_source[r]) {                        // ran to the end on the target: result goes where the caller expects it
            z->T[r] = L;
            int rc = handoff(z, r);
            if (rc) return rc;
        }
    HIP_TRY(hipStreamSynchronize(tg->compute));
    HIP_TRY(hipStreamSynchronize(sr->compute));
    return BZ_OK;
} catch (const std::bad_alloc&) {
    return BZ_ENOMEM;
} catch (...) {
    return BZ_EINVAL;
}

int bz_zz_layers_on_target(const bz_zz* z, int request) {
    if (!z || request < 0 || request >= (int)z->T.size()) return BZ_EINVAL;
    return z->T[request];
}

int bz_zz_trace(const bz_zz* z, bz_zz_event* out, int max_events) {
    if (!z || (!out && max_events > 0) || max_events < 0) return BZ_EINVAL;
    const int n = (int)z->trace.size() < max_events ? (int)z->trace.size() : max_events;
    for (int i = 0; i < n; ++i) {
        out[i].request = z->trace[i].request;
        out[i].instance = z->trace[i].instance;
        out[i].layer_a = z->trace[i].layer_a;
        out[i].layer_b = z->trace[i].layer_b;
        out[i].frontier = z->trace[i].frontier;
        out[i].t_ms = z->trace[i].t_ms;
    }
    return (int)z->trace.size();
}

}  // extern "C"
