// Host runtime of libspmoe: contexts, the per-layer LRU expert cache (Q_cache), the copy stream and
// the slot events that order copies against kernels, the prediction / prefetch entry points (Alg. 1,
// Alg. 2) and the verify-layer orchestration (cached experts first, missing ones on demand).
#include <hip/hip_runtime.h>

#include <algorithm>
#include <condition_variable>
#include <cstdarg>
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>

#include "spmoe_internal.h"

namespace {

struct Slot {
    void* dev = nullptr;
    int expert = -1;              // routed expert id held, -1 = empty
    hipEvent_t ready = nullptr;   // recorded after the slot's last copy, on the stream that carried it
    hipStream_t ready_stream = nullptr;   // that stream
    hipEvent_t freed = nullptr;   // recorded on the compute stream after the last kernel that reads the slot
    bool ready_pending = false;   // a copy was issued and not yet known to have finished
    bool freed_valid = false;     // `freed` has been recorded since the slot was last written
    bool unused_prefetch = false; // filled by spmoe_prefetch and not yet used by a verify pass
    bool by_prefetch = false;     // the slot's last copy was a prefetch
    uint64_t copy_seq = 0;        // issue order of the slot's last copy
};

struct Layer {
    const void* gate = nullptr;
    std::vector<const void*> host_blob;   // [E] pinned packed blobs (borrowed)
    std::vector<int> slot_of;             // [E] slot index or -1
    std::vector<int> lru;                 // resident experts, head (front) = least recently used
    std::vector<Slot> slots;              // [cache_slots_per_layer]
    std::vector<void*> shared_dev;        // [n_shared] HBM copies of the shared experts
};

struct TimedSpan {
    hipEvent_t begin, end;
    int kind, layer, expert;
};

// One entry of Q_load (Alg. 1 l.9-10): a prediction whose routing is still on its way to the host,
// with the event the prefetch worker waits on (Alg. 2 l.5) before it turns it into copies.
struct LoadTask {
    int layer = 0, n = 0;
    int32_t* dev_idx = nullptr;   // [Tmax * pred_k]
    float* dev_p = nullptr;
    int32_t* host_idx = nullptr;  // pinned
    float* host_p = nullptr;
    hipEvent_t ev = nullptr;
};
constexpr int kLoadQueueSlots = 128;

}  // namespace

// Contexts that profile at the same time share one time origin, so their records can be laid on one
// timeline: the first context to start profiling records it, the others reuse it.
static std::mutex g_prof_mu;
static hipEvent_t g_prof_origin = nullptr;
static int g_prof_active = 0;

struct spmoe_ctx {
    spmoe_config cfg;
    hipStream_t compute = nullptr;
    // Copy streams, all at default priority.  Prefetch copies (Alg. 2) and the copies a verify pass is waiting
    // for use different streams, so an on-demand load is not queued behind prefetches; on-demand copies alternate
    // between two streams, which hides the idle time the link otherwise shows between two dependent copies.
    // With the caller's compute stream that makes four streams, one per hardware queue of a process (HIP's
    // default); a fifth stream shares a queue with another one and was measured to serialise behind it.
    hipStream_t copy[2] = {nullptr, nullptr};
    hipStream_t demand[2] = {nullptr, nullptr};
    unsigned copy_rr = 0, demand_rr = 0;
    int io_chunks = 1;               // copies per expert: 1 = the whole blob at once (batched I/O)
    size_t blob_bytes = 0;
    std::vector<Layer> layers;
    spmoe_stats stats;
    uint64_t copy_seq = 0;
    std::string err;

    // device scratch
    SpmoeRouting route{};
    SpmoeRouting pred{};          // routing scratch of spmoe_predict_experts
    void* h = nullptr;            // [A_tot_max][f] bf16 (fp32 for fp32 weights)
    float* ypart = nullptr;       // [splits][A_tot_max][d]
    int down_splits = 1;          // planes of ypart (the largest K-split count any batch size uses)
    int a_tot_max = 0;

    // pinned host staging for the few integers the host needs
    int32_t* host_idx = nullptr;      // [Tmax * top_k] routing of the current verify batch
    int32_t* host_pred_idx = nullptr; // [Tmax * pred_k]
    float* host_pred_p = nullptr;     // [Tmax * pred_k]
    hipEvent_t host_ready = nullptr;

    // prefetch worker ("Prefetcher" thread of Alg. 2) and its task queue Q_load
    std::mutex meta_mu;               // guards cache metadata, statistics, the copy stream's issue order
    std::mutex q_mu;                  // guards the queue counters below
    std::condition_variable q_work, q_done;
    std::vector<LoadTask> q_load;     // ring of kLoadQueueSlots entries, allocated at the first asynchronous call
    uint64_t q_enqueued = 0, q_started = 0, q_finished = 0;
    bool q_stop = false;
    std::thread worker;
    spmoe_status worker_status = SPMOE_OK;
    int device = 0;

    // profiling
    bool profiling = false;
    bool profile_kernels = false;    // also time every kernel launch (adds events between kernels)
    bool profile_log_only = false;   // keep the records (kind, layer, expert, issue order) but record no events
    hipEvent_t prof_origin = nullptr;
    std::vector<TimedSpan> spans;
    hipEvent_t kev[8] = {};          // kernel-boundary events of the last profiled verify call
    std::vector<TimedSpan> kspans;   // kernel spans of the last profiled verify call (kind = kernel index)
};

namespace {

spmoe_status fail(spmoe_ctx* c, spmoe_status st, const char* fmt, ...) {
    if (c) {
        char buf[512];
        va_list ap;
        va_start(ap, fmt);
        vsnprintf(buf, sizeof buf, fmt, ap);
        va_end(ap);
        c->err = buf;
    }
    return st;
}

#define HIP_TRY(c, call)                                                                       \
    do {                                                                                       \
        hipError_t e_ = (call);                                                                \
        if (e_ != hipSuccess) return fail((c), SPMOE_EHIP, "%s: %s", #call, hipGetErrorString(e_)); \
    } while (0)

}  // namespace

bool spmoe_config_ok(const spmoe_config* c, const char** why) {
    if (!c) { *why = "config is NULL"; return false; }
    if (c->weight_dtype != SPMOE_F32 && c->weight_dtype != SPMOE_BF16) { *why = "weight_dtype"; return false; }
    if (c->n_layers < 1) { *why = "n_layers < 1"; return false; }
    if (c->d_model < 32 || c->d_model % 32 || c->d_ff < 32 || c->d_ff % 32) { *why = "d_model and d_ff must be positive multiples of 32"; return false; }
    if (c->weight_dtype == SPMOE_BF16 && c->d_model > 8192) { *why = "d_model > 8192"; return false; }
    if (c->n_experts < 1 || c->n_experts > SPMOE_MAX_EXPERTS) { *why = "n_experts out of range"; return false; }
    if (c->top_k < 1 || c->top_k > SPMOE_MAX_TOPK || c->top_k > c->n_experts) { *why = "top_k out of range"; return false; }
    if (c->n_shared < 0 || c->n_shared > SPMOE_MAX_SHARED) { *why = "n_shared out of range"; return false; }
    if (c->max_tokens < 1 || c->max_tokens > SPMOE_MAX_TOKENS) { *why = "max_tokens out of range"; return false; }
    if (c->cache_slots_per_layer < 1 || c->cache_slots_per_layer > c->n_experts) { *why = "cache_slots_per_layer out of range"; return false; }
    if (c->pred_k < 0 || c->pred_k > SPMOE_MAX_TOPK || c->pred_k > c->n_experts) { *why = "pred_k out of range"; return false; }
    return true;
}

namespace {

bool config_ok(const spmoe_config* c, const char** why) { return spmoe_config_ok(c, why); }

size_t elem_bytes(int dtype) { return dtype == SPMOE_BF16 ? 2 : 4; }

// The kernels read hidden states, gates and weights with 16-byte vector loads.
bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

void lru_touch(Layer& L, int expert) {
    auto it = std::find(L.lru.begin(), L.lru.end(), expert);
    if (it != L.lru.end()) L.lru.erase(it);
    L.lru.push_back(expert);
}

// Picks the slot a new expert goes to: an empty one, else the LRU head's (which is evicted).
int take_slot(spmoe_ctx* c, Layer& L) {
    for (size_t s = 0; s < L.slots.size(); ++s)
        if (L.slots[s].expert < 0) return (int)s;
    const int victim = L.lru.front();
    L.lru.erase(L.lru.begin());
    const int s = L.slot_of[victim];
    L.slot_of[victim] = -1;
    c->stats.evictions += 1;
    if (L.slots[s].unused_prefetch) {
        c->stats.prefetch_wasted += 1;
        L.slots[s].unused_prefetch = false;
    }
    L.slots[s].expert = -1;
    return s;
}

spmoe_status span_begin(spmoe_ctx* c, hipStream_t st, int kind, int layer, int expert, size_t* id) {
    *id = (size_t)-1;
    if (!c->profiling) return SPMOE_OK;
    if (kind >= 4 && !c->profile_kernels) return SPMOE_OK;   // per-kernel spans only on request
    TimedSpan sp{nullptr, nullptr, kind, layer, expert};
    if (!c->profile_log_only) {
        HIP_TRY(c, hipEventCreate(&sp.begin));
        HIP_TRY(c, hipEventCreate(&sp.end));
        HIP_TRY(c, hipEventRecord(sp.begin, st));
    }
    c->spans.push_back(sp);
    *id = c->spans.size() - 1;
    return SPMOE_OK;
}
spmoe_status span_end(spmoe_ctx* c, hipStream_t st, size_t id) {
    if (id == (size_t)-1 || c->profile_log_only) return SPMOE_OK;
    HIP_TRY(c, hipEventRecord(c->spans[id].end, st));
    return SPMOE_OK;
}

// Issues the copy of `expert` into slot s: prefetches on the prefetch stream, copies a verify pass (or a
// warm-up) waits for on the on-demand stream, so that they share the link with prefetches still in flight
// instead of queueing behind them.  The copy waits for the slot's last reader and, when the slot's previous
// copy went over the other stream and may still be running, for that copy.
spmoe_status issue_copy(spmoe_ctx* c, int layer, int expert, int s, bool prefetch) {
    Layer& L = c->layers[layer];
    Slot& sl = L.slots[s];
    hipStream_t stream = prefetch ? c->copy[c->copy_rr++ & 1] : c->demand[c->demand_rr++ & 1];
    if (sl.freed_valid) {
        HIP_TRY(c, hipStreamWaitEvent(stream, sl.freed, 0));
        sl.freed_valid = false;
    }
    if (sl.ready_pending && sl.ready_stream != stream) HIP_TRY(c, hipStreamWaitEvent(stream, sl.ready, 0));
    size_t span;
    spmoe_status st = span_begin(c, stream, prefetch ? 1 : 2, layer, expert, &span);
    if (st != SPMOE_OK) return st;
    // An expert is one contiguous blob, so its three matrices move in one copy (the paper's batched I/O);
    // io_chunks > 1 splits it into that many copies to measure what the batching is worth.
    const size_t chunk = ((c->blob_bytes + c->io_chunks - 1) / c->io_chunks + 255) & ~(size_t)255;
    for (size_t off = 0; off < c->blob_bytes; off += chunk) {
        const size_t nbytes = std::min(chunk, c->blob_bytes - off);
        HIP_TRY(c, hipMemcpyAsync(static_cast<char*>(sl.dev) + off, static_cast<const char*>(L.host_blob[expert]) + off,
                                  nbytes, hipMemcpyHostToDevice, stream));
    }
    st = span_end(c, stream, span);
    if (st != SPMOE_OK) return st;
    HIP_TRY(c, hipEventRecord(sl.ready, stream));
    sl.ready_stream = stream;
    sl.ready_pending = true;
    sl.copy_seq = ++c->copy_seq;
    sl.expert = expert;
    sl.unused_prefetch = prefetch;
    sl.by_prefetch = prefetch;
    L.slot_of[expert] = s;
    L.lru.push_back(expert);
    if (prefetch) {
        c->stats.prefetch_issued += 1;
        c->stats.h2d_bytes_prefetch += (int64_t)c->blob_bytes;
    } else {
        c->stats.ondemand_loads += 1;
        c->stats.h2d_bytes_ondemand += (int64_t)c->blob_bytes;
    }
    return SPMOE_OK;
}

bool copy_done(Slot& sl) {
    if (!sl.ready_pending) return true;
    if (hipEventQuery(sl.ready) == hipSuccess) {
        sl.ready_pending = false;
        return true;
    }
    (void)hipGetLastError();   // hipErrorNotReady is not an error here
    return false;
}

SpmoeShape shape_of(const spmoe_ctx* c, int T) {
    return SpmoeShape{T, c->cfg.top_k, c->cfg.n_experts, c->cfg.n_shared, c->cfg.d_model, c->cfg.d_ff};
}

void kernel_mark(spmoe_ctx* c, int i) {
    if (c->profiling && c->profile_kernels && c->kev[i]) (void)hipEventRecord(c->kev[i], c->compute);
}

// One launch of the two expert GEMMs for the experts in `list`, timed per kernel when profiling.
spmoe_status launch_experts(spmoe_ctx* c, int layer, const SpmoeShape& sh, const SpmoeExpertList& list, const float* x,
                            bool first_after_routing = false) {
    if (list.n <= 0) return SPMOE_OK;
    TimedSpan k2{nullptr, nullptr, 1, 0, list.n}, k3{nullptr, nullptr, 2, 0, list.n};
    size_t busy;
    spmoe_status st = span_begin(c, c->compute, 4, layer, list.n, &busy);   // kernels really executing
    if (st != SPMOE_OK) return st;
    const bool timed = c->profiling && c->profile_kernels;
    if (timed) {
        HIP_TRY(c, hipEventCreate(&k2.begin));
        HIP_TRY(c, hipEventCreate(&k2.end));
        HIP_TRY(c, hipEventCreate(&k3.end));
        k3.begin = k2.end;
        HIP_TRY(c, hipEventRecord(k2.begin, c->compute));
    }
    // the routing kernel zeroed the two unit counters: only the first GEMM pair after it may use them
    int32_t* steal = first_after_routing ? c->route.steal : nullptr;
    HIP_TRY(c, spmoe_launch_gate_up(c->compute, c->cfg.weight_dtype, sh, list, c->route, x, c->h, steal));
    if (timed) HIP_TRY(c, hipEventRecord(k2.end, c->compute));
    HIP_TRY(c, spmoe_launch_down(c->compute, c->cfg.weight_dtype, sh, list, c->route, c->h, c->ypart,
                                 spmoe_down_splits(c->cfg.weight_dtype, sh.d, sh.f, sh.T),
                                 steal ? steal + 1 : nullptr));
    if (timed) {
        HIP_TRY(c, hipEventRecord(k3.end, c->compute));
        c->kspans.push_back(k2);
        c->kspans.push_back(k3);
    }
    return span_end(c, c->compute, busy);
}

void free_kspans(spmoe_ctx* c) {
    for (auto& s : c->kspans) {
        if (s.kind == 1) { (void)hipEventDestroy(s.begin); (void)hipEventDestroy(s.end); }
        else (void)hipEventDestroy(s.end);   // kind 2 shares its begin with the preceding kind-1 span's end
    }
    c->kspans.clear();
}

void free_spans(spmoe_ctx* c) {
    for (auto& s : c->spans) {
        if (s.begin) (void)hipEventDestroy(s.begin);
        if (s.end) (void)hipEventDestroy(s.end);
    }
    c->spans.clear();
}

spmoe_status check_layer(spmoe_ctx* c, int layer) {
    if (!c) return SPMOE_EINVAL;
    if (layer < 0 || layer >= c->cfg.n_layers) return fail(c, SPMOE_ERANGE, "layer %d out of range [0, %d)", layer, c->cfg.n_layers);
    return SPMOE_OK;
}

// Host half of Alg. 1 (lines 3-6) on routing that has reached the host: rank the predicted experts
// (most-voted first, then larger summed probability, then lower index), keep at most one per cache slot,
// drop the ones already in Q_cache and move those to the queue tail.  Returns the number of experts left
// in out_ids.
spmoe_status rank_and_filter(spmoe_ctx* c, Layer& L, const int32_t* idx, const float* prob, int n, int32_t* out_ids,
                             int* n_out) {
    const int pk = c->cfg.pred_k, E = c->cfg.n_experts;
    int votes[SPMOE_MAX_EXPERTS] = {0};
    double psum[SPMOE_MAX_EXPERTS] = {0.0};
    for (int i = 0; i < n * pk; ++i) {
        const int e = idx[i];
        if (e < 0 || e >= E) return fail(c, SPMOE_EHIP, "prediction kernel returned expert %d", e);
        votes[e] += 1;
        psum[e] += prob[i];
    }
    std::vector<int> order;
    for (int e = 0; e < E; ++e)
        if (votes[e] > 0) order.push_back(e);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) {
        if (votes[a] != votes[b]) return votes[a] > votes[b];
        if (psum[a] != psum[b]) return psum[a] > psum[b];
        return a < b;
    });
    // A task names at most as many experts as the layer has slots (the least-voted ones are left out), so the
    // experts it keeps plus the experts it loads always fit, and its loads never evict what it predicted.
    if ((int)order.size() > c->cfg.cache_slots_per_layer) order.resize(c->cfg.cache_slots_per_layer);
    int m = 0;
    for (int e : order) {
        if (L.slot_of[e] < 0) out_ids[m++] = e;   // Alg. 1: predicted experts that are already cached are dropped ...
        else lru_touch(L, e);                     // ... and moved to the tail, so this task cannot evict them
    }
    *n_out = m;
    return SPMOE_OK;
}

// Alg. 2 for one task (arguments already validated; metadata lock held).
spmoe_status prefetch_locked(spmoe_ctx* c, int layer, const int32_t* experts, int n) {
    Layer& L = c->layers[layer];
    if (c->cfg.cutoff_layer < 0 || layer > c->cfg.cutoff_layer) return SPMOE_OK;   // Alg. 1: only l <= L
    std::vector<int> uniq;
    for (int i = 0; i < n; ++i)
        if (std::find(uniq.begin(), uniq.end(), experts[i]) == uniq.end()) uniq.push_back(experts[i]);
    if ((int)uniq.size() > c->cfg.cache_slots_per_layer) uniq.resize(c->cfg.cache_slots_per_layer);
    for (int e : uniq)
        if (L.slot_of[e] >= 0) lru_touch(L, e);        // predicted and cached: moved to the tail, not loaded
    for (int e : uniq) {                               // Alg. 2: as many victims as loads, copies back to back
        if (L.slot_of[e] >= 0) continue;
        if (!L.host_blob[e]) return fail(c, SPMOE_ESTATE, "expert %d of layer %d is not registered", e, layer);
        const int s = take_slot(c, L);
        spmoe_status st = issue_copy(c, layer, e, s, true);
        if (st != SPMOE_OK) return st;
    }
    return SPMOE_OK;
}

// Launches the predictor (target gate of `layer` on n draft states, top pred_k, plain softmax
// probabilities) and the two small device-to-host copies of its result, all on the compute stream.
spmoe_status launch_prediction(spmoe_ctx* c, int layer, const float* dev_draft_x, int n, int32_t* dev_idx, float* dev_p,
                               int32_t* host_idx, float* host_p) {
    const int pk = c->cfg.pred_k;
    size_t span;
    spmoe_status st = span_begin(c, c->compute, 3, layer, n, &span);
    if (st != SPMOE_OK) return st;
    HIP_TRY(c, spmoe_launch_gate_topk(c->compute, c->cfg.weight_dtype, dev_draft_x, c->layers[layer].gate, n,
                                      c->cfg.n_experts, c->cfg.d_model, pk, 0, dev_idx, dev_p, nullptr, nullptr, nullptr));
    HIP_TRY(c, hipMemcpyAsync(host_idx, dev_idx, sizeof(int32_t) * n * pk, hipMemcpyDeviceToHost, c->compute));
    HIP_TRY(c, hipMemcpyAsync(host_p, dev_p, sizeof(float) * n * pk, hipMemcpyDeviceToHost, c->compute));
    return span_end(c, c->compute, span);
}

spmoe_status sync_streams(spmoe_ctx* c) {
    for (hipStream_t s : {c->copy[0], c->copy[1], c->demand[0], c->demand[1]}) HIP_TRY(c, hipStreamSynchronize(s));
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    return SPMOE_OK;
}

// Waits until the prefetch worker has executed every task queued so far; returns (and clears) its error.
spmoe_status drain(spmoe_ctx* c) {
    std::unique_lock<std::mutex> lk(c->q_mu);
    c->q_done.wait(lk, [&] { return c->q_finished == c->q_enqueued; });
    const spmoe_status st = c->worker_status;
    c->worker_status = SPMOE_OK;
    return st;
}

// Entry points that read or change cache metadata first let the worker finish what was queued before
// them (so the metadata sequence is the program order of the calls) and then hold the metadata lock.
struct Guard {
    std::unique_lock<std::mutex> lk;
    spmoe_status st;
    explicit Guard(spmoe_ctx* c) : st(drain(c)) { lk = std::unique_lock<std::mutex>(c->meta_mu); }
};

// The "Prefetcher" thread of Alg. 2: pops tasks in order, waits for the task's event, then issues the copies.
void worker_main(spmoe_ctx* c) {
    (void)hipSetDevice(c->device);
    for (;;) {
        LoadTask* t = nullptr;
        {
            std::unique_lock<std::mutex> lk(c->q_mu);
            c->q_work.wait(lk, [&] { return c->q_stop || c->q_started < c->q_enqueued; });
            if (c->q_started == c->q_enqueued) return;       // stopping and nothing left
            t = &c->q_load[c->q_started % kLoadQueueSlots];
            c->q_started += 1;
        }
        spmoe_status st = SPMOE_OK;
        if (hipEventSynchronize(t->ev) != hipSuccess) {      // Alg. 2: Event.wait()
            (void)hipGetLastError();
            st = SPMOE_EHIP;
        } else {
            std::lock_guard<std::mutex> meta(c->meta_mu);
            int32_t ids[SPMOE_MAX_EXPERTS];
            int m = 0;
            st = rank_and_filter(c, c->layers[t->layer], t->host_idx, t->host_p, t->n, ids, &m);
            if (st == SPMOE_OK) st = prefetch_locked(c, t->layer, ids, m);
        }
        {
            std::lock_guard<std::mutex> lk(c->q_mu);
            if (st != SPMOE_OK && c->worker_status == SPMOE_OK) c->worker_status = st;
            c->q_finished += 1;
        }
        c->q_done.notify_all();
    }
}

spmoe_status start_worker(spmoe_ctx* c) {
    if (c->worker.joinable()) return SPMOE_OK;
    const int pk = std::max(c->cfg.pred_k, 1), Tm = c->cfg.max_tokens;
    c->q_load.resize(kLoadQueueSlots);
    // An entry that an earlier, failed attempt already filled is kept (stop_worker frees whatever exists).
    for (auto& t : c->q_load) {
        if (!t.dev_idx) HIP_TRY(c, hipMalloc(&t.dev_idx, sizeof(int32_t) * Tm * pk));
        if (!t.dev_p) HIP_TRY(c, hipMalloc(&t.dev_p, sizeof(float) * Tm * pk));
        if (!t.host_idx)
            HIP_TRY(c, hipHostMalloc(reinterpret_cast<void**>(&t.host_idx), sizeof(int32_t) * Tm * pk, hipHostMallocDefault));
        if (!t.host_p)
            HIP_TRY(c, hipHostMalloc(reinterpret_cast<void**>(&t.host_p), sizeof(float) * Tm * pk, hipHostMallocDefault));
        if (!t.ev) HIP_TRY(c, hipEventCreateWithFlags(&t.ev, hipEventDisableTiming));
    }
    c->worker = std::thread(worker_main, c);
    return SPMOE_OK;
}

void stop_worker(spmoe_ctx* c) {
    if (c->worker.joinable()) {
        {
            std::lock_guard<std::mutex> lk(c->q_mu);
            c->q_stop = true;
        }
        c->q_work.notify_all();
        c->worker.join();
    }
    for (auto& t : c->q_load) {
        if (t.dev_idx) (void)hipFree(t.dev_idx);
        if (t.dev_p) (void)hipFree(t.dev_p);
        if (t.host_idx) (void)hipHostFree(t.host_idx);
        if (t.host_p) (void)hipHostFree(t.host_p);
        if (t.ev) (void)hipEventDestroy(t.ev);
    }
    c->q_load.clear();
}

}  // namespace

extern "C" {

size_t spmoe_expert_blob_bytes(const spmoe_config* cfg) {
    const char* why;
    if (!config_ok(cfg, &why)) return 0;
    return (size_t)3 * cfg->d_model * cfg->d_ff * elem_bytes(cfg->weight_dtype);
}

spmoe_status spmoe_pack_expert(const spmoe_config* cfg, const void* host_w_gate, const void* host_w_up,
                               const void* host_w_down, void* host_blob_out) {
    const char* why;
    if (!config_ok(cfg, &why) || !host_w_gate || !host_w_up || !host_w_down || !host_blob_out) return SPMOE_EINVAL;
    const size_t d = cfg->d_model, f = cfg->d_ff;
    if (cfg->weight_dtype == SPMOE_F32) {
        char* o = static_cast<char*>(host_blob_out);
        memcpy(o, host_w_gate, d * f * 4);
        memcpy(o + d * f * 4, host_w_up, d * f * 4);
        memcpy(o + 2 * d * f * 4, host_w_down, d * f * 4);
        return SPMOE_OK;
    }
    // bf16: 8-element (16-byte) chunks are moved into 16x32 tiles in MFMA A-operand lane order.
    struct Chunk { uint64_t lo, hi; };
    const Chunk* g = static_cast<const Chunk*>(host_w_gate);
    const Chunk* u = static_cast<const Chunk*>(host_w_up);
    const Chunk* dn = static_cast<const Chunk*>(host_w_down);
    Chunk* out = static_cast<Chunk*>(host_blob_out);
    {   // gate / up: rows n in [0,f), contraction over d; tiles interleaved gate, up
        const size_t ks_total = d / 32, chunks_per_row = d / 8;
        #pragma omp parallel for schedule(static)
        for (size_t n = 0; n < f; ++n) {
            const size_t nt = n / 16, r = n % 16;
            for (size_t cidx = 0; cidx < chunks_per_row; ++cidx) {
                const size_t ks = cidx / 4, kg = cidx % 4, lane = kg * 16 + r;
                const size_t tile = (nt * ks_total + ks) * 2;
                out[(tile + 0) * 64 + lane] = g[n * chunks_per_row + cidx];
                out[(tile + 1) * 64 + lane] = u[n * chunks_per_row + cidx];
            }
        }
    }
    {   // down: rows i in [0,d), contraction over f; the tiles of N-tiles 2p and 2p+1 interleaved per k-step
        Chunk* od = out + (2 * d * f) / 8;
        const size_t ks_total = f / 32, chunks_per_row = f / 8;
        #pragma omp parallel for schedule(static)
        for (size_t i = 0; i < d; ++i) {
            const size_t nt = i / 16, r = i % 16;
            for (size_t cidx = 0; cidx < chunks_per_row; ++cidx) {
                const size_t ks = cidx / 4, kg = cidx % 4, lane = kg * 16 + r;
                od[(((nt / 2) * ks_total + ks) * 2 + (nt % 2)) * 64 + lane] = dn[i * chunks_per_row + cidx];
            }
        }
    }
    return SPMOE_OK;
}

spmoe_status spmoe_create(const spmoe_config* cfg, void* compute_stream, spmoe_ctx** out) {
    const char* why = "";
    if (!out) return SPMOE_EINVAL;
    if (!config_ok(cfg, &why)) {
        if (cfg && (cfg->n_experts > SPMOE_MAX_EXPERTS || cfg->max_tokens > SPMOE_MAX_TOKENS || cfg->top_k > SPMOE_MAX_TOPK))
            return SPMOE_ERANGE;
        return SPMOE_EINVAL;
    }
    spmoe_ctx* c = new (std::nothrow) spmoe_ctx();
    if (!c) return SPMOE_ENOMEM;
    c->cfg = *cfg;
    c->compute = static_cast<hipStream_t>(compute_stream);
    (void)hipGetDevice(&c->device);
    c->blob_bytes = spmoe_expert_blob_bytes(cfg);
    memset(&c->stats, 0, sizeof c->stats);
    const int E = cfg->n_experts, S = cfg->cache_slots_per_layer, Tm = cfg->max_tokens;
    const int E_tot = E + cfg->n_shared;
    c->a_tot_max = Tm * cfg->top_k + cfg->n_shared * Tm;
    // ypart holds one plane per K-split of the down projection; batches of at most 16 and of more tokens may split differently
    c->down_splits = std::max(spmoe_down_splits(cfg->weight_dtype, cfg->d_model, cfg->d_ff, 1),
                              spmoe_down_splits(cfg->weight_dtype, cfg->d_model, cfg->d_ff, Tm));

#define CREATE_TRY(call)                                                             \
    do {                                                                             \
        hipError_t e_ = (call);                                                      \
        if (e_ != hipSuccess) {                                                      \
            const bool oom = (e_ == hipErrorOutOfMemory);                            \
            (void)hipGetLastError();                                                 \
            spmoe_destroy(c);                                                        \
            return oom ? SPMOE_ENOMEM : SPMOE_EHIP;                                  \
        }                                                                            \
    } while (0)

    // SPMOE_COPY_STREAMS (measurement only): 1 = a single stream for all copies (on-demand loads queue behind
    // prefetches), 2 = one stream per kind, 3 = one prefetch stream and two on-demand streams, 4 = two per kind
    int n_streams = 3;
    if (const char* e = getenv("SPMOE_COPY_STREAMS")) {
        if (e[0] >= '1' && e[0] <= '4') n_streams = e[0] - '0';
    }
    CREATE_TRY(hipStreamCreateWithFlags(&c->copy[0], hipStreamNonBlocking));
    if (n_streams == 4) CREATE_TRY(hipStreamCreateWithFlags(&c->copy[1], hipStreamNonBlocking));
    else c->copy[1] = c->copy[0];
    if (n_streams == 1) c->demand[0] = c->copy[0];
    else CREATE_TRY(hipStreamCreateWithFlags(&c->demand[0], hipStreamNonBlocking));
    if (n_streams >= 3) CREATE_TRY(hipStreamCreateWithFlags(&c->demand[1], hipStreamNonBlocking));
    else c->demand[1] = c->demand[0];
    // SPMOE_IO_CHUNKS=n (measurement only): every expert is copied as n pieces instead of one
    if (const char* ch = getenv("SPMOE_IO_CHUNKS")) {
        const int v = atoi(ch);
        if (v >= 1 && v <= 4096) c->io_chunks = v;
    }
    CREATE_TRY(hipEventCreateWithFlags(&c->host_ready, hipEventDisableTiming));
    const int pk = std::max(cfg->pred_k, 1);
    auto alloc_routing = [&](SpmoeRouting& r, int k) -> hipError_t {
        hipError_t e;
        if ((e = hipMalloc(&r.idx, sizeof(int32_t) * Tm * k)) != hipSuccess) return e;
        if ((e = hipMalloc(&r.w, sizeof(float) * Tm * k)) != hipSuccess) return e;
        if ((e = hipMalloc(&r.logits, sizeof(float) * Tm * E)) != hipSuccess) return e;
        if ((e = hipMalloc(&r.xb, sizeof(uint16_t) * Tm * cfg->d_model)) != hipSuccess) return e;
        if ((e = hipMalloc(&r.steal, 2 * sizeof(int32_t))) != hipSuccess) return e;
        // the routing kernel zeroes the unit counters before every layer; start them at zero all the same
        if ((e = hipMemsetAsync(r.steal, 0, 2 * sizeof(int32_t), c->compute)) != hipSuccess) return e;
        return hipStreamSynchronize(c->compute);
    };
    CREATE_TRY(alloc_routing(c->route, cfg->top_k));
    CREATE_TRY(alloc_routing(c->pred, pk));
    CREATE_TRY(hipMalloc(&c->h, (size_t)c->a_tot_max * cfg->d_ff * (cfg->weight_dtype == SPMOE_BF16 ? 2 : 4)));
    CREATE_TRY(hipMalloc(&c->ypart, sizeof(float) * (size_t)c->down_splits * c->a_tot_max * cfg->d_model));
    CREATE_TRY(hipHostMalloc(reinterpret_cast<void**>(&c->host_idx), sizeof(int32_t) * Tm * cfg->top_k, hipHostMallocDefault));
    CREATE_TRY(hipHostMalloc(reinterpret_cast<void**>(&c->host_pred_idx), sizeof(int32_t) * Tm * pk, hipHostMallocDefault));
    CREATE_TRY(hipHostMalloc(reinterpret_cast<void**>(&c->host_pred_p), sizeof(float) * Tm * pk, hipHostMallocDefault));

    c->layers.resize(cfg->n_layers);
    for (auto& L : c->layers) {
        L.host_blob.assign(E, nullptr);
        L.slot_of.assign(E, -1);
        L.slots.resize(S);
        L.shared_dev.assign(cfg->n_shared, nullptr);
    }
    for (auto& L : c->layers) {
        for (auto& sl : L.slots) {
            CREATE_TRY(hipMalloc(&sl.dev, c->blob_bytes));
            CREATE_TRY(hipEventCreateWithFlags(&sl.ready, hipEventDisableTiming));
            CREATE_TRY(hipEventCreateWithFlags(&sl.freed, hipEventDisableTiming));
        }
        for (auto& p : L.shared_dev) CREATE_TRY(hipMalloc(&p, c->blob_bytes));
    }
#undef CREATE_TRY
    *out = c;
    return SPMOE_OK;
}

spmoe_status spmoe_destroy(spmoe_ctx* c) {
    if (!c) return SPMOE_OK;
    stop_worker(c);
    (void)hipStreamSynchronize(c->compute);
    for (hipStream_t s : {c->copy[0], c->copy[1], c->demand[0], c->demand[1]})
        if (s) (void)hipStreamSynchronize(s);
    free_spans(c);
    free_kspans(c);
    for (auto& e : c->kev) if (e) (void)hipEventDestroy(e);
    if (c->profiling) {
        std::lock_guard<std::mutex> lk(g_prof_mu);
        g_prof_active -= 1;
    }
    for (auto& L : c->layers) {
        for (auto& sl : L.slots) {
            if (sl.dev) (void)hipFree(sl.dev);
            if (sl.ready) (void)hipEventDestroy(sl.ready);
            if (sl.freed) (void)hipEventDestroy(sl.freed);
        }
        for (auto& p : L.shared_dev) if (p) (void)hipFree(p);
    }
    auto free_routing = [](SpmoeRouting& r) {
        (void)hipFree(r.idx); (void)hipFree(r.w); (void)hipFree(r.logits); (void)hipFree(r.xb); (void)hipFree(r.steal);
    };
    free_routing(c->route);
    free_routing(c->pred);
    (void)hipFree(c->h);
    (void)hipFree(c->ypart);
    if (c->host_idx) (void)hipHostFree(c->host_idx);
    if (c->host_pred_idx) (void)hipHostFree(c->host_pred_idx);
    if (c->host_pred_p) (void)hipHostFree(c->host_pred_p);
    if (c->host_ready) (void)hipEventDestroy(c->host_ready);
    {
        hipStream_t all[4] = {c->copy[0], c->copy[1], c->demand[0], c->demand[1]};
        for (int i = 0; i < 4; ++i) {
            bool seen = !all[i];
            for (int j = 0; j < i; ++j) seen = seen || all[j] == all[i];
            if (!seen) (void)hipStreamDestroy(all[i]);
        }
    }
    delete c;
    return SPMOE_OK;
}

spmoe_status spmoe_sync(spmoe_ctx* c) {
    if (!c) return SPMOE_EINVAL;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    return sync_streams(c);
}

const char* spmoe_last_error(const spmoe_ctx* c) { return c ? c->err.c_str() : ""; }

spmoe_status spmoe_set_gate(spmoe_ctx* c, int layer, const void* dev_wg) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (!dev_wg) return fail(c, SPMOE_EINVAL, "gate pointer is NULL");
    if (!aligned16(dev_wg)) return fail(c, SPMOE_EINVAL, "gate pointer is not 16-byte aligned");
    c->layers[layer].gate = dev_wg;
    return SPMOE_OK;
}

spmoe_status spmoe_set_cutoff(spmoe_ctx* c, int cutoff_layer) {
    if (!c) return SPMOE_EINVAL;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    c->cfg.cutoff_layer = cutoff_layer;
    return SPMOE_OK;
}

spmoe_status spmoe_expert_cache_register(spmoe_ctx* c, int layer, int expert, const void* pinned_blob) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (expert < 0 || expert >= c->cfg.n_experts) return fail(c, SPMOE_ERANGE, "expert %d out of range", expert);
    if (!pinned_blob) return fail(c, SPMOE_EINVAL, "blob pointer is NULL");
    if (!aligned16(pinned_blob)) return fail(c, SPMOE_EINVAL, "blob pointer is not 16-byte aligned");
    c->layers[layer].host_blob[expert] = pinned_blob;
    return SPMOE_OK;
}

spmoe_status spmoe_expert_cache_register_shared(spmoe_ctx* c, int layer, int idx, const void* pinned_blob) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (idx < 0 || idx >= c->cfg.n_shared) return fail(c, SPMOE_ERANGE, "shared expert %d out of range", idx);
    if (!pinned_blob) return fail(c, SPMOE_EINVAL, "blob pointer is NULL");
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    HIP_TRY(c, hipMemcpy(c->layers[layer].shared_dev[idx], pinned_blob, c->blob_bytes, hipMemcpyHostToDevice));
    return SPMOE_OK;
}

spmoe_status spmoe_expert_cache_warm(spmoe_ctx* c, int layer, const int32_t* host_experts, int n) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (n < 0 || (n > 0 && !host_experts)) return fail(c, SPMOE_EINVAL, "bad expert list");
    Layer& L = c->layers[layer];
    for (int i = 0; i < n; ++i) {
        const int e = host_experts[i];
        if (e < 0 || e >= c->cfg.n_experts) return fail(c, SPMOE_ERANGE, "expert %d out of range", e);
        if (!L.host_blob[e]) return fail(c, SPMOE_ESTATE, "expert %d of layer %d is not registered", e, layer);
    }
    for (int i = 0; i < n; ++i) {
        const int e = host_experts[i];
        if (L.slot_of[e] >= 0) { lru_touch(L, e); continue; }
        const int s = take_slot(c, L);
        st = issue_copy(c, layer, e, s, false);
        if (st != SPMOE_OK) return st;
        L.slots[s].unused_prefetch = false;
        // warm-up is bookkeeping-neutral: it is neither a prefetch nor a verify-time miss
        c->stats.ondemand_loads -= 1;
        c->stats.h2d_bytes_ondemand -= (int64_t)c->blob_bytes;
    }
    st = sync_streams(c);
    if (st != SPMOE_OK) return st;
    for (auto& sl : L.slots) sl.ready_pending = false;
    return SPMOE_OK;
}

spmoe_status spmoe_expert_cache_lookup(spmoe_ctx* c, int layer, int expert, int32_t* host_slot_out) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (expert < 0 || expert >= c->cfg.n_experts) return fail(c, SPMOE_ERANGE, "expert %d out of range", expert);
    if (!host_slot_out) return fail(c, SPMOE_EINVAL, "output pointer is NULL");
    *host_slot_out = c->layers[layer].slot_of[expert];
    return SPMOE_OK;
}

spmoe_status spmoe_expert_cache_contents(spmoe_ctx* c, int layer, int32_t* host_lru_order_out, int32_t* host_n_out) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (!host_lru_order_out || !host_n_out) return fail(c, SPMOE_EINVAL, "output pointer is NULL");
    const Layer& L = c->layers[layer];
    for (size_t i = 0; i < L.lru.size(); ++i) host_lru_order_out[i] = L.lru[i];
    *host_n_out = (int32_t)L.lru.size();
    return SPMOE_OK;
}

spmoe_status spmoe_expert_cache_reset(spmoe_ctx* c) {
    if (!c) return SPMOE_EINVAL;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    spmoe_status st = sync_streams(c);
    if (st != SPMOE_OK) return st;
    for (auto& L : c->layers) {
        L.lru.clear();
        std::fill(L.slot_of.begin(), L.slot_of.end(), -1);
        for (auto& sl : L.slots) {
            sl.expert = -1;
            sl.ready_pending = false;
            sl.freed_valid = false;
            sl.unused_prefetch = false;
        }
    }
    memset(&c->stats, 0, sizeof c->stats);
    return SPMOE_OK;
}

spmoe_status spmoe_expert_cache_stats(spmoe_ctx* c, spmoe_stats* host_out) {
    if (!c) return SPMOE_EINVAL;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (!host_out) return fail(c, SPMOE_EINVAL, "output pointer is NULL");
    *host_out = c->stats;
    return SPMOE_OK;
}

// ---- hot path -------------------------------------------------------------------------------------

spmoe_status spmoe_gate_topk(spmoe_ctx* c, int layer, const float* dev_x, int T, int k, int32_t* dev_idx, float* dev_w,
                             float* dev_logits) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (T < 0 || T > c->cfg.max_tokens) return fail(c, SPMOE_ERANGE, "T=%d exceeds max_tokens=%d", T, c->cfg.max_tokens);
    if (k < 1 || k > SPMOE_MAX_TOPK || k > c->cfg.n_experts) return fail(c, SPMOE_ERANGE, "k=%d out of range", k);
    if (T == 0) return SPMOE_OK;   // an empty batch is a no-op (its pointers may be NULL)
    if (!dev_x || !dev_idx || !dev_w) return fail(c, SPMOE_EINVAL, "NULL device pointer");
    if (!aligned16(dev_x)) return fail(c, SPMOE_EINVAL, "dev_x is not 16-byte aligned");
    if (!c->layers[layer].gate) return fail(c, SPMOE_ESTATE, "gate of layer %d not set", layer);
    HIP_TRY(c, spmoe_launch_gate_topk(c->compute, c->cfg.weight_dtype, dev_x, c->layers[layer].gate, T, c->cfg.n_experts,
                                      c->cfg.d_model, k, c->cfg.renorm_topk, dev_idx, dev_w, dev_logits, nullptr, nullptr));
    return SPMOE_OK;
}

spmoe_status spmoe_token_permutation(spmoe_ctx* c, const int32_t* dev_idx, int T, int k, int32_t* dev_counts,
                                     int32_t* dev_offsets, int32_t* dev_perm) {
    if (!c) return SPMOE_EINVAL;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (!dev_idx || !dev_counts || !dev_offsets || !dev_perm) return fail(c, SPMOE_EINVAL, "NULL device pointer");
    if (T < 0 || T > SPMOE_MAX_TOKENS) return fail(c, SPMOE_ERANGE, "T=%d out of range", T);
    if (k < 1 || k > SPMOE_MAX_TOPK) return fail(c, SPMOE_ERANGE, "k=%d out of range", k);
    HIP_TRY(c, spmoe_launch_permute(c->compute, dev_idx, T, k, c->cfg.n_experts, dev_counts, dev_offsets, dev_perm));
    return SPMOE_OK;
}

spmoe_status spmoe_predict_experts(spmoe_ctx* c, int layer, const float* dev_draft_x, int n, int32_t* host_ids_out,
                                   int32_t* host_n_out) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (!dev_draft_x || !host_ids_out || !host_n_out) return fail(c, SPMOE_EINVAL, "NULL pointer");
    if (!aligned16(dev_draft_x)) return fail(c, SPMOE_EINVAL, "dev_draft_x is not 16-byte aligned");
    if (n < 0 || n > c->cfg.max_tokens) return fail(c, SPMOE_ERANGE, "n=%d exceeds max_tokens=%d", n, c->cfg.max_tokens);
    if (c->cfg.cutoff_layer < 0 || layer > c->cfg.cutoff_layer || n == 0 || c->cfg.pred_k < 1) {   // Alg. 1: only l <= L
        *host_n_out = 0;
        return SPMOE_OK;
    }
    Layer& L = c->layers[layer];
    if (!L.gate) return fail(c, SPMOE_ESTATE, "gate of layer %d not set", layer);
    st = launch_prediction(c, layer, dev_draft_x, n, c->pred.idx, c->pred.w, c->host_pred_idx, c->host_pred_p);
    if (st != SPMOE_OK) return st;
    HIP_TRY(c, hipEventRecord(c->host_ready, c->compute));
    HIP_TRY(c, hipEventSynchronize(c->host_ready));
    int m = 0;
    st = rank_and_filter(c, L, c->host_pred_idx, c->host_pred_p, n, host_ids_out, &m);
    if (st != SPMOE_OK) return st;
    *host_n_out = m;
    return SPMOE_OK;
}

spmoe_status spmoe_predict_prefetch_async(spmoe_ctx* c, int layer, const float* dev_draft_x, int n) {
    if (!c) return SPMOE_EINVAL;
    LoadTask* t = nullptr;
    spmoe_status st = SPMOE_OK;
    {
        std::unique_lock<std::mutex> lk(c->q_mu);
        if (c->worker_status != SPMOE_OK) {
            st = c->worker_status;
            c->worker_status = SPMOE_OK;
            return st;
        }
        // a free ring entry: the worker must have finished the task that used it last
        c->q_done.wait(lk, [&] { return c->q_enqueued - c->q_finished < (uint64_t)kLoadQueueSlots; });
    }
    {
        // the error string, the profiling spans and the configuration are shared with the worker
        std::lock_guard<std::mutex> meta(c->meta_mu);
        st = check_layer(c, layer);
        if (st != SPMOE_OK) return st;
        if (n < 0 || n > c->cfg.max_tokens) return fail(c, SPMOE_ERANGE, "n=%d exceeds max_tokens=%d", n, c->cfg.max_tokens);
        if (c->cfg.cutoff_layer < 0 || layer > c->cfg.cutoff_layer || n == 0 || c->cfg.pred_k < 1) return SPMOE_OK;
        if (!dev_draft_x) return fail(c, SPMOE_EINVAL, "NULL pointer");
        if (!aligned16(dev_draft_x)) return fail(c, SPMOE_EINVAL, "dev_draft_x is not 16-byte aligned");
        if (!c->layers[layer].gate) return fail(c, SPMOE_ESTATE, "gate of layer %d not set", layer);
        st = start_worker(c);
        if (st != SPMOE_OK) return st;
        t = &c->q_load[c->q_enqueued % kLoadQueueSlots];   // only this thread advances q_enqueued
        t->layer = layer;
        t->n = n;
        st = launch_prediction(c, layer, dev_draft_x, n, t->dev_idx, t->dev_p, t->host_idx, t->host_p);
        if (st != SPMOE_OK) return st;
        HIP_TRY(c, hipEventRecord(t->ev, c->compute));     // Alg. 1: Event.record, then Q_load.push_back
    }
    {
        std::lock_guard<std::mutex> lk(c->q_mu);
        c->q_enqueued += 1;
    }
    c->q_work.notify_one();
    return SPMOE_OK;
}

spmoe_status spmoe_prefetch_drain(spmoe_ctx* c) {
    if (!c) return SPMOE_EINVAL;
    return drain(c);
}

spmoe_status spmoe_prefetch(spmoe_ctx* c, int layer, const int32_t* host_experts, int n) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (n < 0 || (n > 0 && !host_experts)) return fail(c, SPMOE_EINVAL, "bad expert list");
    Layer& L = c->layers[layer];
    for (int i = 0; i < n; ++i) {
        const int e = host_experts[i];
        if (e < 0 || e >= c->cfg.n_experts) return fail(c, SPMOE_ERANGE, "expert %d out of range", e);
        if (!L.host_blob[e]) return fail(c, SPMOE_ESTATE, "expert %d of layer %d is not registered", e, layer);
    }
    return prefetch_locked(c, layer, host_experts, n);
}

spmoe_status spmoe_moe_verify_layer(spmoe_ctx* c, int layer, const float* dev_x, int T, float* dev_out) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (T < 0 || T > c->cfg.max_tokens) return fail(c, SPMOE_ERANGE, "T=%d exceeds max_tokens=%d", T, c->cfg.max_tokens);
    if (T == 0) return SPMOE_OK;   // an empty batch is a no-op (its pointers may be NULL)
    if (!dev_x || !dev_out) return fail(c, SPMOE_EINVAL, "NULL device pointer");
    if (!aligned16(dev_x) || !aligned16(dev_out)) return fail(c, SPMOE_EINVAL, "dev_x / dev_out is not 16-byte aligned");
    Layer& L = c->layers[layer];
    if (!L.gate) return fail(c, SPMOE_ESTATE, "gate of layer %d not set", layer);
    const int E = c->cfg.n_experts, dt = c->cfg.weight_dtype;
    const SpmoeShape sh = shape_of(c, T);

    if (c->profiling && c->profile_kernels) {
        free_kspans(c);
        for (auto& e : c->kev) if (!e) HIP_TRY(c, hipEventCreate(&e));
    }
    size_t span;
    st = span_begin(c, c->compute, 0, layer, 0, &span);
    if (st != SPMOE_OK) return st;

    kernel_mark(c, 0);
    size_t k1span;
    st = span_begin(c, c->compute, 5, layer, 0, &k1span);
    if (st != SPMOE_OK) return st;
    HIP_TRY(c, spmoe_launch_gate_topk(c->compute, dt, dev_x, L.gate, T, E, c->cfg.d_model, c->cfg.top_k,
                                      c->cfg.renorm_topk, c->route.idx, c->route.w, c->route.logits, c->route.steal, c->route.xb));
    st = span_end(c, c->compute, k1span);
    if (st != SPMOE_OK) return st;
    kernel_mark(c, 1);

    SpmoeExpertList list;
    list.n = 0;
    auto add = [&](int id, const void* blob) { list.id[list.n] = (uint16_t)id; list.blob[list.n] = blob; list.n += 1; };

    if ((int)L.lru.size() == E) {
        // every routed expert is resident: no routing information is needed on the host
        for (int s = 0; s < c->cfg.n_shared; ++s) add(E + s, L.shared_dev[s]);
        for (int e = 0; e < E; ++e) {
            Slot& sl = L.slots[L.slot_of[e]];
            if (!copy_done(sl)) HIP_TRY(c, hipStreamWaitEvent(c->compute, sl.ready, 0));
            add(e, sl.dev);
        }
        st = launch_experts(c, layer, sh, list, dev_x, true);
        if (st != SPMOE_OK) return st;
    } else {
        // offloaded experts: the routing result (T * k expert ids) decides which experts this batch needs
        const int n_asg = T * c->cfg.top_k;
        HIP_TRY(c, hipMemcpyAsync(c->host_idx, c->route.idx, sizeof(int32_t) * n_asg, hipMemcpyDeviceToHost, c->compute));
        HIP_TRY(c, hipEventRecord(c->host_ready, c->compute));
        HIP_TRY(c, hipEventSynchronize(c->host_ready));
        bool needed[SPMOE_MAX_EXPERTS] = {false};
        for (int a = 0; a < n_asg; ++a) needed[std::min(std::max(c->host_idx[a], 0), E - 1)] = true;
        std::vector<int> hits, misses;
        for (int e = 0; e < E; ++e) {
            if (!needed[e]) continue;
            if (L.slot_of[e] >= 0) hits.push_back(e);
            else {
                if (!L.host_blob[e]) return fail(c, SPMOE_ESTATE, "expert %d of layer %d is needed but not registered", e, layer);
                misses.push_back(e);
            }
        }
        c->stats.hits += (int64_t)hits.size();
        c->stats.misses += (int64_t)misses.size();
        // cached experts first ("Computation Implementation"): those whose data has landed in one launch,
        // then the ones still in flight in the order their copies were issued
        std::vector<int> landed, inflight;
        for (int e : hits) {
            Slot& sl = L.slots[L.slot_of[e]];
            lru_touch(L, e);
            if (sl.unused_prefetch) { sl.unused_prefetch = false; c->stats.prefetch_used += 1; }
            if (copy_done(sl)) landed.push_back(e);
            else { inflight.push_back(e); c->stats.late_hits += 1; }
        }
        std::sort(inflight.begin(), inflight.end(), [&](int a, int b) {
            return L.slots[L.slot_of[a]].copy_seq < L.slots[L.slot_of[b]].copy_seq;
        });
        for (int s = 0; s < c->cfg.n_shared; ++s) add(E + s, L.shared_dev[s]);
        for (int e : landed) add(e, L.slots[L.slot_of[e]].dev);
        st = launch_experts(c, layer, sh, list, dev_x, true);
        if (st != SPMOE_OK) return st;
        for (int e : landed) {
            Slot& sl = L.slots[L.slot_of[e]];
            HIP_TRY(c, hipEventRecord(sl.freed, c->compute));
            sl.freed_valid = true;
        }
        auto run_one = [&](int e, int wait_kind) -> spmoe_status {
            Slot& sl = L.slots[L.slot_of[e]];
            size_t wspan;
            spmoe_status s1 = span_begin(c, c->compute, wait_kind, layer, e, &wspan);
            if (s1 != SPMOE_OK) return s1;
            HIP_TRY(c, hipStreamWaitEvent(c->compute, sl.ready, 0));
            s1 = span_end(c, c->compute, wspan);
            if (s1 != SPMOE_OK) return s1;
            list.n = 0;
            add(e, sl.dev);
            spmoe_status s2 = launch_experts(c, layer, sh, list, dev_x);
            if (s2 != SPMOE_OK) return s2;
            HIP_TRY(c, hipEventRecord(sl.freed, c->compute));
            sl.freed_valid = true;
            return SPMOE_OK;
        };
        for (int e : inflight) {
            st = run_one(e, L.slots[L.slot_of[e]].by_prefetch ? 7 : 8);
            if (st != SPMOE_OK) return st;
        }
        // missing experts: loaded on demand into the LRU head's slot, computed as each copy lands
        for (int e : misses) {
            const int s = take_slot(c, L);
            st = issue_copy(c, layer, e, s, false);
            if (st != SPMOE_OK) return st;
            st = run_one(e, 9);
            if (st != SPMOE_OK) return st;
        }
    }
    kernel_mark(c, 2);
    size_t k4span;
    st = span_begin(c, c->compute, 6, layer, 0, &k4span);
    if (st != SPMOE_OK) return st;
    HIP_TRY(c, spmoe_launch_combine(c->compute, sh, c->route, c->ypart, spmoe_down_splits(dt, sh.d, sh.f, sh.T), dev_out));
    st = span_end(c, c->compute, k4span);
    if (st != SPMOE_OK) return st;
    kernel_mark(c, 3);
    return span_end(c, c->compute, span);
}

// ---- cutoff-layer policy ----------------------------------------------------------------------------

spmoe_status spmoe_suggest_cutoff(int n_layers, int n_layers_draft, int k, double t_comp, double t_io, double m_peak,
                                  double m_expert, double m_gpu, int* host_cutoff_out) {
    if (!host_cutoff_out || n_layers < 1 || n_layers_draft < 1 || k < 1) return SPMOE_EINVAL;
    if (!(t_comp > 0) || !(t_io > 0) || m_expert < 0 || m_peak < 0) return SPMOE_EINVAL;
    int best = -1;
    for (int L = 0; L < n_layers; ++L) {
        const double n_expert = (double)(L + 1) * k;
        const bool mem_ok = m_peak + n_expert * m_expert < m_gpu;
        const double finish = std::max((L - 1) * t_comp + k * t_io, n_expert * t_io);
        const bool time_ok = finish <= n_layers_draft * t_comp;
        if (mem_ok && time_ok) best = L;
    }
    *host_cutoff_out = best;
    return SPMOE_OK;
}

spmoe_status spmoe_measure_expert_load_ms(spmoe_ctx* c, int layer, int expert, int repeats, float* host_ms_out) {
    spmoe_status st = check_layer(c, layer);
    if (st != SPMOE_OK) return st;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (expert < 0 || expert >= c->cfg.n_experts) return fail(c, SPMOE_ERANGE, "expert %d out of range", expert);
    if (!host_ms_out || repeats < 1) return fail(c, SPMOE_EINVAL, "bad arguments");
    const void* src = c->layers[layer].host_blob[expert];
    if (!src) return fail(c, SPMOE_ESTATE, "expert %d of layer %d is not registered", expert, layer);
    void* tmp = nullptr;
    if (hipMalloc(&tmp, c->blob_bytes) != hipSuccess) { (void)hipGetLastError(); return fail(c, SPMOE_ENOMEM, "hipMalloc"); }
    hipEvent_t a = nullptr, b = nullptr;
    spmoe_status res = SPMOE_OK;
    float ms = 0.f;
    if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) res = SPMOE_EHIP;
    if (res == SPMOE_OK) {
        bool ok = hipMemcpyAsync(tmp, src, c->blob_bytes, hipMemcpyHostToDevice, c->copy[0]) == hipSuccess;   // warm-up
        ok = ok && hipEventRecord(a, c->copy[0]) == hipSuccess;
        for (int i = 0; ok && i < repeats; ++i)
            ok = hipMemcpyAsync(tmp, src, c->blob_bytes, hipMemcpyHostToDevice, c->copy[0]) == hipSuccess;
        ok = ok && hipEventRecord(b, c->copy[0]) == hipSuccess && hipEventSynchronize(b) == hipSuccess &&
             hipEventElapsedTime(&ms, a, b) == hipSuccess;
        if (!ok) res = fail(c, SPMOE_EHIP, "timed copy failed: %s", hipGetErrorString(hipGetLastError()));
    }
    if (a) (void)hipEventDestroy(a);
    if (b) (void)hipEventDestroy(b);
    (void)hipFree(tmp);
    if (res == SPMOE_OK) *host_ms_out = ms / repeats;
    return res;
}

// ---- introspection ----------------------------------------------------------------------------------

spmoe_status spmoe_gemm_plan(const spmoe_config* cfg, int projection, int32_t host_plan_out[6]) {
    const char* why;
    if (!config_ok(cfg, &why) || !host_plan_out || (projection != 0 && projection != 1)) return SPMOE_EINVAL;
    if (cfg->weight_dtype != SPMOE_BF16) return SPMOE_EINVAL;
    spmoe_describe_plan(projection, cfg->d_model, cfg->d_ff, cfg->max_tokens, host_plan_out);
    return SPMOE_OK;
}

// ---- measurement ------------------------------------------------------------------------------------

spmoe_status spmoe_profile_begin(spmoe_ctx* c, int mode) {
    if (!c) return SPMOE_EINVAL;
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    free_spans(c);
    {
        spmoe_status st = sync_streams(c);
        if (st != SPMOE_OK) return st;
    }
    {
        std::lock_guard<std::mutex> lk(g_prof_mu);
        if (!c->profiling) {
            if (g_prof_active == 0) {
                if (!g_prof_origin) HIP_TRY(c, hipEventCreate(&g_prof_origin));
                HIP_TRY(c, hipEventRecord(g_prof_origin, c->compute));
                HIP_TRY(c, hipEventSynchronize(g_prof_origin));
            }
            g_prof_active += 1;
        }
        c->prof_origin = g_prof_origin;
    }
    c->profiling = true;
    c->profile_kernels = mode == 1;
    c->profile_log_only = mode == 2;
    return SPMOE_OK;
}

spmoe_status spmoe_profile_collect(spmoe_ctx* c, spmoe_profile_record* host_out, int cap, int* host_n_out) {
    if (!c) return SPMOE_EINVAL;
    if (!host_n_out || (cap > 0 && !host_out)) return fail(c, SPMOE_EINVAL, "NULL output pointer");
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (c->profiling) {
        std::lock_guard<std::mutex> lk(g_prof_mu);
        g_prof_active -= 1;
    }
    c->profiling = false;
    spmoe_status st = sync_streams(c);
    if (st != SPMOE_OK) return st;
    if (!c->prof_origin) return fail(c, SPMOE_ESTATE, "profiling was never started");
    const int n = (int)c->spans.size();
    for (int i = 0; i < n && i < cap; ++i) {
        const TimedSpan& s = c->spans[i];
        float b = 0.f, e = 0.f;
        if (s.begin && s.end) {
            // a span whose call failed half-way has an end event that was never recorded: reported as 0, 0
            if (hipEventElapsedTime(&b, c->prof_origin, s.begin) != hipSuccess ||
                hipEventElapsedTime(&e, c->prof_origin, s.end) != hipSuccess) {
                (void)hipGetLastError();
                b = e = 0.f;
            }
        }
        host_out[i] = spmoe_profile_record{s.kind, s.layer, s.expert, 0, b, e};
    }
    *host_n_out = n;
    return SPMOE_OK;
}

spmoe_status spmoe_last_layer_kernel_ms(spmoe_ctx* c, float host_ms_out[4]) {
    if (!c) return SPMOE_EINVAL;
    if (!host_ms_out) return fail(c, SPMOE_EINVAL, "NULL output pointer");
    Guard guard(c);
    if (guard.st != SPMOE_OK) return guard.st;
    if (!c->kev[0]) return fail(c, SPMOE_ESTATE, "no verify-layer call has run with profiling on");
    HIP_TRY(c, hipStreamSynchronize(c->compute));
    float ms[4] = {0.f, 0.f, 0.f, 0.f};
    HIP_TRY(c, hipEventElapsedTime(&ms[0], c->kev[0], c->kev[1]));
    HIP_TRY(c, hipEventElapsedTime(&ms[3], c->kev[2], c->kev[3]));
    for (const auto& s : c->kspans) {
        float t = 0.f;
        HIP_TRY(c, hipEventElapsedTime(&t, s.begin, s.end));
        ms[s.kind] += t;
    }
    for (int i = 0; i < 4; ++i) host_ms_out[i] = ms[i];
    return SPMOE_OK;
}

}  // extern "C"

