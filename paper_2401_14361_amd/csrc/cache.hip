// The expert cache (Sec. 4.7, Alg. 1 of the paper) as a pool of HBM slots with a
// host-side slot table, miss fills from pinned host memory on a copy stream, and the
// fused per-layer decode step that strings the five steps together.
#include <stdlib.h>
#include <string.h>

#include <atomic>
#include <chrono>
#include <new>
#include <vector>

#include "kernels.hpp"
#include "score.hpp"

namespace moei {

namespace {

thread_local char g_err[512] = "";

constexpr int kMaxAct = 64;  // k + n_shared never exceeds one wavefront
constexpr int kRing = 4;     // buffer sets handed from the routing to the side stream, used in turn
constexpr int kMaxPrefetch = 32;  // prefetch candidates considered per layer step

enum Policy { kPolicyEam = 0, kPolicyLru = 1, kPolicyCount = 2 };

struct SlotUpdates {
    int n;
    int32_t fid[2 * kMaxAct];
    int32_t slot[2 * kMaxAct];
};

// The entries are applied in list order by one thread: a list may name an expert twice (evicted by
// one entry, brought back by a later one) and the last entry must win.
__global__ void apply_slot_updates_kernel(int32_t* __restrict__ slot_of, SlotUpdates u) {
    if (threadIdx.x == 0)
        for (int t = 0; t < u.n; ++t) slot_of[u.fid[t]] = u.slot[t];
}

// Host mirrors in pinned memory so that the device-to-host copies are asynchronous.
struct Pinned {
    int32_t idx[kMaxAct];
    float w[kMaxAct];
    int32_t ev_head[kMaxAct + kMaxPrefetch];
    int32_t pf_head[kMaxPrefetch];
    int32_t best;
    float best_sim;
    int32_t n_list[2];  // n_pf, n_ev
    int32_t flags;
    int32_t best_seq;  // number of the step whose `best` is in place (written by the scoring workgroup after it)
};

}  // namespace

// The synchronous step reads a few words that a kernel writes straight into pinned host memory.
// Waiting for an event costs 10-15 us each time; polling the words themselves costs the time the
// stores take to arrive.  `ready` is polled for at most `limit_us`; false = not seen in time (the
// caller then waits for the event, which also surfaces a failed launch).
template <typename Ready>
static bool poll_pinned(Ready ready, double limit_us) {
    const auto t0 = std::chrono::steady_clock::now();
    for (int spin = 0;; ++spin) {
        if (ready()) {
            std::atomic_thread_fence(std::memory_order_acquire);
            return true;
        }
        if ((spin & 63) == 63 &&
            std::chrono::duration<double, std::micro>(std::chrono::steady_clock::now() - t0).count() > limit_us)
            return false;
        __builtin_ia32_pause();
    }
}
constexpr int32_t kNotWritten = -2;  // a pick the routing kernel has not stored yet (picks are >= -1)
constexpr double kPollLimitUs = 500.0;

void set_error(const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
}

int check_desc(const moei_model_desc* d) {
    MOEI_REQUIRE(d->L >= 1 && d->E >= 1 && d->H >= 1 && d->I >= 1, "model: L, E, H, I must be positive");
    MOEI_REQUIRE(d->k >= 1 && d->k <= d->E, "model: k = %d outside [1, E = %d]", d->k, d->E);
    MOEI_REQUIRE(d->n_shared >= 0 && d->k + d->n_shared <= kMaxAct, "model: k + n_shared = %d exceeds %d",
                 d->k + d->n_shared, kMaxAct);
    MOEI_REQUIRE(d->wdtype == MOEI_WDTYPE_FP32 || d->wdtype == MOEI_WDTYPE_BF16, "model: unknown wdtype %d", d->wdtype);
    MOEI_REQUIRE(d->H <= 16384, "model: H = %d exceeds 16384", d->H);
    MOEI_REQUIRE((long long)d->L * d->E <= (1 << 24), "model: L*E too large");
    MOEI_REQUIRE(d->eps >= 0.f, "model: eps must not be negative");
    return MOEI_OK;
}

}  // namespace moei

using namespace moei;

struct moei_cache {
    moei_model_desc d{};
    int S = 0, n_total = 0, wb = 2;
    size_t slot_elems = 0, slot_bytes = 0;
    unsigned char* d_pool = nullptr;
    const unsigned char* h_experts = nullptr;
    int n_host = 0;
    std::vector<int32_t> slot_of, owner;
    int32_t* d_slot_of = nullptr;
    int32_t* d_flags = nullptr;
    unsigned* d_ticket = nullptr;
    hipStream_t copy_stream = nullptr, side_stream = nullptr;
    hipEvent_t ev_copy = nullptr, ev_routed = nullptr, ev_side = nullptr, ev_main = nullptr;
    hipEvent_t ev_match[kRing] = {};             // end of the side chain of the last step with this parity;
                                                  // ev_side aliases the most recent of the two
    bool match_pending[kRing] = {};
    bool side_pending = false;
    bool poll = true;      // the synchronous step polls pinned memory before it falls back to events (MOEI_SYNC_POLL=0: events only)
    int32_t step_seq = 0;  // number of the last step whose scoring writes into pinned memory
    int parity = 0;  // which buffer set the current step writes
    FfnScratch ffn;
    void* d_items = nullptr;        // batched FFN: token groups, allocated at the first batched call
    int32_t* d_n_items = nullptr;
    float* d_gpart = nullptr;
    float* d_logits = nullptr;
    int32_t* d_idx2[kRing] = {};  // picks of the last kRing steps (the side stream reads one set while the
                                  // routing of later steps writes the others)
    int32_t* d_idx = nullptr;                 // = d_idx2[parity] of the most recent step
    int32_t* d_snap[kRing] = {};  // EAM snapshots the match reads, same rotation
    float* d_w = nullptr;
    int32_t* d_slot_ids = nullptr;
    float* d_gate = nullptr;
    int32_t* d_best = nullptr;  // [kMaxMatchBatch] matched traces of the last step, most similar first
    int match_m = 1;            // traces aggregated by the layer step's prediction
    float* d_best_sim = nullptr;
    float *d_P = nullptr, *d_V = nullptr;
    unsigned long long* d_keys = nullptr;  // [2][L*E] sort keys of the last step (prefetch, eviction)
    int32_t *d_pf_head = nullptr, *d_ev_head = nullptr;  // leading entries of the orders, selected by the step itself
    int last_h_pf = 0, last_h_ev = 0;      // heads the last step was asked to select
    int32_t *d_pf_order = nullptr, *d_ev_order = nullptr, *d_n_pf = nullptr, *d_n_ev = nullptr;
    Pinned* pin = nullptr;
    float* pin_V = nullptr;  // [L*E] eviction scores of the last step (pinned), for the prefetch admission
    Pinned* pin_dev = nullptr;  // the same two blocks as the device addresses them
    float* pin_V_dev = nullptr;
    // eviction policy and its host-side state
    int policy = kPolicyEam;
    std::vector<int64_t> stamp;  // per slot: clock value of its last use (0 = never)
    std::vector<int64_t> count;  // per expert: activations served so far
    int64_t clock = 0;
    // prefetching: copies on their own stream; a slot is "pending" until some stream that reads
    // it has been made to wait for its copy
    int pf_depth = 0;
    hipStream_t pf_stream = nullptr;
    std::vector<hipEvent_t> slot_ev;
    std::vector<char> slot_pending;
    int n_pending = 0;
    long n_prefetched = 0;
    PrefillScratch prefill;  // allocated at the first prefill call, grown when a longer prompt comes
    int32_t last_pf_fid[kMaxPrefetch] = {}, last_pf_victim[kMaxPrefetch] = {};
    int32_t last_n_pf = 0;  // prefetches issued by the last layer step
    // an asynchronous step with prefetching leaves its plan (heads and scores in pinned memory) to be
    // carried out by the host at the next call on this cache: nothing else touches the cache in between
    bool plan_pending = false;
    hipEvent_t plan_event = nullptr;  // end of the side chain that writes the plan
    int plan_depth = 0, plan_k = 0;
    bool pf_gate_recorded = false;  // ev_main already marks the point on the caller's stream that prefetch copies wait for
};

namespace {
void prefill_scratch_free(PrefillScratch* p) {
    (void)hipFree(p->d_idx);
    (void)hipFree(p->d_w);
    (void)hipFree(p->d_perm);
    (void)hipFree(p->d_pgate);
    (void)hipFree(p->d_where);
    (void)hipFree(p->d_items);
    (void)hipFree(p->d_meta);
    (void)hipFree(p->d_act);
    (void)hipFree(p->d_yc);
    *p = PrefillScratch{};
}
}  // namespace

extern "C" const char* moei_last_error(void) { return g_err; }
extern "C" const char* moei_version(void) { return "moei 0.1 (gfx950)"; }

extern "C" int moei_cache_destroy(moei_cache* c) {
    if (!c) return MOEI_OK;
    if (c->copy_stream) (void)hipStreamSynchronize(c->copy_stream);
    if (c->side_stream) (void)hipStreamSynchronize(c->side_stream);
    (void)hipFree(c->d_pool);
    (void)hipFree(c->d_slot_of);
    (void)hipFree(c->d_flags);
    (void)hipFree(c->d_ticket);
    ffn_scratch_free(&c->ffn);
    (void)hipFree(c->d_items);
    (void)hipFree(c->d_n_items);
    (void)hipFree(c->d_gpart);
    (void)hipFree(c->d_logits);
    for (int r = 0; r < kRing; ++r) {
        (void)hipFree(c->d_idx2[r]);
        (void)hipFree(c->d_snap[r]);
        if (c->ev_match[r]) (void)hipEventDestroy(c->ev_match[r]);
    }
    (void)hipFree(c->d_w);
    (void)hipFree(c->d_slot_ids);
    (void)hipFree(c->d_gate);
    (void)hipFree(c->d_best);
    (void)hipFree(c->d_best_sim);
    (void)hipFree(c->d_P);
    (void)hipFree(c->d_V);
    (void)hipFree(c->d_keys);
    (void)hipFree(c->d_pf_head);
    (void)hipFree(c->d_ev_head);
    (void)hipFree(c->d_pf_order);
    (void)hipFree(c->d_ev_order);
    (void)hipFree(c->d_n_pf);
    (void)hipFree(c->d_n_ev);
    prefill_scratch_free(&c->prefill);
    if (c->pin) (void)hipHostFree(c->pin);
    if (c->pin_V) (void)hipHostFree(c->pin_V);
    if (c->pf_stream) {
        (void)hipStreamSynchronize(c->pf_stream);
        (void)hipStreamDestroy(c->pf_stream);
    }
    for (hipEvent_t e : c->slot_ev)
        if (e) (void)hipEventDestroy(e);
    if (c->ev_copy) (void)hipEventDestroy(c->ev_copy);
    if (c->ev_routed) (void)hipEventDestroy(c->ev_routed);
    if (c->ev_main) (void)hipEventDestroy(c->ev_main);
    if (c->copy_stream) (void)hipStreamDestroy(c->copy_stream);
    if (c->side_stream) (void)hipStreamDestroy(c->side_stream);
    delete c;
    return MOEI_OK;
}

namespace {

int upload_slot_table(moei_cache* c) {
    MOEI_HIP(hipMemcpy(c->d_slot_of, c->slot_of.data(), c->slot_of.size() * 4, hipMemcpyHostToDevice));
    return MOEI_OK;
}

int cache_alloc(moei_cache* c) {
    const moei_model_desc& d = c->d;
    const size_t LE = (size_t)d.L * d.E;
    const int na = d.k + d.n_shared;
#define MOEI_DMALLOC(ptr, bytes)                                                                           \
    do {                                                                                                   \
        hipError_t e__ = hipMalloc((void**)&(ptr), (bytes));                                               \
        if (e__ != hipSuccess)                                                                             \
            MOEI_FAIL(MOEI_ENOMEM, "moei_cache_create: device allocation of %zu bytes failed: %s",        \
                      (size_t)(bytes), hipGetErrorString(e__));                                            \
    } while (0)
    MOEI_DMALLOC(c->d_pool, (size_t)c->n_total * c->slot_bytes);
    MOEI_DMALLOC(c->d_slot_of, LE * 4);
    MOEI_DMALLOC(c->d_flags, 4);
    MOEI_DMALLOC(c->d_ticket, 4);
    MOEI_DMALLOC(c->d_logits, (size_t)d.E * 4);
    for (int r = 0; r < kRing; ++r) {
        MOEI_DMALLOC(c->d_idx2[r], (size_t)kMaxAct * 4);
        MOEI_DMALLOC(c->d_snap[r], LE * 4);
    }
    c->d_idx = c->d_idx2[0];
    MOEI_DMALLOC(c->d_w, (size_t)kMaxAct * 4);
    MOEI_DMALLOC(c->d_slot_ids, (size_t)kMaxAct * 4);
    MOEI_DMALLOC(c->d_gate, (size_t)kMaxAct * 4);
    MOEI_DMALLOC(c->d_best, kMaxMatchBatch * 4);
    MOEI_DMALLOC(c->d_best_sim, kMaxMatchBatch * 4);
    MOEI_DMALLOC(c->d_P, LE * 4);
    MOEI_DMALLOC(c->d_V, LE * 4);
    MOEI_DMALLOC(c->d_keys, 2 * LE * 8);
    MOEI_DMALLOC(c->d_pf_head, (size_t)kMaxPrefetch * 4);
    MOEI_DMALLOC(c->d_ev_head, (size_t)(kMaxAct + kMaxPrefetch) * 4);
    MOEI_DMALLOC(c->d_pf_order, LE * 4);
    MOEI_DMALLOC(c->d_ev_order, LE * 4);
    MOEI_DMALLOC(c->d_n_pf, 4);
    MOEI_DMALLOC(c->d_n_ev, 4);
#undef MOEI_DMALLOC
    MOEI_HIP(hipMemset(c->d_flags, 0, 4));
    MOEI_HIP(hipMemset(c->d_ticket, 0, 4));
    MOEI_HIP(hipMemset(c->d_n_pf, 0, 4));
    MOEI_HIP(hipMemset(c->d_n_ev, 0, 4));
    MOEI_HIP(hipMemset(c->d_best, 0xff, kMaxMatchBatch * 4));
    int rc = ffn_scratch_alloc(d, na, &c->ffn);
    if (rc) return rc;
    {
        const char* v = getenv("MOEI_SYNC_POLL");  // read when a cache is created
        c->poll = !(v && *v == '0');
    }
    // mapped, coherent host memory: the routing and scoring kernels of a synchronous step store what the
    // host reads next (picks, matched trace, heads, scores) straight into it
    MOEI_HIP(hipHostMalloc((void**)&c->pin, sizeof(Pinned), hipHostMallocMapped | hipHostMallocCoherent));
    memset(c->pin, 0, sizeof(Pinned));
    MOEI_HIP(hipHostMalloc((void**)&c->pin_V, LE * sizeof(float), hipHostMallocMapped | hipHostMallocCoherent));
    MOEI_HIP(hipHostGetDevicePointer((void**)&c->pin_dev, c->pin, 0));
    MOEI_HIP(hipHostGetDevicePointer((void**)&c->pin_V_dev, c->pin_V, 0));
    MOEI_HIP(hipStreamCreateWithFlags(&c->pf_stream, hipStreamNonBlocking));
    MOEI_HIP(hipStreamCreateWithFlags(&c->copy_stream, hipStreamNonBlocking));
    MOEI_HIP(hipStreamCreateWithFlags(&c->side_stream, hipStreamNonBlocking));
    MOEI_HIP(hipEventCreateWithFlags(&c->ev_copy, hipEventDisableTiming));
    MOEI_HIP(hipEventCreateWithFlags(&c->ev_routed, hipEventDisableTiming));
    for (int r = 0; r < kRing; ++r) MOEI_HIP(hipEventCreateWithFlags(&c->ev_match[r], hipEventDisableTiming));
    MOEI_HIP(hipEventCreateWithFlags(&c->ev_main, hipEventDisableTiming));
    return MOEI_OK;
}

}  // namespace

extern "C" int moei_cache_create(const moei_model_desc* desc, int32_t n_slots, const void* h_experts,
                                 int32_t n_host_experts, const void* h_shared, moei_cache** out) {
    MOEI_REQUIRE(desc && out, "moei_cache_create: null pointer");
    *out = nullptr;
    int rc = check_desc(desc);
    if (rc) return rc;
    MOEI_REQUIRE(n_slots >= 1, "moei_cache_create: n_slots = %d must be positive", n_slots);
    if (n_slots < desc->k)
        MOEI_FAIL(MOEI_ECAPACITY, "moei_cache_create: %d slots cannot hold one layer's %d picks", n_slots, desc->k);
    MOEI_REQUIRE(!h_experts || n_host_experts >= 1, "moei_cache_create: n_host_experts must be positive");
    moei_cache* c = new (std::nothrow) moei_cache();
    if (!c) MOEI_FAIL(MOEI_ENOMEM, "moei_cache_create: out of host memory");
    c->d = *desc;
    c->S = n_slots;
    c->n_total = n_slots + desc->L * desc->n_shared;
    c->wb = desc->wdtype == MOEI_WDTYPE_BF16 ? 2 : 4;
    c->slot_elems = (size_t)3 * desc->H * desc->I;
    c->slot_bytes = c->slot_elems * c->wb;
    c->h_experts = reinterpret_cast<const unsigned char*>(h_experts);
    c->n_host = h_experts ? n_host_experts : 0;
    try {
        c->slot_of.assign((size_t)desc->L * desc->E, -1);
        c->owner.assign((size_t)n_slots, -1);
        c->stamp.assign((size_t)n_slots, 0);
        c->count.assign((size_t)desc->L * desc->E, 0);
        c->slot_ev.assign((size_t)n_slots, nullptr);
        c->slot_pending.assign((size_t)n_slots, 0);
    } catch (...) {
        delete c;
        MOEI_FAIL(MOEI_ENOMEM, "moei_cache_create: out of host memory");
    }
    rc = cache_alloc(c);
    if (rc == MOEI_OK) rc = upload_slot_table(c);
    if (rc == MOEI_OK && h_shared && desc->n_shared > 0) {
        hipError_t e = hipMemcpy(c->d_pool + (size_t)n_slots * c->slot_bytes, h_shared,
                                 (size_t)desc->L * desc->n_shared * c->slot_bytes, hipMemcpyHostToDevice);
        if (e != hipSuccess) {
            set_error("moei_cache_create: copying the shared experts failed: %s", hipGetErrorString(e));
            rc = MOEI_EHIP;
        }
    }
    if (rc) {
        char keep[sizeof(g_err)];
        memcpy(keep, g_err, sizeof(keep));
        moei_cache_destroy(c);
        memcpy(g_err, keep, sizeof(keep));
        return rc;
    }
    *out = c;
    return MOEI_OK;
}

extern "C" int moei_cache_reset(moei_cache* c, int32_t n_resident) {
    MOEI_REQUIRE(c, "moei_cache_reset: null pointer");
    const int LE = c->d.L * c->d.E;
    MOEI_REQUIRE(n_resident >= 0 && n_resident <= c->S && n_resident <= LE,
                 "moei_cache_reset: n_resident = %d outside [0, min(S, L*E)]", n_resident);
    MOEI_HIP(hipDeviceSynchronize());
    c->side_pending = false;
    c->plan_pending = false;
    for (int r = 0; r < kRing; ++r) c->match_pending[r] = false;
    std::fill(c->slot_of.begin(), c->slot_of.end(), -1);
    std::fill(c->owner.begin(), c->owner.end(), -1);
    std::fill(c->stamp.begin(), c->stamp.end(), 0);
    std::fill(c->count.begin(), c->count.end(), 0);
    std::fill(c->slot_pending.begin(), c->slot_pending.end(), 0);
    c->clock = 0;
    c->n_pending = 0;
    c->n_prefetched = 0;
    for (int s = 0; s < n_resident; ++s) {
        c->slot_of[s] = s;
        c->owner[s] = s;
        if (c->h_experts)
            MOEI_HIP(hipMemcpy(c->d_pool + (size_t)s * c->slot_bytes,
                               c->h_experts + (size_t)(s % c->n_host) * c->slot_bytes, c->slot_bytes,
                               hipMemcpyHostToDevice));
    }
    MOEI_HIP(hipMemset(c->d_flags, 0, 4));
    MOEI_HIP(hipMemset(c->d_ticket, 0, 4));
    return upload_slot_table(c);
}

extern "C" int moei_cache_slot_ptr(moei_cache* c, int32_t slot, void** d_ptr) {
    MOEI_REQUIRE(c && d_ptr, "moei_cache_slot_ptr: null pointer");
    MOEI_REQUIRE(slot >= 0 && slot < c->n_total, "moei_cache_slot_ptr: slot %d outside [0, %d)", slot, c->n_total);
    *d_ptr = c->d_pool + (size_t)slot * c->slot_bytes;
    return MOEI_OK;
}

extern "C" int moei_cache_slot_table(moei_cache* c, const int32_t** d_slot_of) {
    MOEI_REQUIRE(c && d_slot_of, "moei_cache_slot_table: null pointer");
    *d_slot_of = c->d_slot_of;
    return MOEI_OK;
}

extern "C" int moei_cache_get_slots(const moei_cache* c, int32_t* h_slot_of) {
    MOEI_REQUIRE(c && h_slot_of, "moei_cache_get_slots: null pointer");
    memcpy(h_slot_of, c->slot_of.data(), c->slot_of.size() * 4);
    return MOEI_OK;
}

namespace {

// A stream that is about to read or overwrite `slot` first waits for a prefetch copy into it
// that nobody has waited for yet.
int settle_pending(moei_cache* c, int slot, hipStream_t waiter) {
    if (slot >= 0 && slot < c->S && c->slot_pending[slot]) {
        MOEI_HIP(hipStreamWaitEvent(waiter, c->slot_ev[slot], 0));
        c->slot_pending[slot] = 0;
        --c->n_pending;
    }
    return MOEI_OK;
}

}  // namespace

extern "C" int moei_cache_retrieve(moei_cache* c, int32_t layer, const int32_t* h_idx, int32_t n,
                                   const int32_t* h_ev_order, int32_t n_ev, int32_t* h_slots, int32_t* h_victims,
                                   int32_t* h_n_miss, void* stream) {
    MOEI_REQUIRE(c && h_idx && h_slots, "moei_cache_retrieve: null pointer");
    MOEI_REQUIRE(layer >= 0 && layer < c->d.L, "moei_cache_retrieve: layer %d outside [0, %d)", layer, c->d.L);
    MOEI_REQUIRE(n >= 0 && n <= kMaxAct, "moei_cache_retrieve: n = %d outside [0, %d]", n, kMaxAct);
    MOEI_REQUIRE(n_ev >= 0 && (n_ev == 0 || h_ev_order), "moei_cache_retrieve: bad eviction order");
    const int E = c->d.E, LE = c->d.L * c->d.E;
    hipStream_t s = as_stream(stream);
    int n_miss = 0;
    for (int j = 0; j < n; ++j) {
        MOEI_REQUIRE(h_idx[j] >= 0 && h_idx[j] < E, "moei_cache_retrieve: expert index %d outside [0, %d)", h_idx[j], E);
        for (int m = 0; m < j; ++m)
            MOEI_REQUIRE(h_idx[m] != h_idx[j], "moei_cache_retrieve: expert %d picked twice", h_idx[j]);
        if (c->slot_of[layer * E + h_idx[j]] < 0) ++n_miss;
    }
    if (n > c->S) MOEI_FAIL(MOEI_ECAPACITY, "moei_cache_retrieve: %d picks exceed the %d slots", n, c->S);
    if (n_miss > 0 && !c->h_experts)
        MOEI_FAIL(MOEI_ESTATE, "moei_cache_retrieve: %d expert(s) not resident and the cache has no host copy", n_miss);
    auto needed = [&](int fid) {
        if (fid < layer * E || fid >= (layer + 1) * E) return false;
        for (int j = 0; j < n; ++j)
            if (h_idx[j] == fid - layer * E) return true;
        return false;
    };
    int pos = 0;
    // the expert that gives up its slot when the cache is full (never one of these picks)
    auto pick_victim = [&]() -> int {
        if (c->policy == kPolicyLru) {  // least recently used slot, ties to the lowest slot
            int best = -1;
            for (int t = 0; t < c->S; ++t)
                if (!needed(c->owner[t]) && (best < 0 || c->stamp[t] < c->stamp[best])) best = t;
            return c->owner[best];
        }
        if (c->policy == kPolicyCount) {  // least often activated expert, ties to the lowest id
            int best = -1;
            for (int t = 0; t < c->S; ++t) {
                const int f = c->owner[t];
                if (needed(f)) continue;
                if (best < 0 || c->count[f] < c->count[best] || (c->count[f] == c->count[best] && f < best)) best = f;
            }
            return best;
        }
        while (pos < n_ev) {  // Alg. 1: lowest eviction priority first
            int cand = h_ev_order[pos++];
            if (cand >= 0 && cand < LE && c->slot_of[cand] >= 0 && !needed(cand)) return cand;
        }
        for (int t = 0; t < c->S; ++t)
            if (!needed(c->owner[t])) return c->owner[t];
        return -1;
    };
    SlotUpdates upd{};
    bool waited = false;
    for (int j = 0; j < n; ++j) {
        const int fid = layer * E + h_idx[j];
        ++c->count[fid];
        int slot = c->slot_of[fid];
        int victim = -1;
        if (slot >= 0) {
            int rc = settle_pending(c, slot, s);  // a hit on a prefetched expert whose copy may be in flight
            if (rc) return rc;
        } else {
            for (int t = 0; t < c->S; ++t)
                if (c->owner[t] < 0) {
                    slot = t;
                    break;
                }
            if (slot < 0) {
                victim = pick_victim();
                if (victim < 0) MOEI_FAIL(MOEI_ESTATE, "moei_cache_retrieve: no slot can be freed");
                slot = c->slot_of[victim];
                c->slot_of[victim] = -1;
                upd.fid[upd.n] = victim;
                upd.slot[upd.n++] = -1;
            }
            c->slot_of[fid] = slot;
            c->owner[slot] = fid;
            upd.fid[upd.n] = fid;
            upd.slot[upd.n++] = slot;
            if (!waited) {  // the slot may still be read by work queued on `stream`
                MOEI_HIP(hipEventRecord(c->ev_main, s));
                MOEI_HIP(hipStreamWaitEvent(c->copy_stream, c->ev_main, 0));
                waited = true;
            }
            int rc = settle_pending(c, slot, c->copy_stream);  // a prefetch into this slot goes first
            if (rc) return rc;
            MOEI_HIP(hipMemcpyAsync(c->d_pool + (size_t)slot * c->slot_bytes,
                                    c->h_experts + (size_t)(fid % c->n_host) * c->slot_bytes, c->slot_bytes,
                                    hipMemcpyHostToDevice, c->copy_stream));
        }
        c->stamp[slot] = ++c->clock;
        h_slots[j] = slot;
        if (h_victims) h_victims[j] = victim;
    }
    if (n_miss > 0) {
        MOEI_HIP(hipEventRecord(c->ev_copy, c->copy_stream));
        MOEI_HIP(hipStreamWaitEvent(s, c->ev_copy, 0));
        launch(K_ROUTE_TOPK, apply_slot_updates_kernel, dim3(1), dim3(kWave), 0, s, c->d_slot_of, upd);
        MOEI_LAUNCH_CHECK();
    }
    if (h_n_miss) *h_n_miss = n_miss;
    return MOEI_OK;
}

extern "C" int moei_cache_set_policy(moei_cache* c, int32_t policy) {
    MOEI_REQUIRE(c, "moei_cache_set_policy: null pointer");
    MOEI_REQUIRE(policy >= kPolicyEam && policy <= kPolicyCount, "moei_cache_set_policy: unknown policy %d", policy);
    c->policy = policy;
    return MOEI_OK;
}

extern "C" int moei_cache_set_prefetch(moei_cache* c, int32_t depth) {
    MOEI_REQUIRE(c, "moei_cache_set_prefetch: null pointer");
    MOEI_REQUIRE(depth >= 0 && depth <= kMaxPrefetch, "moei_cache_set_prefetch: depth = %d outside [0, %d]", depth,
                 kMaxPrefetch);
    if (depth > 0 && !c->h_experts)
        MOEI_FAIL(MOEI_ESTATE, "moei_cache_set_prefetch: the cache has no host copy to prefetch from");
    c->pf_depth = depth;
    return MOEI_OK;
}

extern "C" int moei_cache_prefetch(moei_cache* c, const int32_t* h_pf_order, int32_t n_pf, const int32_t* h_ev_order,
                                   int32_t n_ev, const float* h_V, int32_t depth, const int32_t* h_protect,
                                   int32_t n_protect, int32_t* h_fids, int32_t* h_victims, int32_t* h_slots,
                                   int32_t* h_n_issued, void* stream) {
    MOEI_REQUIRE(c && h_V, "moei_cache_prefetch: null pointer");
    MOEI_REQUIRE(n_pf >= 0 && (n_pf == 0 || h_pf_order), "moei_cache_prefetch: bad prefetch order");
    MOEI_REQUIRE(n_ev >= 0 && (n_ev == 0 || h_ev_order), "moei_cache_prefetch: bad eviction order");
    MOEI_REQUIRE(n_protect >= 0 && (n_protect == 0 || h_protect), "moei_cache_prefetch: bad protect list");
    MOEI_REQUIRE(depth >= 0 && depth <= kMaxPrefetch, "moei_cache_prefetch: depth = %d outside [0, %d]", depth,
                 kMaxPrefetch);
    if (!c->h_experts) MOEI_FAIL(MOEI_ESTATE, "moei_cache_prefetch: the cache has no host copy to prefetch from");
    const int LE = c->d.L * c->d.E;
    const int n_cand = n_pf < depth ? n_pf : depth;
    for (int i = 0; i < n_cand; ++i)
        MOEI_REQUIRE(h_pf_order[i] >= 0 && h_pf_order[i] < LE, "moei_cache_prefetch: expert id %d outside [0, %d)",
                     h_pf_order[i], LE);
    hipStream_t s = as_stream(stream);
    auto is_protected = [&](int fid) {
        for (int i = 0; i < n_protect; ++i)
            if (h_protect[i] == fid) return true;
        return false;
    };
    SlotUpdates upd{};
    int pos = 0, issued = 0;
    bool gated = false;
    for (int i = 0; i < n_cand; ++i) {
        const int fid = h_pf_order[i];
        if (c->slot_of[fid] >= 0) continue;
        int slot = -1, victim = -1;
        for (int t = 0; t < c->S; ++t)
            if (c->owner[t] < 0) {
                slot = t;
                break;
            }
        if (slot < 0) {
            // the cheapest victim that is still there; it is displaced only by a candidate that Alg. 1's
            // own score values more (fp32, the precision the scores are handed over in)
            while (pos < n_ev) {
                const int v = h_ev_order[pos];
                if (v >= 0 && v < LE && c->slot_of[v] >= 0 && !is_protected(v)) break;
                ++pos;
            }
            if (pos >= n_ev) break;
            const int v = h_ev_order[pos];
            if (!(h_V[fid] > h_V[v])) continue;
            victim = v;
            ++pos;
            slot = c->slot_of[victim];
            c->slot_of[victim] = -1;
            upd.fid[upd.n] = victim;
            upd.slot[upd.n++] = -1;
        }
        c->slot_of[fid] = slot;
        c->owner[slot] = fid;
        c->stamp[slot] = ++c->clock;
        upd.fid[upd.n] = fid;
        upd.slot[upd.n++] = slot;
        if (!gated) {  // work already queued on `stream` may still read the slots that are given up
            if (!c->pf_gate_recorded) MOEI_HIP(hipEventRecord(c->ev_main, s));
            MOEI_HIP(hipStreamWaitEvent(c->pf_stream, c->ev_main, 0));
            gated = true;
        }
        if (c->slot_pending[slot]) {  // an unfinished prefetch into this slot: same stream, runs first
            c->slot_pending[slot] = 0;
            --c->n_pending;
        }
        MOEI_HIP(hipMemcpyAsync(c->d_pool + (size_t)slot * c->slot_bytes,
                                c->h_experts + (size_t)(fid % c->n_host) * c->slot_bytes, c->slot_bytes,
                                hipMemcpyHostToDevice, c->pf_stream));
        if (!c->slot_ev[slot]) MOEI_HIP(hipEventCreateWithFlags(&c->slot_ev[slot], hipEventDisableTiming));
        MOEI_HIP(hipEventRecord(c->slot_ev[slot], c->pf_stream));
        c->slot_pending[slot] = 1;
        ++c->n_pending;
        ++c->n_prefetched;
        if (h_fids) h_fids[issued] = fid;
        if (h_victims) h_victims[issued] = victim;
        if (h_slots) h_slots[issued] = slot;
        ++issued;
    }
    if (issued > 0) {
        // the device table names the new owners at once; whoever reads such a slot waits for its copy
        launch(K_ROUTE_TOPK, apply_slot_updates_kernel, dim3(1), dim3(kWave), 0, s, c->d_slot_of, upd);
        MOEI_LAUNCH_CHECK();
    }
    if (h_n_issued) *h_n_issued = issued;
    return MOEI_OK;
}

extern "C" int expert_ffn_gemv(moei_cache* c, const int32_t* d_slot_ids, const float* d_gate_w, int32_t n_act,
                               const void* d_x, float* d_y, void* stream) {
    MOEI_REQUIRE(c && d_x && d_y, "expert_ffn_gemv: null pointer");
    MOEI_REQUIRE(n_act >= 0 && n_act <= c->ffn.n_act_max, "expert_ffn_gemv: n_act = %d outside [0, k + n_shared = %d]",
                 n_act, c->ffn.n_act_max);
    MOEI_REQUIRE(n_act == 0 || (d_slot_ids && d_gate_w), "expert_ffn_gemv: null slot ids or gate weights");
    return launch_expert_ffn(c->d, c->d_pool, c->slot_elems, c->n_total, c->ffn, d_slot_ids, d_gate_w, n_act, d_x, d_y,
                             c->d_flags, as_stream(stream));
}

extern "C" int expert_ffn_gemv_static(moei_cache* c, const int32_t* d_slot_ids, const float* d_gate_w, int32_t n_act,
                                      const void* d_x, float* d_y, void* stream) {
    MOEI_REQUIRE(c && d_x && d_y, "expert_ffn_gemv_static: null pointer");
    MOEI_REQUIRE(n_act >= 0 && n_act <= c->ffn.n_act_max,
                 "expert_ffn_gemv_static: n_act = %d outside [0, k + n_shared = %d]", n_act, c->ffn.n_act_max);
    MOEI_REQUIRE(n_act == 0 || (d_slot_ids && d_gate_w), "expert_ffn_gemv_static: null slot ids or gate weights");
    return launch_expert_ffn_static(c->d, c->d_pool, c->slot_elems, c->n_total, c->ffn.n_part, d_slot_ids, d_gate_w,
                                    n_act, d_x, d_y, c->d_flags, as_stream(stream));
}

extern "C" int expert_ffn_grouped(moei_cache* c, int32_t layer, const int32_t* d_idx, const float* d_w, int32_t B,
                                  const void* d_x, float* d_y, void* stream) {
    MOEI_REQUIRE(c && d_idx && d_w && d_x && d_y, "expert_ffn_grouped: null pointer");
    MOEI_REQUIRE(layer >= 0 && layer < c->d.L, "expert_ffn_grouped: layer %d outside [0, %d)", layer, c->d.L);
    MOEI_REQUIRE(B >= 1 && B <= 16, "expert_ffn_grouped: B = %d outside [1, 16]", B);
    if (!c->d_items) {  // scratch of the batched path, on first use
        hipError_t e = hipMalloc(&c->d_items, (size_t)grouped_max_items(c->d) * grouped_item_bytes());
        if (e == hipSuccess) e = hipMalloc((void**)&c->d_n_items, 4);
        if (e == hipSuccess) e = hipMalloc((void**)&c->d_gpart, grouped_part_floats(c->d) * sizeof(float));
        if (e != hipSuccess) {
            (void)hipFree(c->d_items);
            (void)hipFree(c->d_n_items);
            c->d_items = nullptr;
            c->d_n_items = nullptr;
            MOEI_FAIL(MOEI_ENOMEM, "expert_ffn_grouped: scratch allocation failed: %s", hipGetErrorString(e));
        }
    }
    return launch_expert_ffn_grouped(c->d, c->d_pool, c->slot_elems, c->d_items, c->d_n_items, c->d_gpart,
                                     c->d_slot_of + (size_t)layer * c->d.E, c->S + layer * c->d.n_shared, d_idx, d_w, B,
                                     d_x, d_y, c->d_flags, as_stream(stream));
}

extern "C" int moe_prefill_layer(moei_cache* c, int32_t* d_eam, int32_t layer, const void* d_router_w,
                                 const float* d_router_bias, const void* d_X, int32_t n, float* d_Y, int32_t* d_idx_out,
                                 float* d_w_out, void* stream) {
    MOEI_REQUIRE(c && d_eam && d_router_w, "moe_prefill_layer: null pointer");
    const moei_model_desc& d = c->d;
    MOEI_REQUIRE(layer >= 0 && layer < d.L, "moe_prefill_layer: layer %d outside [0, %d)", layer, d.L);
    MOEI_REQUIRE(n >= 0 && n <= 8192, "moe_prefill_layer: n = %d outside [0, 8192]", n);
    int rc = prefill_check(d);
    if (rc) return rc;
    if (n == 0) return MOEI_OK;
    MOEI_REQUIRE(d_X && d_Y, "moe_prefill_layer: null pointer");
    hipStream_t s = as_stream(stream);
    PrefillScratch& p = c->prefill;
    if (n > p.n_max) {  // scratch for the longest prompt so far (not a stream operation: drains the device)
        MOEI_HIP(hipDeviceSynchronize());
        prefill_scratch_free(&p);
        const int n_max = n < 512 ? 512 : n;
        const size_t nk = (size_t)n_max * d.k;
        hipError_t e = hipMalloc((void**)&p.d_idx, nk * 4);
        if (e == hipSuccess) e = hipMalloc((void**)&p.d_w, nk * 4);
        if (e == hipSuccess) e = hipMalloc((void**)&p.d_perm, nk * 4);
        if (e == hipSuccess) e = hipMalloc((void**)&p.d_pgate, nk * 4);
        if (e == hipSuccess) e = hipMalloc((void**)&p.d_where, nk * 4);
        if (e == hipSuccess) e = hipMalloc(&p.d_items, (size_t)prefill_max_items(d, n_max) * prefill_item_bytes());
        if (e == hipSuccess) e = hipMalloc((void**)&p.d_meta, 8);
        if (e == hipSuccess) e = hipMalloc((void**)&p.d_act, prefill_rows(d, n_max) * d.I * 2);
        if (e == hipSuccess) e = hipMalloc((void**)&p.d_yc, prefill_rows(d, n_max) * d.H * sizeof(float));
        if (e != hipSuccess) {
            prefill_scratch_free(&p);
            MOEI_FAIL(MOEI_ENOMEM, "moe_prefill_layer: scratch allocation failed: %s", hipGetErrorString(e));
        }
        p.n_max = n_max;
    }
    rc = launch_prefill(d, p, c->d_pool, c->slot_elems, c->n_total, c->d_slot_of + (size_t)layer * d.E,
                        c->S + layer * d.n_shared, d_eam + (size_t)layer * d.E, d_router_w, d_router_bias, d_X, n, d_Y,
                        c->d_flags, s);
    if (rc) return rc;
    if (d_idx_out) MOEI_HIP(hipMemcpyAsync(d_idx_out, p.d_idx, (size_t)n * d.k * 4, hipMemcpyDeviceToDevice, s));
    if (d_w_out) MOEI_HIP(hipMemcpyAsync(d_w_out, p.d_w, (size_t)n * d.k * 4, hipMemcpyDeviceToDevice, s));
    return MOEI_OK;
}

extern "C" int moei_cache_error_flags(moei_cache* c, int32_t* h_flags, void* stream) {
    MOEI_REQUIRE(c && h_flags, "moei_cache_error_flags: null pointer");
    hipStream_t s = as_stream(stream);
    MOEI_HIP(hipMemcpyAsync(&c->pin->flags, c->d_flags, 4, hipMemcpyDeviceToHost, s));
    MOEI_HIP(hipStreamSynchronize(s));
    *h_flags = c->pin->flags;
    if (c->pin->flags) {
        MOEI_HIP(hipMemsetAsync(c->d_flags, 0, 4, s));
        MOEI_HIP(hipStreamSynchronize(s));
    }
    return MOEI_OK;
}

namespace {
// Carries out the prefetch plan an asynchronous layer step has left behind: waits for that step's
// side chain, then runs the same admission as the synchronous step on the heads and scores it
// wrote to pinned memory.  The cache is in the state that step left it in, so the result is the one
// the synchronous step would have produced right away.
int flush_prefetch_plan(moei_cache* c, hipStream_t s) {
    if (!c->plan_pending) return MOEI_OK;
    c->plan_pending = false;
    MOEI_HIP(hipEventSynchronize(c->plan_event));
    const int LE = c->d.L * c->d.E;
    const int cap_pf = c->plan_depth < LE ? c->plan_depth : LE;
    const int cap_ev = c->plan_k + c->plan_depth < LE ? c->plan_k + c->plan_depth : LE;
    const int n_pf = c->pin->n_list[0] < cap_pf ? c->pin->n_list[0] : cap_pf;
    const int n_ev = c->pin->n_list[1] < cap_ev ? c->pin->n_list[1] : cap_ev;
    return moei_cache_prefetch(c, c->pin->pf_head, n_pf, c->pin->ev_head, n_ev, c->pin_V, c->plan_depth, nullptr, 0,
                               c->last_pf_fid, c->last_pf_victim, nullptr, &c->last_n_pf, s);
}
}  // namespace

extern "C" int moe_decode_layer(moei_cache* c, const moei_eamc* eamc, int32_t* d_eam, int32_t layer,
                                const void* d_router_w, const float* d_router_bias, const void* d_x, float* d_y,
                                int32_t* h_topk_idx, int32_t* h_best, int32_t* h_n_miss, void* stream) {
    MOEI_REQUIRE(c && eamc && d_eam && d_router_w && d_x && d_y, "moe_decode_layer: null pointer");
    const moei_model_desc& d = c->d;
    MOEI_REQUIRE(eamc->d.L == d.L && eamc->d.E == d.E, "moe_decode_layer: EAMC is %dx%d, cache is %dx%d", eamc->d.L,
                 eamc->d.E, d.L, d.E);
    MOEI_REQUIRE(layer >= 0 && layer < d.L, "moe_decode_layer: layer %d outside [0, %d)", layer, d.L);
    hipStream_t s = as_stream(stream);
    const bool sync_mode = h_topk_idx || h_best || h_n_miss;
    const int k = d.k, E = d.E;
    int rc;
    // an asynchronous step plans its prefetches on the device and leaves them to the host; the host
    // cannot be asked in the middle of a stream capture
    const bool plan_prefetch = !sync_mode && c->pf_depth > 0 && c->policy == kPolicyEam && c->h_experts;
    if (plan_prefetch || c->plan_pending) {
        hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
        MOEI_HIP(hipStreamIsCapturing(s, &cap));
        if (cap != hipStreamCaptureStatusNone)
            MOEI_FAIL(MOEI_ESTATE, "moe_decode_layer: prefetching needs the host between layer steps and cannot be captured "
                                   "(moei_cache_set_prefetch(c, 0) before the capture)");
    }
    rc = flush_prefetch_plan(c, s);
    if (rc) return rc;

    // Routing hands the side stream a snapshot of the updated EAM and its picks in one of
    // kRing buffer sets used in turn, so the main stream never waits for the match and scoring
    // of recent steps: it only must not overwrite a set that the step kRing steps back still
    // reads (a wait that has long been satisfied unless the side stream falls far behind).
    c->parity = (c->parity + 1) % kRing;
    if (c->match_pending[c->parity]) MOEI_HIP(hipStreamWaitEvent(s, c->ev_match[c->parity], 0));
    // The asynchronous step picks its slots on the device, so the host cannot tell which
    // prefetch copies it depends on: the stream waits for all that are still unsettled (none in
    // a run that never prefetches; the synchronous step waits slot by slot instead).
    if (!sync_mode && c->n_pending > 0)
        for (int t = 0; t < c->S; ++t) {
            rc = settle_pending(c, t, s);
            if (rc) return rc;
        }
    c->d_idx = c->d_idx2[c->parity];
    int32_t* d_snap = c->d_snap[c->parity];

    RouteFusedArgs ra{};
    ra.W = d_router_w;
    ra.bias = d_router_bias;
    ra.x = d_x;
    ra.H = d.H;
    ra.logits = c->d_logits;
    ra.ticket = c->d_ticket;
    ra.E = E;
    ra.k = k;
    ra.renorm = d.renorm_topk != 0;
    ra.idx = c->d_idx;
    ra.w = c->d_w;
    ra.eam = d_eam;
    ra.snap = d_snap;
    ra.LE = d.L * E;
    ra.layer = layer;
    ra.slot_of_row = c->d_slot_of + (size_t)layer * E;
    ra.n_shared = d.n_shared;
    ra.shared_base = c->S + layer * d.n_shared;
    ra.slot_ids = c->d_slot_ids;
    ra.gate = c->d_gate;
    ra.flags = sync_mode ? nullptr : c->d_flags;
    ra.host_idx = sync_mode ? c->pin_dev->idx : nullptr;
    if (sync_mode && c->poll) {  // only synchronous steps write these words, and each waits for its own
        volatile int32_t* pi = c->pin->idx;
        for (int j = 0; j < k; ++j) pi[j] = kNotWritten;
    }
    rc = launch_route_fused(ra, d.wdtype, s);
    if (rc) return rc;
    MOEI_HIP(hipEventRecord(c->ev_routed, s));
    // Asynchronous step: the expert FFNs go onto the main stream right behind the routing,
    // before any side-stream work is enqueued, so that neither the host-side enqueue time of
    // the match nor a captured graph's branch placement comes between routing and FFN.
    if (!sync_mode) {
        rc = launch_expert_ffn(d, c->d_pool, c->slot_elems, c->n_total, c->ffn, c->d_slot_ids, c->d_gate,
                               k + d.n_shared, d_x, d_y, c->d_flags, s);
        if (rc) return rc;
    }

    // side stream: EAMC match and priorities from the EAM that now holds this layer's routing
    hipStream_t side = c->side_stream;
    MOEI_HIP(hipStreamWaitEvent(side, c->ev_routed, 0));
    // match and scoring in one launch sequence (the workgroup that finishes the match scores
    // the matched trace), then the two orders
    // Alg. 1 takes the victims from the head of the eviction order (one per miss at most) and prefetching
    // looks at `depth` candidates: the step computes those heads; the complete orders are ranked from the
    // step's keys when moei_cache_last_step asks for them
    ScoreArgs sc = make_score_args(eamc, c->d_best, c->match_m, layer, c->d_slot_of, d.eps, c->d_idx, k, c->d_P,
                                   c->d_V, c->d_n_pf, c->d_n_ev);
    sc.keys = c->d_keys;
    sc.pf_order = c->d_pf_head;
    sc.ev_order = c->d_ev_head;
    sc.h_pf = c->pf_depth;
    sc.h_ev = k + c->pf_depth;
    c->last_h_pf = sc.h_pf;
    c->last_h_ev = sc.h_ev;
    if (sync_mode || plan_prefetch) {  // what the host reads goes straight into pinned memory: no copies behind the kernels
        sc.host_best = &c->pin_dev->best;
        sc.host_n = c->pin_dev->n_list;
        sc.host_pf_head = c->pin_dev->pf_head;
        sc.host_ev_head = c->pin_dev->ev_head;
        sc.host_V = (c->pf_depth > 0 && c->policy == kPolicyEam) ? c->pin_V_dev : nullptr;
        sc.host_seq = &c->pin_dev->best_seq;
        sc.seq = ++c->step_seq;
    }
    if (c->match_m == 1)
        rc = launch_match(eamc, d_snap, 1, d.L - 1, c->d_best, c->d_best_sim, nullptr, &sc, side);
    else
        rc = launch_match_topm(eamc, d_snap, d.L - 1, c->match_m, c->d_best, c->d_best_sim, nullptr, &sc, side);
    if (rc) return rc;
    const bool do_prefetch = sync_mode && c->pf_depth > 0 && c->policy == kPolicyEam;
    const int LE = d.L * E;
    const int n_ev_copy = do_prefetch ? (k + c->pf_depth < LE ? k + c->pf_depth : LE) : k;
    const int n_pf_copy = c->pf_depth < LE ? c->pf_depth : LE;
    // one event per step at the end of the side chain (an event record between two kernels
    // costs a few microseconds on its stream): it releases this step's buffer set and is what
    // a join or a host-side wait refers to
    MOEI_HIP(hipEventRecord(c->ev_match[c->parity], side));
    c->match_pending[c->parity] = true;
    c->ev_side = c->ev_match[c->parity];
    c->side_pending = true;

    if (plan_prefetch) {
        c->plan_pending = true;
        c->plan_event = c->ev_match[c->parity];
        c->plan_depth = c->pf_depth;
        c->plan_k = k;
    }
    if (!sync_mode) return MOEI_OK;
    {
        {
            volatile int32_t* pi = c->pin->idx;
            const bool seen = c->poll && poll_pinned([&] {
                for (int j = 0; j < k; ++j)
                    if (pi[j] == kNotWritten) return false;
                return true;
            }, kPollLimitUs);
            if (!seen) MOEI_HIP(hipEventSynchronize(c->ev_routed));
        }
        int n_miss = 0;
        int32_t protect[kMaxAct];
        for (int j = 0; j < k; ++j) {
            int e = c->pin->idx[j];
            if (e < 0 || e >= E)
                MOEI_FAIL(MOEI_ESTATE,
                          "moe_decode_layer: the router produced expert %d (logits that are NaN or have no finite "
                          "maximum give a token no picks)", e);
            if (c->slot_of[layer * E + e] < 0) ++n_miss;
            protect[j] = layer * E + e;
        }
        bool side_done = false;
        // the eviction order is needed only when a pick misses under the paper's policy
        int n_ev = 0;
        if (n_miss > 0 && c->policy == kPolicyEam) {
            MOEI_HIP(hipEventSynchronize(c->ev_side));
            side_done = true;
            n_ev = c->pin->n_list[1] < k ? c->pin->n_list[1] : k;
        }
        // under the comparison policies nothing above waited for the side stream, whose scoring still
        // reads the device slot table that the retrieval is about to change
        if (n_miss > 0 && !side_done) MOEI_HIP(hipStreamWaitEvent(s, c->ev_side, 0));
        int32_t slots[kMaxAct];
        rc = moei_cache_retrieve(c, layer, c->pin->idx, k, c->pin->ev_head, n_ev, slots, nullptr, nullptr, s);
        if (rc) return rc;
        if (n_miss > 0) {
            rc = launch_gather_slots(c->d_idx, k, c->d_slot_of + (size_t)layer * E, c->d_slot_ids + d.n_shared, c->d_flags, s);
            if (rc) return rc;
        }
        // the experts run as soon as their slots are settled: what is left below (prefetch planning,
        // the matched trace for the caller) waits for the side stream while the FFN streams
        // (prefetch copies wait for what is on the stream up to here - earlier steps may still read the
        // slots they take - but not for this layer's experts, whose slots they never touch)
        if (do_prefetch) MOEI_HIP(hipEventRecord(c->ev_main, s));
        rc = launch_expert_ffn(d, c->d_pool, c->slot_elems, c->n_total, c->ffn, c->d_slot_ids, c->d_gate, k + d.n_shared,
                               d_x, d_y, c->d_flags, s);
        if (rc) return rc;
        if (do_prefetch) {
            if (!side_done) MOEI_HIP(hipEventSynchronize(c->ev_side));
            side_done = true;
            const int n_pf = c->pin->n_list[0] < n_pf_copy ? c->pin->n_list[0] : n_pf_copy;
            const int n_ev_all = c->pin->n_list[1] < n_ev_copy ? c->pin->n_list[1] : n_ev_copy;
            c->pf_gate_recorded = true;
            rc = moei_cache_prefetch(c, c->pin->pf_head, n_pf, c->pin->ev_head, n_ev_all, c->pin_V, c->pf_depth, protect,
                                     k, c->last_pf_fid, c->last_pf_victim, nullptr, &c->last_n_pf, s);
            c->pf_gate_recorded = false;
            if (rc) return rc;
        } else {
            c->last_n_pf = 0;
        }
        if (h_topk_idx) memcpy(h_topk_idx, c->pin->idx, (size_t)k * 4);
        if (h_n_miss) *h_n_miss = n_miss;
        if (h_best) {
            if (!side_done) {  // only the matched trace is needed: it is announced by the step's number
                volatile int32_t* ps = &c->pin->best_seq;
                const int32_t want = c->step_seq;
                const bool seen = c->poll && poll_pinned([&] { return *ps == want; }, kPollLimitUs);
                if (!seen) MOEI_HIP(hipEventSynchronize(c->ev_side));
            }
            *h_best = c->pin->best;
        }
    }
    return MOEI_OK;
}

extern "C" int moei_cache_last_heads(moei_cache* c, int32_t* h_pf_head, int32_t cap_pf, int32_t* h_n_pf_head,
                                     int32_t* h_ev_head, int32_t cap_ev, int32_t* h_n_ev_head, void* stream) {
    MOEI_REQUIRE(c && h_n_pf_head && h_n_ev_head, "moei_cache_last_heads: null pointer");
    MOEI_HIP(hipStreamSynchronize(as_stream(stream)));
    MOEI_HIP(hipStreamSynchronize(c->side_stream));
    int32_t n_pf = 0, n_ev = 0;
    MOEI_HIP(hipMemcpy(&n_pf, c->d_n_pf, 4, hipMemcpyDeviceToHost));
    MOEI_HIP(hipMemcpy(&n_ev, c->d_n_ev, 4, hipMemcpyDeviceToHost));
    const int h_pf = c->last_h_pf < n_pf ? c->last_h_pf : n_pf;
    const int h_ev = c->last_h_ev < n_ev ? c->last_h_ev : n_ev;
    if (h_pf > cap_pf || h_ev > cap_ev)
        MOEI_FAIL(MOEI_ECAPACITY, "moei_cache_last_heads: room for %d / %d entries, %d / %d needed", cap_pf, cap_ev, h_pf, h_ev);
    MOEI_REQUIRE((h_pf == 0 || h_pf_head) && (h_ev == 0 || h_ev_head), "moei_cache_last_heads: null pointer");
    if (h_pf > 0) MOEI_HIP(hipMemcpy(h_pf_head, c->d_pf_head, (size_t)h_pf * 4, hipMemcpyDeviceToHost));
    if (h_ev > 0) MOEI_HIP(hipMemcpy(h_ev_head, c->d_ev_head, (size_t)h_ev * 4, hipMemcpyDeviceToHost));
    *h_n_pf_head = h_pf;
    *h_n_ev_head = h_ev;
    return MOEI_OK;
}

extern "C" int moei_cache_last_prefetch(moei_cache* c, int32_t* h_fids, int32_t* h_victims, int32_t cap, int32_t* h_n) {
    MOEI_REQUIRE(c && h_n, "moei_cache_last_prefetch: null pointer");
    MOEI_REQUIRE(cap >= c->last_n_pf, "moei_cache_last_prefetch: room for %d entries, %d needed", cap, c->last_n_pf);
    if (h_fids) memcpy(h_fids, c->last_pf_fid, (size_t)c->last_n_pf * 4);
    if (h_victims) memcpy(h_victims, c->last_pf_victim, (size_t)c->last_n_pf * 4);
    *h_n = c->last_n_pf;
    return MOEI_OK;
}

extern "C" int moei_cache_set_match_count(moei_cache* c, int32_t m) {
    MOEI_REQUIRE(c, "moei_cache_set_match_count: null pointer");
    MOEI_REQUIRE(m >= 1 && m <= kMaxMatchBatch, "moei_cache_set_match_count: m = %d outside [1, %d]", m, kMaxMatchBatch);
    c->match_m = m;
    return MOEI_OK;
}

extern "C" int moei_cache_last_matches(moei_cache* c, int32_t* h_top, float* h_top_sim, int32_t cap, int32_t* h_m,
                                       void* stream) {
    MOEI_REQUIRE(c && h_m, "moei_cache_last_matches: null pointer");
    MOEI_REQUIRE(cap >= c->match_m, "moei_cache_last_matches: room for %d entries, %d needed", cap, c->match_m);
    MOEI_HIP(hipStreamSynchronize(as_stream(stream)));
    MOEI_HIP(hipStreamSynchronize(c->side_stream));
    if (h_top) MOEI_HIP(hipMemcpy(h_top, c->d_best, (size_t)c->match_m * 4, hipMemcpyDeviceToHost));
    if (h_top_sim) MOEI_HIP(hipMemcpy(h_top_sim, c->d_best_sim, (size_t)c->match_m * 4, hipMemcpyDeviceToHost));
    *h_m = c->match_m;
    return MOEI_OK;
}

extern "C" int moei_cache_join(moei_cache* c, void* stream) {
    MOEI_REQUIRE(c, "moei_cache_join: null pointer");
    if (c->plan_pending) {  // the prefetches the last asynchronous step planned are issued now
        int rc = flush_prefetch_plan(c, as_stream(stream));
        if (rc) return rc;
    }
    if (c->side_pending) MOEI_HIP(hipStreamWaitEvent(as_stream(stream), c->ev_side, 0));
    if (c->n_pending > 0) {  // prefetch copies that no stream has waited for yet
        for (int t = 0; t < c->S; ++t) {
            int rc = settle_pending(c, t, as_stream(stream));
            if (rc) return rc;
        }
    }
    return MOEI_OK;
}

extern "C" int moei_cache_sync(moei_cache* c) {
    MOEI_REQUIRE(c, "moei_cache_sync: null pointer");
    MOEI_HIP(hipStreamSynchronize(c->side_stream));
    MOEI_HIP(hipStreamSynchronize(c->copy_stream));
    MOEI_HIP(hipStreamSynchronize(c->pf_stream));
    std::fill(c->slot_pending.begin(), c->slot_pending.end(), 0);
    c->n_pending = 0;
    c->side_pending = false;
    for (int r = 0; r < kRing; ++r) c->match_pending[r] = false;
    return MOEI_OK;
}

extern "C" int moei_cache_last_step(moei_cache* c, float* h_gate_w, float* h_best_sim, float* h_prefetch,
                                    float* h_evict, int32_t* h_pf_order, int32_t* h_n_pf, int32_t* h_ev_order,
                                    int32_t* h_n_ev, void* stream) {
    MOEI_REQUIRE(c, "moei_cache_last_step: null pointer");
    MOEI_HIP(hipStreamSynchronize(as_stream(stream)));
    MOEI_HIP(hipStreamSynchronize(c->side_stream));
    if (h_pf_order || h_ev_order) {  // the step selected the heads only: the complete orders are ranked from its keys now
        int rc = launch_priority_rank(c->d, c->d_keys, c->d_n_pf, c->d_n_ev, c->d_pf_order, c->d_ev_order, c->side_stream);
        if (rc) return rc;
        MOEI_HIP(hipStreamSynchronize(c->side_stream));
    }
    const size_t LE = (size_t)c->d.L * c->d.E;
    if (h_gate_w) MOEI_HIP(hipMemcpy(h_gate_w, c->d_w, (size_t)c->d.k * 4, hipMemcpyDeviceToHost));
    if (h_best_sim) MOEI_HIP(hipMemcpy(h_best_sim, c->d_best_sim, 4, hipMemcpyDeviceToHost));
    if (h_prefetch) MOEI_HIP(hipMemcpy(h_prefetch, c->d_P, LE * 4, hipMemcpyDeviceToHost));
    if (h_evict) MOEI_HIP(hipMemcpy(h_evict, c->d_V, LE * 4, hipMemcpyDeviceToHost));
    if (h_pf_order) MOEI_HIP(hipMemcpy(h_pf_order, c->d_pf_order, LE * 4, hipMemcpyDeviceToHost));
    if (h_n_pf) MOEI_HIP(hipMemcpy(h_n_pf, c->d_n_pf, 4, hipMemcpyDeviceToHost));
    if (h_ev_order) MOEI_HIP(hipMemcpy(h_ev_order, c->d_ev_order, LE * 4, hipMemcpyDeviceToHost));
    if (h_n_ev) MOEI_HIP(hipMemcpy(h_n_ev, c->d_n_ev, 4, hipMemcpyDeviceToHost));
    return MOEI_OK;
}
