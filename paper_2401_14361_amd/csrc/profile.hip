// Per-launch start/stop events for the library's kernels (diagnostic; see moei.h).
#include <vector>

#include "common.hpp"

namespace moei {

bool g_prof_on = false;

namespace {

struct Sample {
    int id;
    hipEvent_t b, e;
};
std::vector<Sample> g_pool;  // pre-created events: nothing is allocated inside a timed region
size_t g_used = 0;

const char* const kNames[K_COUNT] = {
    "route_topk_kernel", "eamc_dot_kernel",   "eamc_pick_kernel", "priority_score_kernel",
    "priority_rank_kernel", "ffn_fused_kernel", "ffn_reduce_kernel", "prefill_group_kernels",
    "prefill_route_kernel", "prefill_gateup_kernel", "prefill_down_kernel", "prefill_reduce_kernel",
};

void drop_pool() {
    for (auto& s : g_pool) {
        (void)hipEventDestroy(s.b);
        (void)hipEventDestroy(s.e);
    }
    g_pool.clear();
    g_used = 0;
}

}  // namespace

bool prof_take(int id, hipEvent_t* start, hipEvent_t* stop) {
    if (g_used >= g_pool.size()) return false;
    Sample& s = g_pool[g_used++];
    s.id = id;
    *start = s.b;
    *stop = s.e;
    return true;
}

}  // namespace moei

using namespace moei;

extern "C" int moei_profile_enable(int32_t max_samples) {
    MOEI_REQUIRE(max_samples >= 1 && max_samples <= (1 << 22), "moei_profile_enable: max_samples = %d outside [1, 2^22]",
                 max_samples);
    g_prof_on = false;
    MOEI_HIP(hipDeviceSynchronize());
    drop_pool();
    g_pool.reserve(max_samples);
    for (int i = 0; i < max_samples; ++i) {
        Sample s{-1, nullptr, nullptr};
        MOEI_HIP(hipEventCreate(&s.b));
        hipError_t e = hipEventCreate(&s.e);
        if (e != hipSuccess) {
            (void)hipEventDestroy(s.b);
            MOEI_FAIL(MOEI_EHIP, "hipEventCreate failed: %s", hipGetErrorString(e));
        }
        g_pool.push_back(s);
    }
    g_prof_on = true;
    return MOEI_OK;
}

extern "C" int moei_profile_disable(void) {
    g_prof_on = false;
    (void)hipDeviceSynchronize();
    drop_pool();
    return MOEI_OK;
}

extern "C" int moei_profile_kernels(void) { return K_COUNT; }

extern "C" const char* moei_profile_kernel_name(int32_t id) { return (id >= 0 && id < K_COUNT) ? kNames[id] : ""; }

extern "C" int moei_profile_read(int32_t id, double* total_ms, int32_t* count) {
    MOEI_REQUIRE(total_ms && count, "moei_profile_read: null pointer");
    MOEI_REQUIRE(id >= 0 && id < K_COUNT, "moei_profile_read: kernel id %d outside [0, %d)", id, (int)K_COUNT);
    MOEI_HIP(hipDeviceSynchronize());
    double t = 0.0;
    int n = 0;
    for (size_t i = 0; i < g_used; ++i) {
        if (g_pool[i].id != id) continue;
        float ms = 0.f;
        MOEI_HIP(hipEventElapsedTime(&ms, g_pool[i].b, g_pool[i].e));
        t += ms;
        ++n;
    }
    *total_ms = t;
    *count = n;
    return MOEI_OK;
}

extern "C" int moei_profile_samples(int32_t id, float* h_ms, int32_t cap, int32_t* count) {
    MOEI_REQUIRE(count, "moei_profile_samples: null pointer");
    MOEI_REQUIRE(id >= 0 && id < K_COUNT, "moei_profile_samples: kernel id %d outside [0, %d)", id, (int)K_COUNT);
    MOEI_REQUIRE(cap >= 0 && (cap == 0 || h_ms), "moei_profile_samples: bad buffer");
    MOEI_HIP(hipDeviceSynchronize());
    int n = 0;
    for (size_t i = 0; i < g_used; ++i) {
        if (g_pool[i].id != id) continue;
        if (n < cap) MOEI_HIP(hipEventElapsedTime(&h_ms[n], g_pool[i].b, g_pool[i].e));
        ++n;
    }
    *count = n;
    return MOEI_OK;
}
