// Shared host/device helpers of the moei library (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>
#include <stdint.h>
#include <stdarg.h>
#include <stdio.h>

#include "moei.h"

namespace moei {

// ------------------------------------------------------------------ errors
void set_error(const char* fmt, ...) __attribute__((format(printf, 1, 2)));

#define MOEI_FAIL(code, ...)            \
    do {                                \
        ::moei::set_error(__VA_ARGS__); \
        return (code);                  \
    } while (0)

#define MOEI_REQUIRE(cond, ...)                      \
    do {                                             \
        if (!(cond)) MOEI_FAIL(MOEI_EINVAL, __VA_ARGS__); \
    } while (0)

#define MOEI_HIP(expr)                                                                   \
    do {                                                                                 \
        hipError_t e__ = (expr);                                                         \
        if (e__ != hipSuccess)                                                           \
            MOEI_FAIL(MOEI_EHIP, "%s failed: %s (%s:%d)", #expr, hipGetErrorString(e__), \
                      __FILE__, __LINE__);                                               \
    } while (0)

// A kernel launch is checked right after it is enqueued.
#define MOEI_LAUNCH_CHECK() MOEI_HIP(hipGetLastError())

int check_desc(const moei_model_desc* d);

static inline hipStream_t as_stream(void* s) { return reinterpret_cast<hipStream_t>(s); }

constexpr int kWave = 64;

// ------------------------------------------------------------------ kernel timing
// Optional per-launch start/stop events for every kernel of the library (see
// moei_profile_enable in moei.h).  Disabled: one predictable branch per launch.
enum KernelId {
    K_ROUTER_GEMV = 0,
    K_ROUTE_TOPK,
    K_MATCH_DOT,
    K_MATCH_ARGMAX,
    K_PRIO_SCORE,
    K_PRIO_RANK,
    K_FFN_FUSED,
    K_FFN_REDUCE,
    K_COUNT
};
extern bool g_prof_on;
// Hands out the next pre-created event pair for kernel `id`; false when the pool is used up.
bool prof_take(int id, hipEvent_t* start, hipEvent_t* stop);

// ------------------------------------------------------------------ device helpers
#if defined(__HIPCC__)

// Every kernel of the library is launched through here.  With timing enabled the
// launch carries a start/stop event pair that the runtime stamps with the kernel's own
// begin and end times (no extra packets between kernels).
template <typename... KArgs, typename... Args>
inline void launch(int id, void (*kernel)(KArgs...), dim3 grid, dim3 block, size_t smem, hipStream_t s,
                   Args... args) {
    hipEvent_t b = nullptr, e = nullptr;
    if (g_prof_on && prof_take(id, &b, &e))
        hipExtLaunchKernelGGL(kernel, grid, block, (uint32_t)smem, s, b, e, 0u, KArgs(args)...);
    else
        hipLaunchKernelGGL(kernel, grid, block, (uint32_t)smem, s, KArgs(args)...);
}

// Butterfly reductions over the 64 lanes of a wavefront; every lane ends with the result.
template <typename T>
__device__ __forceinline__ T wave_sum(T v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__device__ __forceinline__ unsigned long long wave_sum_u64(unsigned long long v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) {
        unsigned lo = __shfl_xor((unsigned)(v & 0xffffffffull), off, 64);
        unsigned hi = __shfl_xor((unsigned)(v >> 32), off, 64);
        v += ((unsigned long long)hi << 32) | lo;
    }
    return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, 64));
    return v;
}

// bf16 pair packed in a 32-bit word (element 0 in the low half) -> two fp32, exactly.
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ float bf16_one(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }

#endif  // __HIPCC__

}  // namespace moei
