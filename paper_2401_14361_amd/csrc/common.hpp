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
    K_ROUTE_TOPK = 0,
    K_MATCH_DOT,
    K_MATCH_ARGMAX,
    K_PRIO_SCORE,
    K_PRIO_RANK,
    K_FFN_FUSED,
    K_FFN_REDUCE,
    K_FFN_GROUP,
    K_PF_ROUTE,
    K_PF_GATEUP,
    K_PF_DOWN,
    K_PF_REDUCE,
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

// The same reductions without LDS traffic: DPP inside each row of 16 lanes, then the four
// row results are read through scalar registers.  Every lane gets the result.
#define MOEI_DPP_F32(v, ctrl) \
    __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, (v)), (ctrl), 0xF, 0xF, false))
__device__ __forceinline__ float wave_sum_dpp(float v) {
    v += MOEI_DPP_F32(v, 0xB1);   // quad_perm [1,0,3,2]
    v += MOEI_DPP_F32(v, 0x4E);   // quad_perm [2,3,0,1]
    v += MOEI_DPP_F32(v, 0x141);  // row_half_mirror
    v += MOEI_DPP_F32(v, 0x140);  // row_mirror
    const int b = __builtin_bit_cast(int, v);
    float r = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    r += __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16));
    r += __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32));
    r += __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48));
    return r;
}
__device__ __forceinline__ float wave_max_dpp(float v) {
    v = fmaxf(v, MOEI_DPP_F32(v, 0xB1));
    v = fmaxf(v, MOEI_DPP_F32(v, 0x4E));
    v = fmaxf(v, MOEI_DPP_F32(v, 0x141));
    v = fmaxf(v, MOEI_DPP_F32(v, 0x140));
    const int b = __builtin_bit_cast(int, v);
    float r = __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 0));
    r = fmaxf(r, __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 16)));
    r = fmaxf(r, __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 32)));
    r = fmaxf(r, __builtin_bit_cast(float, __builtin_amdgcn_readlane(b, 48)));
    return r;
}

#define MOEI_DPP_U32(v, ctrl) ((unsigned)__builtin_amdgcn_update_dpp(0, (int)(v), (ctrl), 0xF, 0xF, false))
__device__ __forceinline__ unsigned wave_sum_u32_dpp(unsigned v) {
    v += MOEI_DPP_U32(v, 0xB1);
    v += MOEI_DPP_U32(v, 0x4E);
    v += MOEI_DPP_U32(v, 0x141);
    v += MOEI_DPP_U32(v, 0x140);
    return (unsigned)__builtin_amdgcn_readlane((int)v, 0) + (unsigned)__builtin_amdgcn_readlane((int)v, 16) +
           (unsigned)__builtin_amdgcn_readlane((int)v, 32) + (unsigned)__builtin_amdgcn_readlane((int)v, 48);
}
// Exact 64-bit sum over the wavefront: four 16-bit digits are summed separately (each digit
// sum stays below 2^22) and recombined.
__device__ __forceinline__ unsigned long long wave_sum_u64_dpp(unsigned long long v) {
    const unsigned long long d0 = wave_sum_u32_dpp((unsigned)(v & 0xffffu));
    const unsigned long long d1 = wave_sum_u32_dpp((unsigned)((v >> 16) & 0xffffu));
    const unsigned long long d2 = wave_sum_u32_dpp((unsigned)((v >> 32) & 0xffffu));
    const unsigned long long d3 = wave_sum_u32_dpp((unsigned)(v >> 48));
    return d0 + (d1 << 16) + (d2 << 32) + (d3 << 48);
}

// bf16 pair packed in a 32-bit word (element 0 in the low half) -> two fp32, exactly.
__device__ __forceinline__ float bf16_lo(uint32_t u) { return __uint_as_float(u << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t u) { return __uint_as_float(u & 0xffff0000u); }
__device__ __forceinline__ float bf16_one(uint16_t u) { return __uint_as_float(((uint32_t)u) << 16); }

// A 16-byte load per lane that goes from global memory straight into LDS: the wavefront's 64 pieces
// land side by side, 1 KiB from `lds_addr` on (an LDS byte address, the same in every lane).  The
// load counts as a vector memory operation of the wavefront (vmcnt); nothing says when the data is
// in LDS but a later wait on that counter.  m0 (the LDS base of such loads) is a register the
// compiler reserves and sets itself right before each of its own uses, so writing it here is safe.
__device__ __forceinline__ void load16_to_lds(const void* gsrc, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gsrc) : "memory");
}
__device__ __forceinline__ uint32_t lds_address(const void* p) {
    return (uint32_t)(uintptr_t)(__attribute__((address_space(3))) const void*)p;
}
// waits until at most N of the wavefront's vector memory operations are outstanding; no memory access of
// the program moves across it
template <int N>
__device__ __forceinline__ void wait_vm_fence() {
    static_assert(N >= 0 && N < 64, "vmcnt has six bits");
    asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// waits until the wavefront's LDS reads have returned (before their LDS is written again by such a load)
__device__ __forceinline__ void wait_lds_fence() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

#endif  // __HIPCC__

}  // namespace moei
