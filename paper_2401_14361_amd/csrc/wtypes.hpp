// 16-byte vector access to stored weights (fp32 or bf16 bit patterns) with fp32 maths.
#pragma once

#include "common.hpp"

namespace moei {

#if defined(__HIPCC__)

// A 16-byte load of data that is read once (expert weights, long trace scans): the
// non-temporal hint keeps such lines from displacing what the caches hold; measured on
// gfx950, a read-only stream of 12 KiB runs reaches 7.0 instead of 6.2 TB/s with it.
typedef unsigned int moei_u32x4 __attribute__((ext_vector_type(4)));
__device__ __forceinline__ uint4 load_once_16(const void* p) {
    const moei_u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const moei_u32x4*>(p));
    return make_uint4(v.x, v.y, v.z, v.w);
}

template <typename WT>
struct WVec;

template <>
struct WVec<float> {
    static constexpr int N = 4;  // elements per 16-byte load
    using raw = float4;
    static __device__ __forceinline__ raw load(const float* p) { return *reinterpret_cast<const float4*>(p); }
    static __device__ __forceinline__ raw load_once(const float* p) {
        const uint4 v = load_once_16(p);
        return make_float4(__uint_as_float(v.x), __uint_as_float(v.y), __uint_as_float(v.z), __uint_as_float(v.w));
    }
    static __device__ __forceinline__ raw zero() { return make_float4(0.f, 0.f, 0.f, 0.f); }
    // acc += sum_i w[i] * xf[i], in element order
    static __device__ __forceinline__ float dot(raw w, const float* xf, float acc) {
        acc = __builtin_fmaf(w.x, xf[0], acc);
        acc = __builtin_fmaf(w.y, xf[1], acc);
        acc = __builtin_fmaf(w.z, xf[2], acc);
        acc = __builtin_fmaf(w.w, xf[3], acc);
        return acc;
    }
    static __device__ __forceinline__ void unpack(raw w, float* f) {
        f[0] = w.x; f[1] = w.y; f[2] = w.z; f[3] = w.w;
    }
    static __device__ __forceinline__ float one(const float* p) { return *p; }
};

template <>
struct WVec<uint16_t> {
    static constexpr int N = 8;
    using raw = uint4;
    static __device__ __forceinline__ raw load(const uint16_t* p) { return *reinterpret_cast<const uint4*>(p); }
    static __device__ __forceinline__ raw load_once(const uint16_t* p) { return load_once_16(p); }
    static __device__ __forceinline__ raw zero() { return make_uint4(0u, 0u, 0u, 0u); }
    static __device__ __forceinline__ float dot(raw w, const float* xf, float acc) {
        acc = __builtin_fmaf(bf16_lo(w.x), xf[0], acc);
        acc = __builtin_fmaf(bf16_hi(w.x), xf[1], acc);
        acc = __builtin_fmaf(bf16_lo(w.y), xf[2], acc);
        acc = __builtin_fmaf(bf16_hi(w.y), xf[3], acc);
        acc = __builtin_fmaf(bf16_lo(w.z), xf[4], acc);
        acc = __builtin_fmaf(bf16_hi(w.z), xf[5], acc);
        acc = __builtin_fmaf(bf16_lo(w.w), xf[6], acc);
        acc = __builtin_fmaf(bf16_hi(w.w), xf[7], acc);
        return acc;
    }
    // acc += sum_i w[i] * x[i] with x given as eight bf16 values too: four two-element dot products
    // with fp32 accumulation (v_dot2c_f32_bf16), a quarter of the instructions of the form above
    static __device__ __forceinline__ float dot_packed(raw w, uint4 x, float acc) {
        typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.x), __builtin_bit_cast(bf16x2, x.x), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.y), __builtin_bit_cast(bf16x2, x.y), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.z), __builtin_bit_cast(bf16x2, x.z), acc, false);
        acc = __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2, w.w), __builtin_bit_cast(bf16x2, x.w), acc, false);
        return acc;
    }
    static __device__ __forceinline__ void unpack(raw w, float* f) {
        f[0] = bf16_lo(w.x); f[1] = bf16_hi(w.x);
        f[2] = bf16_lo(w.y); f[3] = bf16_hi(w.y);
        f[4] = bf16_lo(w.z); f[5] = bf16_hi(w.z);
        f[6] = bf16_lo(w.w); f[7] = bf16_hi(w.w);
    }
    static __device__ __forceinline__ float one(const uint16_t* p) { return bf16_one(*p); }
};

// Copies n stored values to fp32 (all threads of the block take part; caller syncs).
template <typename WT>
__device__ __forceinline__ void stage_as_f32(const WT* __restrict__ src, float* __restrict__ dst, int n,
                                             float scale = 1.0f) {
    for (int i = threadIdx.x; i < n; i += blockDim.x) dst[i] = WVec<WT>::one(src + i) * scale;
}

#endif

}  // namespace moei
