// Softmax + top-k of one token's router logits by a single wavefront (Sec. 2 of the paper:
// every token goes to k of a layer's E experts).  Shared by the routing
// kernels and by the fused layer kernel.
#pragma once

#include "common.hpp"

namespace moei {

#if defined(__HIPCC__)

struct Cand {
    float v;
    int e;  // -1: none
};

__device__ __forceinline__ Cand better(Cand a, Cand b) {
    // larger logit first; equal logits go to the lower expert index
    if (b.e < 0) return a;
    if (a.e < 0) return b;
    if (a.v > b.v) return a;
    if (b.v > a.v) return b;
    return (a.e < b.e) ? a : b;
}

// Logits for which no softmax exists: a NaN anywhere, or no finite maximum (all -inf, or a +inf).
// Called by all 64 lanes of one wavefront; the answer is the same in every lane.  The routing
// kernels then give the token no picks (index -1, weight 0) instead of ranking garbage.
__device__ __forceinline__ bool wave_logits_bad(const float* z, int E, int lane) {
    bool nan = false;
    float m = -INFINITY;
    for (int e = lane; e < E; e += kWave) {
        const float v = z[e];
        nan |= (v != v);
        m = fmaxf(m, v);  // ignores a NaN operand
    }
    m = wave_max_dpp(m);
    return __ballot(nan) != 0ull || !(fabsf(m) < INFINITY);
}

// Softmax + top-k of z[0..E) (in LDS) by one wavefront, k <= 64.  Every expert's rank is
// the number of experts that come before it (larger logit, or equal logit and lower
// index), counted against broadcast LDS reads; rank r < k is pick r.  The picks land in
// s_idx[k] / s_w[k] (LDS); the caller reads them after a __syncthreads().
// With renorm the pick weights are divided by their sum: here if the calling wavefront is the
// whole workgroup (divide_here), else by the caller, after its own barrier, with the
// returned sum (valid in every lane).
constexpr int kRankMaxE = 1024;
// part_rank (or null): [n_part][E] counts in LDS, formed beforehand by n_part wavefronts, each over its
// own range of the experts (rank_part below): the rank is then their sum and the quadratic loop is
// shared by the workgroup.
// how many of z[j0..j1) come before (v, e): larger, or equal with a lower index.  The broadcast
// reads go out eight at a time, so that their latencies overlap, and the three comparisons are
// combined as bits: written with && and || they become a branch per element.
__device__ __forceinline__ int comes_before(float u, int j, float v, int e) {
    return (int)(u > v) | ((int)(u == v) & (int)(j < e));
}
__device__ __forceinline__ int count_before(const float* z, int j0, int j1, float v, int e) {
    int c = 0, j = j0;
    for (; j + 8 <= j1; j += 8) {
        float u[8];
#pragma unroll
        for (int q = 0; q < 8; ++q) u[q] = z[j + q];
#pragma unroll
        for (int q = 0; q < 8; ++q) c += comes_before(u[q], j + q, v, e);
    }
    for (; j < j1; ++j) c += comes_before(z[j], j, v, e);
    return c;
}
__device__ __forceinline__ void rank_part(const float* z, int E, int lane, int j0, int j1, int* out) {
    for (int e = lane; e < E; e += kWave) out[e] = count_before(z, j0, j1, z[e], e);
}
__device__ __forceinline__ float wave_topk_rank(const float* z, int E, int k, int renorm, int lane, int* s_idx,
                                                float* s_w, bool divide_here = true, const int* part_rank = nullptr,
                                                int n_part = 0) {
    const int per = (E + kWave - 1) / kWave;
    float m = -INFINITY;
    for (int r = 0; r < per; ++r) {
        int e = lane + r * kWave;
        if (e < E) m = fmaxf(m, z[e]);
    }
    m = wave_max_dpp(m);
    float s = 0.f;
    for (int r = 0; r < per; ++r) {
        int e = lane + r * kWave;
        if (e < E) s += expf(z[e] - m);
    }
    s = wave_sum_dpp(s);
    float sel = 0.f;
    for (int r = 0; r < per; ++r) {
        const int e = lane + r * kWave;
        if (e < E) {
            const float v = z[e];
            int rank = 0;
            if (part_rank) {
                for (int w = 0; w < n_part; ++w) rank += part_rank[w * E + e];
            } else {
                rank = count_before(z, 0, E, v, e);
            }
            if (rank < k) {
                const float p = expf(v - m) / s;
                s_idx[rank] = e;
                s_w[rank] = p;
                sel += p;
            }
        }
    }
    sel = wave_sum_dpp(sel);
    if (renorm && divide_here) {
        __syncthreads();  // single-wavefront workgroup: orders the LDS writes above with the reads below
        if (lane < k) s_w[lane] = s_w[lane] / sel;
    }
    return sel;
}

// The same by k rounds of a 64-lane butterfly arg-max (any E up to 4096).
// Lane j < k returns pick j in (idx, w); other lanes return idx = -1.
__device__ __forceinline__ void wave_topk(const float* z, int E, int k, int renorm, int lane, int& idx_out,
                                          float& w_out) {
    const int per = (E + kWave - 1) / kWave;  // <= 64, so one 64-bit mask per lane marks taken entries
    float m = -INFINITY;
    for (int r = 0; r < per; ++r) {
        int e = lane + r * kWave;
        if (e < E) m = fmaxf(m, z[e]);
    }
    m = wave_max(m);
    float s = 0.f;
    for (int r = 0; r < per; ++r) {
        int e = lane + r * kWave;
        if (e < E) s += expf(z[e] - m);
    }
    s = wave_sum(s);

    unsigned long long taken = 0ull;
    idx_out = -1;
    w_out = 0.f;
    float sel_sum = 0.f;
    for (int j = 0; j < k; ++j) {
        Cand c{0.f, -1};
        for (int r = 0; r < per; ++r) {
            int e = lane + r * kWave;
            if (e < E && !((taken >> r) & 1ull)) {
                float v = z[e];
                if (c.e < 0 || v > c.v) c = Cand{v, e};
            }
        }
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) {
            Cand o;
            o.v = __shfl_xor(c.v, off, 64);
            o.e = __shfl_xor(c.e, off, 64);
            c = better(c, o);
        }
        // c is now identical in all lanes; k <= E guarantees c.e >= 0
        if ((c.e & (kWave - 1)) == lane) taken |= 1ull << (c.e / kWave);
        float p = expf(c.v - m) / s;
        sel_sum += p;
        if (lane == j) {
            idx_out = c.e;
            w_out = p;
        }
    }
    if (renorm) w_out = w_out / sel_sum;
}

#endif

}  // namespace moei
