// Step 1 and 2 of the layer step: router GEMV, softmax + top-k, EAM update.
//
// Every token goes to k of a layer's E experts (Sec. 2 of the paper); each such pick
// adds one to the request's Expert Activation Matrix (Sec. 4.3).  One wavefront serves
// one token: the E logits sit in LDS and every expert's rank is counted against them.
#include <type_traits>

#include "kernels.hpp"
#include "topk.hpp"
#include "wtypes.hpp"

namespace moei {

namespace {

constexpr int kMaxE = 4096;

__global__ void __launch_bounds__(kWave) route_topk_kernel(const float* __restrict__ logits, int E, int k,
                                                           int renorm, int32_t* __restrict__ idx,
                                                           float* __restrict__ w) {
    extern __shared__ float z[];
    __shared__ int s_idx[kWave];
    __shared__ float s_w[kWave];
    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    for (int e = lane; e < E; e += kWave) z[e] = logits[(size_t)b * E + e];
    __syncthreads();
    int my_idx;
    float my_w;
    if (wave_logits_bad(z, E, lane)) {  // uniform: no picks for this token
        my_idx = -1;
        my_w = 0.f;
    } else if (E <= kRankMaxE) {
        wave_topk_rank(z, E, k, renorm, lane, s_idx, s_w);
        __syncthreads();
        my_idx = lane < k ? s_idx[lane] : -1;
        my_w = lane < k ? s_w[lane] : 0.f;
    } else {
        wave_topk(z, E, k, renorm, lane, my_idx, my_w);
    }
    if (lane < k) {
        idx[(size_t)b * k + lane] = my_idx;
        w[(size_t)b * k + lane] = my_w;
    }
}

// k > 64: serial rounds writing straight to memory (rare: k is 1..8 in practice).
__global__ void __launch_bounds__(kWave) route_topk_wide_kernel(const float* __restrict__ logits, int E, int k,
                                                                int renorm, int32_t* __restrict__ idx,
                                                                float* __restrict__ w) {
    extern __shared__ float z[];
    const int b = blockIdx.x;
    const int lane = threadIdx.x;
    for (int e = lane; e < E; e += kWave) z[e] = logits[(size_t)b * E + e];
    __syncthreads();
    if (wave_logits_bad(z, E, lane)) {  // uniform: no picks for this token
        for (int j = lane; j < k; j += kWave) {
            idx[(size_t)b * k + j] = -1;
            w[(size_t)b * k + j] = 0.f;
        }
        return;
    }
    const int per = (E + kWave - 1) / kWave;
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
        if ((c.e & (kWave - 1)) == lane) taken |= 1ull << (c.e / kWave);
        float p = expf(c.v - m) / s;
        sel_sum += p;
        if (lane == 0) {
            idx[(size_t)b * k + j] = c.e;
            w[(size_t)b * k + j] = p;
        }
    }
    if (renorm) {
        __syncthreads();
        for (int j = lane; j < k; j += kWave) w[(size_t)b * k + j] = w[(size_t)b * k + j] / sel_sum;
    }
}

__global__ void eam_update_kernel(int32_t* __restrict__ eam, int B, int L, int E, int layer,
                                  const int32_t* __restrict__ idx, int k) {
    int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t >= B * k) return;
    int b = t / k;
    int e = idx[t];
    // picks of one token are distinct and every token has its own matrix: no two
    // threads touch the same cell
    if (e >= 0 && e < E) eam[((size_t)b * L + layer) * E + e] += 1;
}

// Routing of the fused layer step for one token in ONE launch: a wavefront per expert
// forms logit = <W_r[e], x> + b_e; the last workgroup to finish (arrival counter) then takes
// the top-k, updates the EAM row and writes the slot ids / gate weights the FFN reads.
constexpr int kRouteWaves = 4;  // expert rows per workgroup: fewer workgroups, fewer device-scope fences
template <typename WT>
__global__ void __launch_bounds__(kRouteWaves * kWave) route_fused_kernel(RouteFusedArgs a) {
    using V = WVec<WT>;
    extern __shared__ float z[];  // E logits, then E slot ids, the E counts of this layer's EAM row, 4 x E partial ranks
    __shared__ unsigned s_ticket;
    __shared__ int s_pick[kWave];
    __shared__ float s_pw[kWave];
    int* s_slot = reinterpret_cast<int*>(z + a.E);
    int* s_eam = s_slot + a.E;
    int* s_prank = s_eam + a.E;
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    constexpr int NT = kRouteWaves * kWave;
    const int e = blockIdx.x * kRouteWaves + wv;
    int32_t* eam_row = a.eam + (size_t)a.layer * a.E;
    // Everything this workgroup reads before the arrival counter is requested at once, the router row
    // and the token first (a wavefront's loads complete in issue order, and the logit is what the
    // other workgroups wait for); one trip to the cache instead of three.
    constexpr int CW = kWave * V::N;
    const WT* row = reinterpret_cast<const WT*>(a.W) + (size_t)(e < a.E ? e : 0) * a.H;
    const WT* x = reinterpret_cast<const WT*>(a.x);
    const bool one_round = a.vec_ok && a.H <= 4 * CW;  // the whole row in four chunk loads per lane
    typename V::raw wr[4], xv[4];
    if (one_round) {
        const int c0 = lane * V::N;
        const int cin = c0 < a.H ? c0 : 0;  // rows shorter than 64 vectors: the lanes past the end read the start
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int c = c0 + q * CW < a.H ? c0 + q * CW : cin;
            wr[q] = V::load(row + c);
            xv[q] = V::load(x + c);
        }
    }
    // any workgroup may turn out to be the last: each fetches the layer's slot row and EAM row
    // now, so that nothing but the logits is left to load after the arrival counter
    const int j0 = tid < a.E ? tid : 0;
    const int slot0 = a.slot_of_row[j0], eam0 = eam_row[j0];
    // every workgroup copies its share of the EAM into the snapshot the match will read
    // (this step's k increments are added to the snapshot by the last workgroup)
    const int seg = (a.LE + (int)gridDim.x - 1) / (int)gridDim.x;
    const int i0 = blockIdx.x * seg + tid, i1 = min(a.LE, ((int)blockIdx.x + 1) * seg);
    const int snap0 = a.eam[i0 < a.LE ? i0 : 0];
    float acc = 0.f;
    if (e < a.E) {  // uniform over the wavefront
        if (one_round) {
            const int c0 = lane * V::N;
#pragma unroll
            for (int q = 0; q < 4; ++q) {  // the sum runs over the chunks in ascending order
                if (c0 + q * CW < a.H) {
                    float xf[V::N];
                    V::unpack(xv[q], xf);
                    acc = V::dot(wr[q], xf, acc);
                }
            }
        } else if (a.vec_ok) {
            // longer rows: ten chunk loads go out together (one round trip for 5,120 bf16 values)
            constexpr int NQ = 10;
            for (int c0 = lane * V::N; c0 < a.H; c0 += NQ * CW) {
                typename V::raw wr10[NQ], xv10[NQ];
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    const int c = c0 + q * CW < a.H ? c0 + q * CW : c0;
                    wr10[q] = V::load(row + c);
                    xv10[q] = V::load(x + c);
                }
#pragma unroll
                for (int q = 0; q < NQ; ++q) {
                    if (c0 + q * CW < a.H) {
                        float xf[V::N];
                        V::unpack(xv10[q], xf);
                        acc = V::dot(wr10[q], xf, acc);
                    }
                }
            }
        } else {
            for (int c = lane; c < a.H; c += kWave) acc = __builtin_fmaf(V::one(row + c), V::one(x + c), acc);
        }
        acc = wave_sum_dpp(acc);
        if (lane == 0) a.logits[e] = acc + (a.bias ? a.bias[e] : 0.f);
    }
    if (tid < a.E) {
        s_slot[tid] = slot0;
        s_eam[tid] = eam0;
    }
    for (int j = tid + NT; j < a.E; j += NT) {
        s_slot[j] = a.slot_of_row[j];
        s_eam[j] = eam_row[j];
    }
    if (i0 < i1) a.snap[i0] = snap0;
    for (int i = i0 + NT; i < i1; i += NT) a.snap[i] = a.eam[i];
    __syncthreads();
    if (tid == 0) {
        // release by the fence, then a relaxed arrival count (an acquire-release read-modify-write
        // would repeat the cache write-back and add an invalidate); only the last workgroup to
        // arrive needs the acquire, which is the fence below
        __threadfence();
        s_ticket = __hip_atomic_fetch_add(a.ticket, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    __syncthreads();
    if (s_ticket != gridDim.x - 1) return;
    if (tid == 0) __threadfence();
    __syncthreads();
    for (int j = tid; j < a.E; j += NT)
        z[j] = __hip_atomic_load(&a.logits[j], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    // every expert's rank is a count over all experts: each of the four wavefronts counts over a quarter
    // of them (at 160 experts the loop of one wavefront alone took as long as the rest of the kernel)
    const bool by_rank = a.E <= kRankMaxE;
    if (by_rank) {
        const int q = (a.E + kRouteWaves - 1) / kRouteWaves;
        rank_part(z, a.E, lane, min(a.E, wv * q), min(a.E, (wv + 1) * q), s_prank + wv * a.E);
        __syncthreads();
    }
    if (wv != 0) return;
    int my_idx;
    float my_w;
    const bool bad = wave_logits_bad(z, a.E, lane);  // uniform
    if (bad) {
        // no softmax exists: the token gets no picks, the EAM stays as it is, the FFN sees slot -1
        // (which contributes nothing) and the flag tells the host
        my_idx = -1;
        my_w = 0.f;
        if (lane == 0 && a.flags) atomicOr(a.flags, 4);
    } else if (by_rank) {
        const float sel = wave_topk_rank(z, a.E, a.k, a.renorm, lane, s_pick, s_pw, false, s_prank, kRouteWaves);
        __builtin_amdgcn_fence(__ATOMIC_ACQ_REL, "wavefront");
        __builtin_amdgcn_wave_barrier();
        my_idx = lane < a.k ? s_pick[lane] : -1;
        my_w = lane < a.k ? (a.renorm ? s_pw[lane] / sel : s_pw[lane]) : 0.f;
    } else {
        wave_topk(z, a.E, a.k, a.renorm, lane, my_idx, my_w);
    }
    // the synchronous step reads the picks on the host: they go straight into pinned host memory (what a
    // kernel has written there is visible to the host once the kernel has completed), no copy behind the kernel
    if (lane < a.k && a.host_idx) a.host_idx[lane] = bad ? -1 : my_idx;
    if (lane < a.k && bad) {
        a.idx[lane] = -1;
        a.w[lane] = 0.f;
        a.slot_ids[a.n_shared + lane] = -1;
        a.gate[a.n_shared + lane] = 0.f;
    } else if (lane < a.k) {
        a.idx[lane] = my_idx;
        a.w[lane] = my_w;
        const int cnt = s_eam[my_idx] + 1;  // one writer per cell
        eam_row[my_idx] = cnt;
        a.snap[(size_t)a.layer * a.E + my_idx] = cnt;
        // activated experts of the step: the always-on shared experts first, then the picks
        int slot = s_slot[my_idx];
        a.slot_ids[a.n_shared + lane] = slot;
        a.gate[a.n_shared + lane] = my_w;
        if (slot < 0 && a.flags) atomicOr(a.flags, 2);
    } else if (lane < a.k + a.n_shared) {
        a.slot_ids[lane - a.k] = a.shared_base + (lane - a.k);
        a.gate[lane - a.k] = 1.0f;
    }
    if (lane == 0) *a.ticket = 0;  // ready for the next launch on this stream
}

// Slot ids of already chosen picks (after the host has served the misses).
__global__ void gather_slots_kernel(const int32_t* __restrict__ idx, int k, const int32_t* __restrict__ slot_of_row,
                                    int32_t* __restrict__ slot_ids, int32_t* __restrict__ flags) {
    int j = threadIdx.x;
    if (j < k) {
        int slot = slot_of_row[idx[j]];
        slot_ids[j] = slot;
        if (slot < 0) atomicOr(flags, 2);
    }
}

}  // namespace

int launch_route_fused(RouteFusedArgs a, int wdtype, hipStream_t s) {
    if (a.E > kMaxE || a.k > kWave || a.k + a.n_shared > kWave)
        MOEI_FAIL(MOEI_EINVAL, "fused routing needs E <= %d and k + n_shared <= %d", kMaxE, kWave);
    const int n = wdtype == MOEI_WDTYPE_BF16 ? 8 : 4;
    a.vec_ok = (a.H % n == 0) && ((uintptr_t)a.W % 16 == 0) && ((uintptr_t)a.x % 16 == 0);
    if (wdtype == MOEI_WDTYPE_BF16)
        launch(K_ROUTE_TOPK, route_fused_kernel<uint16_t>, dim3((a.E + kRouteWaves - 1) / kRouteWaves), dim3(kRouteWaves * kWave),
               (3 + (a.E <= kRankMaxE ? kRouteWaves : 0)) * a.E * sizeof(float), s, a);
    else
        launch(K_ROUTE_TOPK, route_fused_kernel<float>, dim3((a.E + kRouteWaves - 1) / kRouteWaves), dim3(kRouteWaves * kWave),
               (3 + (a.E <= kRankMaxE ? kRouteWaves : 0)) * a.E * sizeof(float), s, a);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

int launch_gather_slots(const int32_t* d_idx, int k, const int32_t* d_slot_of_row, int32_t* d_slot_ids,
                        int32_t* d_flags, hipStream_t s) {
    launch(K_ROUTE_TOPK, gather_slots_kernel, dim3(1), dim3(kWave), 0, s, d_idx, k, d_slot_of_row, d_slot_ids, d_flags);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

}  // namespace moei

using namespace moei;

extern "C" int moe_route_topk(const float* d_logits, int32_t B, int32_t E, int32_t k, int32_t renorm, int32_t* d_idx,
                              float* d_w, void* stream) {
    MOEI_REQUIRE(B >= 0, "moe_route_topk: B = %d is negative", B);
    MOEI_REQUIRE(E >= 1 && E <= kMaxE, "moe_route_topk: E = %d outside [1, %d]", E, kMaxE);
    MOEI_REQUIRE(k >= 1 && k <= E, "moe_route_topk: k = %d outside [1, E = %d]", k, E);
    if (B == 0) return MOEI_OK;  // nothing to route: the (empty) buffers may be null
    MOEI_REQUIRE(d_logits && d_idx && d_w, "moe_route_topk: null pointer");
    hipStream_t s = as_stream(stream);
    launch(K_ROUTE_TOPK, k <= kWave ? route_topk_kernel : route_topk_wide_kernel, dim3(B), dim3(kWave),
           E * sizeof(float), s, d_logits, E, k, (int)(renorm != 0), d_idx, d_w);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}

extern "C" int eam_update(int32_t* d_eam, int32_t B, int32_t L, int32_t E, int32_t layer, const int32_t* d_idx,
                          int32_t k, void* stream) {
    MOEI_REQUIRE(B >= 0 && L >= 1 && E >= 1 && k >= 1 && k <= E, "eam_update: bad shape B=%d L=%d E=%d k=%d", B, L, E,
                 k);
    MOEI_REQUIRE(layer >= 0 && layer < L, "eam_update: layer %d outside [0, %d)", layer, L);
    if (B == 0) return MOEI_OK;
    MOEI_REQUIRE(d_eam && d_idx, "eam_update: null pointer");
    int n = B * k;
    launch(K_ROUTE_TOPK, eam_update_kernel, dim3((n + 255) / 256), dim3(256), 0, as_stream(stream), d_eam, B, L, E, layer,
           d_idx, k);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}
