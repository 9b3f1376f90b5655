// Step 5 of the layer step: the activated experts' FFN as ONE streaming pass over
// their cache slots.
//
// An expert is a feed-forward network (Sec. 2 of the paper); here in SwiGLU form,
//   o = W_down ( silu(W_gate x) * (W_up x) ),  y = sum_e w_e o_e.
// At batch 1 this is one flop per weight byte, so the only thing that matters is how
// the weight bytes stream out of HBM.  A slot stores an expert row-interleaved,
//   for i in 0..I-1:  W_gate[i][0..H) | W_up[i][0..H) | W_down[0..H)[i]
// (the down projection transposed), so that everything intermediate unit i needs is
// one contiguous run of 3*H values.  A wavefront takes such a run, forms the two dot
// products with x (held in LDS as fp32), reduces them over its 64 lanes, and adds
// a_i * W_down[:, i] into a running y kept in registers: no intermediate vector ever
// leaves the CU and each weight byte is read exactly once.  Work is dealt out
// statically (unit t goes to wavefront t mod W), one workgroup per compute unit, so
// the summation order - and with it every output bit - is the same on every run.
// Workgroup partial sums are added in index order by a small second kernel.
#include <stdlib.h>
#include <string.h>

#include <type_traits>

#include "kernels.hpp"
#include "wtypes.hpp"

namespace moei {

namespace {

struct FfnArgs {
    const void* pool;
    size_t slot_elems;
    int n_slots_total;
    const int32_t* slot_ids;
    const float* gate_w;
    const void* x;
    float* part;  // [gridDim.x][H] workgroup partial sums
    int H, I, n_act;
    int waves;    // wavefronts per workgroup
    int ygroup;   // wavefronts whose y rows fit in LDS together
    int32_t* flags;
};

__device__ __forceinline__ float silu(float g) { return g / (1.0f + expf(-g)); }

// Adds the wavefronts' y rows in wavefront order and writes the workgroup's partial row.
// Rows go through LDS `ygroup` at a time; `store_my_row` writes the calling wavefront's.
template <typename Store>
__device__ __forceinline__ void block_sum_rows(float* yp, int H, int waves, int ygroup, int wv, float* out,
                                               Store store_my_row) {
    const int tid = threadIdx.x, nthr = blockDim.x;
    for (int g0 = 0; g0 < waves; g0 += ygroup) {
        if (wv >= g0 && wv < g0 + ygroup) store_my_row(yp + (size_t)(wv - g0) * H);
        __syncthreads();
        const int ng = min(ygroup, waves - g0);
        for (int c = tid; c < H; c += nthr) {
            float s = g0 == 0 ? 0.f : out[c];  // each column is owned by one thread across rounds
            for (int k = 0; k < ng; ++k) s += yp[(size_t)k * H + c];
            out[c] = s;
        }
        __syncthreads();
    }
}

// Fast path: H is NCH chunks of 64 lanes x 16 bytes, so unit i is a run of 3*NCH
// 16-byte loads per lane (gate and up chunks interleaved, then the down chunks).  The
// wavefront keeps a rolling window of PF loads in flight: each step consumes the oldest
// load and issues the one PF steps ahead, across unit boundaries, so its stream never
// drains.  grid = one workgroup per compute unit, block = waves * 64 threads,
// LDS = x (H floats) + ygroup y rows.
template <int NCH>
struct StreamShape {
    static constexpr int kSteps = 3 * NCH;
    // window depth: all steps of a unit if they are at most 16, else half of them if that is at most 12
    // (15 loads in flight for rows of 10 chunks left no registers: 3 spills), else a third
    static constexpr int kWindow = kSteps <= 16 ? kSteps : (kSteps / 2 <= 12 && kSteps % 2 == 0 ? kSteps / 2 : kSteps / 3);
    // register budget: window + y accumulators decide how many wavefronts fit a SIMD
    static constexpr int kMaxWaves = NCH <= 4 ? 16 : (NCH <= 10 ? 12 : 8);
};

template <typename WT, int NCH>
__global__ void __launch_bounds__((StreamShape<NCH>::kMaxWaves * kWave)) ffn_fused_kernel(FfnArgs a) {
    using V = WVec<WT>;
    using Raw = typename V::raw;
    constexpr int N = V::N;
    constexpr int CW = kWave * N;  // columns per chunk
    constexpr int STEPS = StreamShape<NCH>::kSteps;
    constexpr int PF = StreamShape<NCH>::kWindow;
    static_assert(STEPS % PF == 0, "the window must divide the steps of a unit");
    extern __shared__ __align__(16) float smem[];
    float* xs = smem;
    float* yp = smem + a.H;
    constexpr bool kPacked = std::is_same<WT, uint16_t>::value;  // bf16: x stays bf16 in LDS, products by v_dot2c_f32_bf16
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    // the wavefront index in a scalar register: unit ids, slot ids and base addresses are
    // then scalar too
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int H = a.H, I = a.I;
    const int W = gridDim.x * a.waves;
    const int NT = a.n_act * I;
    const WT* pool = reinterpret_cast<const WT*>(a.pool);
    const unsigned lane_off = (unsigned)lane * N;  // this lane's elements inside a chunk
    int* s_slot = reinterpret_cast<int*>(yp);      // slot ids and gate weights of the call, staged
    float* s_gate = yp + 64;                       // in LDS (the y rows are not in use before the end)

    auto scalar = [](size_t v) -> size_t {
        uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
        uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
        return (size_t)(((uint64_t)hi << 32) | lo);
    };
    // element offset of unit t in the pool; a bad slot id reads slot 0 and is weighted by zero
    auto unit_off = [&](int slot, int i, bool& ok) -> size_t {
        ok = slot >= 0 && slot < a.n_slots_total;
        if (!ok && lane == 0) atomicOr(a.flags, 1);
        return scalar((size_t)(ok ? slot : 0) * a.slot_elems + (size_t)i * 3 * H);
    };
    // element offset of load step s inside a unit: g0 u0 g1 u1 ... then d0 d1 ...
    auto step_off = [&](int s) -> int {
        return s < 2 * NCH ? ((s & 1) ? H : 0) + (s >> 1) * CW : 2 * H + (s - 2 * NCH) * CW;
    };
    auto ld = [&](size_t unit, int off) -> Raw { return V::load_once(pool + unit + off + lane_off); };

    float acc[NCH * N];
#pragma unroll
    for (int k = 0; k < NCH * N; ++k) acc[k] = 0.f;
    Raw win[PF];

    // unit t -> wavefront t mod W, numbered wavefront-major (w = wv * workgroups + workgroup): when
    // the units do not fill the last round, every compute unit keeps most of its wavefronts busy
    // instead of whole workgroups running out of work
    int t = wv * gridDim.x + blockIdx.x;
    float gate = 0.f, gate_n = 0.f;
    bool ok = false, ok_n = false;
    size_t p = 0;
    // A wavefront's loads complete in issue order, so what is staged into LDS is requested BEFORE the
    // first window: its data is then there after one trip to the cache, the wavefront starts on the
    // window's first load as soon as that one arrives and refills from then on.  Requested behind the
    // window it would arrive after the window's last load, and until then no refill would be issued.
    constexpr int kXRounds = (NCH + 3) / 4;  // x is NCH x 64 pieces of 16 bytes, a workgroup has at least 256 threads
    static_assert(kXRounds <= 4, "four named registers sets hold the token");
    // (named variables, not an array: an array indexed in two loops is kept in scratch memory here)
    uint4 xv0 = make_uint4(0u, 0u, 0u, 0u), xv1 = xv0, xv2 = xv0, xv3 = xv0;
    if constexpr (kPacked) {
        // a piece past the row is read as the row's last one (and not stored)
        auto piece = [&](int u) { return reinterpret_cast<const uint4*>(a.x)[min(tid + u * (int)blockDim.x, NCH * kWave - 1)]; };
        xv0 = piece(0);
        if constexpr (kXRounds > 1) xv1 = piece(1);
        if constexpr (kXRounds > 2) xv2 = piece(2);
        if constexpr (kXRounds > 3) xv3 = piece(3);
    }
    const int act = min(tid, a.n_act - 1);
    const int my_slot = a.slot_ids[act];
    const float my_gate = a.gate_w[act];
    {  // the first window is on its way while x is staged; a wavefront without units reads the pool's
       // first unit instead, so that there is one path and the wait counts stay exact
        const bool any = t < NT;
        const int e = any ? t / I : 0;
        const int slot0 = a.slot_ids[e];
        gate = a.gate_w[e];
        if (any) p = unit_off(slot0, t - e * I, ok);
#pragma unroll
        for (int s = 0; s < PF; ++s) win[s] = ld(p, step_off(s));
    }
    if constexpr (kPacked) {
        uint4* dst = reinterpret_cast<uint4*>(xs);
        auto put = [&](int u, uint4 v) {
            const int c = tid + u * (int)blockDim.x;
            if (c < NCH * kWave) dst[c] = v;
        };
        put(0, xv0);
        if constexpr (kXRounds > 1) put(1, xv1);
        if constexpr (kXRounds > 2) put(2, xv2);
        if constexpr (kXRounds > 3) put(3, xv3);
    } else {
        stage_as_f32(reinterpret_cast<const WT*>(a.x), xs, H);
    }
    if (tid < a.n_act) {
        s_slot[tid] = my_slot;
        s_gate[tid] = my_gate;
    }
    __syncthreads();

    while (t < NT) {
        const int tn = t + W;
        const bool more = tn < NT;
        size_t pn = p;
        if (more) {
            const int e = tn / I;
            pn = unit_off(s_slot[e], tn - e * I, ok_n);
            gate_n = s_gate[e];
        }
        float g = 0.f, u = 0.f, ai = 0.f;
        float xf[N];
        uint4 xp = make_uint4(0u, 0u, 0u, 0u);
#pragma unroll
        for (int s = 0; s < STEPS; ++s) {
            const Raw cur = win[s % PF];
            if (s < 2 * NCH) {
                if constexpr (kPacked) {
                    if ((s & 1) == 0) xp = reinterpret_cast<const uint4*>(xs)[(s >> 1) * kWave + lane];
                    if ((s & 1) == 0)
                        g = V::dot_packed(cur, xp, g);
                    else
                        u = V::dot_packed(cur, xp, u);
                } else {
                    if ((s & 1) == 0) {
#pragma unroll
                        for (int k = 0; k < N; k += 4)
                            *reinterpret_cast<float4*>(xf + k) =
                                *reinterpret_cast<const float4*>(xs + (s >> 1) * CW + lane * N + k);
                        g = V::dot(cur, xf, g);
                    } else {
                        u = V::dot(cur, xf, u);
                    }
                }
            } else {
                if (s == 2 * NCH) {
                    g = wave_sum_dpp(g);
                    u = wave_sum_dpp(u);
                    ai = ok ? silu(g) * u * gate : 0.f;
                }
                float d[N];
                V::unpack(cur, d);
#pragma unroll
                for (int k = 0; k < N; ++k)
                    acc[(s - 2 * NCH) * N + k] = __builtin_fmaf(ai, d[k], acc[(s - 2 * NCH) * N + k]);
            }
            // The consumed slot is free again: refill it with the load PF steps ahead.  After
            // the last unit the refills read the pool's first chunk (the same kilobyte for every
            // wavefront, so it comes from the cache), so that every step issues exactly one load
            // and the loop body has no branch.  The scheduling barriers keep the compiler from
            // hoisting refills and growing the window.
            __builtin_amdgcn_sched_barrier(0);
            if (s + PF < STEPS)
                win[s % PF] = ld(p, step_off(s + PF));
            else
                win[s % PF] = ld(more ? pn : 0, more ? step_off(s + PF - STEPS) : 0);
            __builtin_amdgcn_sched_barrier(0);
        }
        t = tn;
        p = pn;
        gate = gate_n;
        ok = ok_n;
    }
    __syncthreads();  // the LDS behind the y rows held the slot ids until here
    float* out = a.part + (size_t)blockIdx.x * H;
    block_sum_rows(yp, H, a.waves, a.ygroup, wv, out, [&](float* row) {
#pragma unroll
        for (int c = 0; c < NCH; ++c)
#pragma unroll
            for (int k = 0; k < N; k += 4)
                *reinterpret_cast<float4*>(row + c * CW + lane * N + k) =
                    make_float4(acc[c * N + k], acc[c * N + k + 1], acc[c * N + k + 2], acc[c * N + k + 3]);
    });
}

// Any H: the same dealing of units to wavefronts, scalar loads, y rows accumulated in LDS.
template <typename WT>
__global__ void __launch_bounds__(1024) ffn_fused_generic_kernel(FfnArgs a) {
    using V = WVec<WT>;
    extern __shared__ __align__(16) float smem[];
    float* xs = smem;
    float* yp = smem + a.H;  // [waves][H]
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int H = a.H, I = a.I;
    const int W = gridDim.x * a.waves;
    const int NT = a.n_act * I;
    const WT* pool = reinterpret_cast<const WT*>(a.pool);
    float* my = yp + (size_t)wv * H;
    stage_as_f32(reinterpret_cast<const WT*>(a.x), xs, H);
    for (int c = lane; c < H; c += kWave) my[c] = 0.f;
    __syncthreads();
    for (int t = blockIdx.x * a.waves + wv; t < NT; t += W) {
        const int e = t / I, i = t - e * I;
        const int slot = a.slot_ids[e];
        if (slot < 0 || slot >= a.n_slots_total) {
            if (lane == 0) atomicOr(a.flags, 1);
            continue;
        }
        const WT* p = pool + (size_t)slot * a.slot_elems + (size_t)i * 3 * H;
        float g = 0.f, u = 0.f;
        for (int c = lane; c < H; c += kWave) {
            g = __builtin_fmaf(V::one(p + c), xs[c], g);
            u = __builtin_fmaf(V::one(p + H + c), xs[c], u);
        }
        g = wave_sum_dpp(g);
        u = wave_sum_dpp(u);
        const float ai = silu(g) * u * a.gate_w[e];
        for (int c = lane; c < H; c += kWave) my[c] = __builtin_fmaf(ai, V::one(p + 2 * H + c), my[c]);
    }
    __syncthreads();
    float* out = a.part + (size_t)blockIdx.x * H;
    for (int c = tid; c < H; c += blockDim.x) {
        float s = 0.f;
        for (int k = 0; k < a.waves; ++k) s += yp[(size_t)k * H + c];
        out[c] = s;
    }
}

// y[h] = sum of the n_part workgroup partials.  A workgroup owns 32 columns; its 256
// threads are 8 column quads x 32 slices of the partial list; every thread adds its
// slice in index order, then the 32 slice sums are added in slice order.
__global__ void __launch_bounds__(256) ffn_reduce_kernel(const float* __restrict__ part, int n_part, int H,
                                                         float* __restrict__ y) {
    __shared__ float s_sum[32][32];
    const int cq = threadIdx.x & 7, sl = threadIdx.x >> 3;
    const int h = blockIdx.x * 32 + cq * 4;
    const int per = (n_part + 31) / 32;
    const int p0 = sl * per, p1 = min(n_part, p0 + per);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    if (h + 3 < H) {
#pragma unroll 8
        for (int p = p0; p < p1; ++p) {
            const float4 v = *reinterpret_cast<const float4*>(part + (size_t)p * H + h);
            acc.x += v.x; acc.y += v.y; acc.z += v.z; acc.w += v.w;
        }
    } else {
        for (int p = p0; p < p1; ++p) {
            const float* r = part + (size_t)p * H;
            if (h < H) acc.x += r[h];
            if (h + 1 < H) acc.y += r[h + 1];
            if (h + 2 < H) acc.z += r[h + 2];
        }
    }
    s_sum[sl][cq * 4 + 0] = acc.x;
    s_sum[sl][cq * 4 + 1] = acc.y;
    s_sum[sl][cq * 4 + 2] = acc.z;
    s_sum[sl][cq * 4 + 3] = acc.w;
    __syncthreads();
    if (threadIdx.x < 32) {
        const int hh = blockIdx.x * 32 + threadIdx.x;
        float t = 0.f;
#pragma unroll
        for (int k = 0; k < 32; ++k) t += s_sum[k][threadIdx.x];
        if (hh < H) y[hh] = t;
    }
}

int env_int(const char* name, int dflt) {
    const char* v = getenv(name);
    if (!v || !*v) return dflt;
    return atoi(v);
}

int g_cus = 0;
int compute_units() {
    if (g_cus == 0) {
        int dev = 0, n = 0;
        if (hipGetDevice(&dev) != hipSuccess ||
            hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
            n = 256;
        g_cus = n;
    }
    return g_cus;
}

constexpr size_t kLdsBudget = 150 * 1024;  // of the 160 KiB per compute unit

// Wavefronts per workgroup: the count in [4, max_waves] that wastes the fewest unit slots when
// n_units are dealt out to blocks * waves wavefronts (ties go to more wavefronts).
int plan_waves(int n_units, int blocks, int max_waves) {
    static const int forced = env_int("MOEI_FFN_WAVES", 0);  // the environment is read once per process
    if (forced >= 1 && forced <= max_waves) return forced;
    // a layer step repeats the same shape call after call: the last plan is kept
    static int memo_key[3] = {-1, -1, -1}, memo_val = 0;
    if (memo_key[0] == n_units && memo_key[1] == blocks && memo_key[2] == max_waves) return memo_val;
    int best = max_waves;
    double best_eff = -1.0;
    for (int m = max_waves; m >= (max_waves < 4 ? 1 : 4); --m) {
        long per = ((long)n_units + (long)blocks * m - 1) / ((long)blocks * m);
        double eff = (double)n_units / ((double)per * blocks * m);
        if (eff > best_eff + 1e-9) {
            best_eff = eff;
            best = m;
        }
    }
    memo_key[0] = n_units;
    memo_key[1] = blocks;
    memo_key[2] = max_waves;
    memo_val = best;
    return best;
}

// Raises a kernel's dynamic-LDS limit above 64 KiB, once per kernel and size (the call
// is not a stream operation, so it stays out of the per-launch path and of captures).
template <typename K>
int allow_big_lds(K kernel, size_t bytes) {
    static const void* seen_fn[64];
    static size_t seen_bytes[64];
    static int n_seen = 0;
    if (bytes <= 64 * 1024) return MOEI_OK;
    const void* fn = reinterpret_cast<const void*>(kernel);
    for (int i = 0; i < n_seen; ++i)
        if (seen_fn[i] == fn && seen_bytes[i] >= bytes) return MOEI_OK;
    MOEI_HIP(hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes));
    if (n_seen < 64) {
        seen_fn[n_seen] = fn;
        seen_bytes[n_seen++] = bytes;
    }
    return MOEI_OK;
}

template <typename WT>
int launch_ffn_typed(FfnArgs a, bool fast, int grid, float* d_y, hipStream_t s) {
    using V = WVec<WT>;
    const int H = a.H;
    int rc = MOEI_OK;
    const int nch = H / (kWave * V::N);
    const size_t row = (size_t)H * sizeof(float);
    if (fast) {
#define MOEI_FFN_CASE(N_)                                                                            \
    case N_: {                                                                                       \
        a.waves = plan_waves(a.n_act * a.I, grid, StreamShape<N_>::kMaxWaves);                       \
        int yg = (int)((kLdsBudget - row) / row);                                                    \
        a.ygroup = yg < 1 ? 1 : (yg > a.waves ? a.waves : yg);                                       \
        const size_t smem = row * (1 + a.ygroup);                                                    \
        rc = allow_big_lds(ffn_fused_kernel<WT, N_>, smem);                                          \
        if (rc) return rc;                                                                           \
        launch(K_FFN_FUSED, ffn_fused_kernel<WT, N_>, dim3(grid), dim3(a.waves * kWave), smem, s, a); \
        break;                                                                                       \
    }
        switch (nch) {
            MOEI_FFN_CASE(1)
            MOEI_FFN_CASE(2)
            MOEI_FFN_CASE(3)
            MOEI_FFN_CASE(4)
            MOEI_FFN_CASE(5)
            MOEI_FFN_CASE(6)
            MOEI_FFN_CASE(8)
            MOEI_FFN_CASE(10)
            MOEI_FFN_CASE(12)
            MOEI_FFN_CASE(16)
            default:
                fast = false;
        }
#undef MOEI_FFN_CASE
    }
    if (!fast) {
        int m = (int)((kLdsBudget - row) / row);
        if (m > 8) m = 8;
        if (m < 1) MOEI_FAIL(MOEI_ECAPACITY, "expert_ffn_gemv: H = %d does not fit the LDS staging", H);
        a.waves = m;
        a.ygroup = m;
        const size_t smem = row * (1 + m);
        rc = allow_big_lds(ffn_fused_generic_kernel<WT>, smem);
        if (rc) return rc;
        launch(K_FFN_FUSED, ffn_fused_generic_kernel<WT>, dim3(grid), dim3(m * kWave), smem, s, a);
    }
    MOEI_LAUNCH_CHECK();
    launch(K_FFN_REDUCE, ffn_reduce_kernel, dim3((H + 31) / 32), dim3(256), 0, s, (const float*)a.part, grid, H, d_y);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}


// ------------------------------------------------------------------ decode batch B > 1
// Tokens are grouped per activated expert; an "item" is one expert with up to kMaxGroup of its
// tokens, so the expert's weights are streamed once per item.  The items' intermediate units
// are split evenly over the workgroups as contiguous ranges.  A wavefront streams a unit once
// and uses it for every token of the item; y accumulators exist per token.
constexpr int kMaxGroup = 4;
constexpr int kGroupedWaves = 8;
constexpr int kMaxBatch = 16;

struct GroupItem {
    int32_t slot;
    int32_t ntok;
    int32_t tok[kMaxGroup];
    float w[kMaxGroup];
};

struct GroupArgs {
    const int32_t* idx;          // [B][k] picks
    const float* w;              // [B][k] gate weights
    const int32_t* slot_of_row;  // slot_of + layer*E
    int B, k, E, n_shared, shared_base, tb;
    GroupItem* items;
    int32_t* n_items;
    int32_t* flags;
};

// The item list of a call, built by every workgroup for itself (the picks of a batch are a few
// hundred bytes, the list a few kilobytes of LDS; a launch of its own would cost more than all
// workgroups repeating it).  The tokens routed to an expert, in token order, are cut into items of
// at most tb tokens; item positions follow expert order, the shared experts last.  The work is
// spread over the picks: the thread of pick p counts the earlier picks of the same expert (its
// rank there), LDS counters give every expert its number of tokens, a scan over the experts gives
// each its first item, and the thread then writes its token into place.  All threads of the
// workgroup call (at least 256 of them); with `publish` the list also goes to global memory for
// the reduction kernel and a pick that is not resident raises its flag.  Returns the item count
// (in every thread).  E <= 256 (checked by the host).
struct ItemScratch {
    int cnt[256];    // tokens routed to the expert
    int start[256];  // its first item
    int slot[256];   // its slot, -1: not resident
    int wsum[4];
};

__device__ __forceinline__ int build_items(const GroupArgs& a, GroupItem* s_items, int* s_pick, ItemScratch* sc,
                                           bool publish) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const int n_pick = a.B * a.k;
    float* s_pickw = reinterpret_cast<float*>(s_pick + n_pick);
    for (int p = tid; p < n_pick; p += blockDim.x) {
        int e = a.idx[p];
        if (e < 0 || e >= a.E) e = -1;  // a token without picks (no softmax exists for its logits)
        s_pick[p] = e;
        s_pickw[p] = a.w[p];
    }
    if (tid < 256) sc->cnt[tid] = 0;
    __syncthreads();
    // rank of every pick among the picks of its expert; tokens per expert
    int my_rank[2] = {0, 0};  // a thread takes at most two picks (16 tokens x k picks over >= 256 threads)
    int my_n = 0;
    for (int p = tid; p < n_pick && my_n < 2; p += blockDim.x, ++my_n) {
        const int e = s_pick[p];
        int r = 0;  // four picks per LDS read (the weights behind the picks make the last read safe)
        for (int q = 0; q < p; q += 4) {
            const int4 v = *reinterpret_cast<const int4*>(s_pick + q);
            r += (v.x == e) + ((q + 1 < p) & (v.y == e)) + ((q + 2 < p) & (v.z == e)) + ((q + 3 < p) & (v.w == e));
        }
        my_rank[my_n] = r;
        if (e >= 0) atomicAdd(&sc->cnt[e], 1);
    }
    __syncthreads();
    // items per expert, scanned over the experts
    int mine = 0;
    if (tid < 256) {
        int slot = -1, ntok = tid < a.E ? sc->cnt[tid] : 0;
        if (ntok > 0) {
            slot = a.slot_of_row[tid];
            if (slot < 0) {  // not resident: contributes nothing, flagged
                if (publish) atomicOr(a.flags, 2);
                ntok = 0;
            }
        }
        sc->slot[tid] = slot;
        mine = (ntok + a.tb - 1) / a.tb;
    }
    int incl = mine;
#pragma unroll
    for (int off = 1; off < kWave; off <<= 1) {
        const int up = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += up;
    }
    if (lane == kWave - 1 && wv < 4) sc->wsum[wv] = incl;
    __syncthreads();
    if (tid < 256) {
        int before = 0;
        for (int w = 0; w < wv; ++w) before += sc->wsum[w];
        sc->start[tid] = before + incl - mine;
    }
    int n = sc->wsum[0] + sc->wsum[1] + sc->wsum[2] + sc->wsum[3];
    __syncthreads();
    // every pick writes its token into its item; the first of an item also writes the item's head
    my_n = 0;
    for (int p = tid; p < n_pick && my_n < 2; p += blockDim.x, ++my_n) {
        const int e = s_pick[p];
        if (e < 0 || sc->slot[e] < 0) continue;
        const int r = my_rank[my_n];
        GroupItem* it = s_items + sc->start[e] + r / a.tb;
        const int pos = r % a.tb;
        it->tok[pos] = p / a.k;
        it->w[pos] = s_pickw[p];
        if (pos == 0) {
            const int ntok = min(a.tb, sc->cnt[e] - r);
            it->slot = sc->slot[e];
            it->ntok = ntok;
            for (int j = ntok; j < kMaxGroup; ++j) {
                it->tok[j] = 0;
                it->w[j] = 0.f;
            }
        }
    }
    const int tiles = (a.B + a.tb - 1) / a.tb;
    for (int q = tid; q < a.n_shared * tiles; q += blockDim.x) {
        const int sh = q / tiles, t0 = (q - sh * tiles) * a.tb;
        GroupItem it;
        it.slot = a.shared_base + sh;
        it.ntok = min(a.tb, a.B - t0);
        for (int j = 0; j < kMaxGroup; ++j) {
            it.tok[j] = j < it.ntok ? t0 + j : 0;
            it.w[j] = j < it.ntok ? 1.0f : 0.f;
        }
        s_items[n + q] = it;
    }
    n += a.n_shared * tiles;
    __syncthreads();
    if (publish) {
        for (int q = tid; q < n; q += blockDim.x) a.items[q] = s_items[q];
        if (tid == 0) *a.n_items = n;
    }
    return n;
}

struct GroupedFfnArgs {
    const void* pool;
    size_t slot_elems;
    GroupArgs grp;   // picks, gate weights, slot row; the item list goes to grp.items / grp.n_items
    int max_items;   // room in the LDS item list
    const void* x;  // [B][H]
    float* part;    // [workgroups][seg_max][TB][H]
    int H, I;
    int seg_max;
};

template <int NCH>
struct GroupedShape {
    static constexpr int kTB = NCH <= 4 ? 4 : 1;  // y accumulators per token must fit the register file
};

// The activated items' intermediate units form one row space of n_items * I rows; workgroup g
// takes the contiguous range [total*g/G, total*(g+1)/G).  A range crosses at most
// ceil(n_items / G) item boundaries, so it is cut into at most that many + 1 segments, each
// inside one item; a segment yields one partial y row per token of the item.
__device__ __host__ inline long grouped_range_begin(long total, int g, int G) { return total * g / G; }

__host__ inline int grouped_seg_max(int max_items, int G) { return (max_items + G - 1) / G + 1; }

template <typename WT, int NCH>
__global__ void __launch_bounds__((kGroupedWaves * kWave)) ffn_grouped_kernel(GroupedFfnArgs a) {
    using V = WVec<WT>;
    using Raw = typename V::raw;
    constexpr int N = V::N;
    constexpr int CW = kWave * N;
    constexpr int TB = GroupedShape<NCH>::kTB;
    constexpr int STEPS = StreamShape<NCH>::kSteps;
    constexpr int PF = StreamShape<NCH>::kWindow;
    extern __shared__ __align__(16) float smem[];
    __shared__ ItemScratch s_is;
    // [TB][H] inputs of the item's tokens: fp32 for fp32 weights; for bf16 weights the stored bf16 values
    // themselves, in the first half of each row, for the two-element dot products
    constexpr bool kPacked = std::is_same<WT, uint16_t>::value;
    float* xs = smem;
    float* yp = smem + TB * a.H;   // [kGroupedWaves][H] y rows of one token, one per wavefront
    GroupItem* s_items = reinterpret_cast<GroupItem*>(yp + (size_t)kGroupedWaves * a.H);  // [max_items]
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wv = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int H = a.H, I = a.I;
    const WT* pool = reinterpret_cast<const WT*>(a.pool);
    const unsigned lane_off = (unsigned)lane * N;
    int* s_pick = reinterpret_cast<int*>(s_items + a.max_items);  // [2][B*k]
    const int n_items = build_items(a.grp, s_items, s_pick, &s_is, blockIdx.x == 0);
    const long total = (long)n_items * I;
    const long R0 = grouped_range_begin(total, blockIdx.x, gridDim.x);
    const long R1 = grouped_range_begin(total, blockIdx.x + 1, gridDim.x);
    auto scalar = [](size_t v) -> size_t {
        uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)v);
        uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)((uint64_t)v >> 32));
        return (size_t)(((uint64_t)hi << 32) | lo);
    };
    auto step_off = [&](int s) -> int {
        return s < 2 * NCH ? ((s & 1) ? H : 0) + (s >> 1) * CW : 2 * H + (s - 2 * NCH) * CW;
    };
    auto ld = [&](size_t unit, int off) -> Raw { return V::load_once(pool + unit + off + lane_off); };

    int seg = 0;
    for (long row = R0; row < R1 && seg < a.seg_max; ++seg) {  // uniform over the workgroup
        const int item = (int)(row / I);
        const int r0 = (int)(row - (long)item * I);
        const int r1 = (int)min((long)I, r0 + (R1 - row));
        row += r1 - r0;
        const GroupItem it = s_items[item];
        // this wavefront's rows of the segment: r0 + wv, r0 + wv + 8, ...
        const int nr = (r1 - r0 - wv + kGroupedWaves - 1) / kGroupedWaves;  // may be <= 0
        const size_t row_stride = (size_t)kGroupedWaves * 3 * H;
        size_t p = scalar((size_t)it.slot * a.slot_elems + (size_t)(r0 + wv) * 3 * H);
        Raw win[PF];
        if (nr > 0) {  // the first window is on its way while the inputs are staged
#pragma unroll
            for (int s = 0; s < PF; ++s) win[s] = ld(p, step_off(s));
        }
        __syncthreads();  // the previous segment is done with xs and yp
        for (int j = 0; j < TB; ++j)
            if (j < it.ntok) {
                const WT* xsrc = reinterpret_cast<const WT*>(a.x) + (size_t)it.tok[j] * H;
                if constexpr (kPacked) {
                    uint4* dst = reinterpret_cast<uint4*>(xs + (size_t)j * H);
                    for (int c = tid; c < H / 8; c += kGroupedWaves * kWave) dst[c] = *reinterpret_cast<const uint4*>(xsrc + c * 8);
                } else {
                    stage_as_f32(xsrc, xs + (size_t)j * H, H);
                }
            }
        __syncthreads();
        float acc[TB][NCH * N];
#pragma unroll
        for (int j = 0; j < TB; ++j)
#pragma unroll
            for (int q = 0; q < NCH * N; ++q) acc[j][q] = 0.f;
        for (int r = 0; r < nr; ++r) {
            const bool more = r + 1 < nr;
            const size_t pn = more ? p + row_stride : p;
            float gs[TB], us[TB], ai[TB];
#pragma unroll
            for (int j = 0; j < TB; ++j) gs[j] = us[j] = ai[j] = 0.f;
#pragma unroll
            for (int s = 0; s < STEPS; ++s) {
                const Raw cur = win[s % PF];
                if (s < 2 * NCH) {
#pragma unroll
                    for (int j = 0; j < TB; ++j) {
                        if (j < it.ntok) {  // uniform
                            if constexpr (kPacked) {
                                const uint4 xp = reinterpret_cast<const uint4*>(xs + (size_t)j * H)[(s >> 1) * kWave + lane];
                                if ((s & 1) == 0)
                                    gs[j] = V::dot_packed(cur, xp, gs[j]);
                                else
                                    us[j] = V::dot_packed(cur, xp, us[j]);
                            } else {
                                float xf[N];
#pragma unroll
                                for (int t = 0; t < N; t += 4)
                                    *reinterpret_cast<float4*>(xf + t) = *reinterpret_cast<const float4*>(
                                        xs + (size_t)j * H + (s >> 1) * CW + lane * N + t);
                                if ((s & 1) == 0)
                                    gs[j] = V::dot(cur, xf, gs[j]);
                                else
                                    us[j] = V::dot(cur, xf, us[j]);
                            }
                        }
                    }
                } else {
                    if (s == 2 * NCH) {
#pragma unroll
                        for (int j = 0; j < TB; ++j)
                            if (j < it.ntok) ai[j] = silu(wave_sum_dpp(gs[j])) * wave_sum_dpp(us[j]) * it.w[j];
                    }
                    float df[N];
                    V::unpack(cur, df);
#pragma unroll
                    for (int j = 0; j < TB; ++j)
#pragma unroll
                        for (int t = 0; t < N; ++t)
                            acc[j][(s - 2 * NCH) * N + t] = __builtin_fmaf(ai[j], df[t], acc[j][(s - 2 * NCH) * N + t]);
                }
                __builtin_amdgcn_sched_barrier(0);
                if (s + PF < STEPS)
                    win[s % PF] = ld(p, step_off(s + PF));
                else
                    win[s % PF] = ld(more ? pn : 0, more ? step_off(s + PF - STEPS) : 0);
                __builtin_amdgcn_sched_barrier(0);
            }
            p = pn;
        }
        // the segment's partial row of every token of the item: wavefront rows added in order
#pragma unroll
        for (int j = 0; j < TB; ++j) {
            if (j < it.ntok) {  // uniform
                __syncthreads();
                float* rowp = yp + (size_t)wv * H;
#pragma unroll
                for (int q = 0; q < NCH; ++q)
#pragma unroll
                    for (int t = 0; t < N; t += 4)
                        *reinterpret_cast<float4*>(rowp + q * CW + lane * N + t) =
                            make_float4(acc[j][q * N + t], acc[j][q * N + t + 1], acc[j][q * N + t + 2],
                                        acc[j][q * N + t + 3]);
                __syncthreads();
                float* out = a.part + (((size_t)blockIdx.x * a.seg_max + seg) * TB + j) * H;
                for (int h = tid; h < H; h += kGroupedWaves * kWave) {
                    float s = 0.f;
#pragma unroll
                    for (int k = 0; k < kGroupedWaves; ++k) s += yp[(size_t)k * H + h];
                    out[h] = s;
                }
            }
        }
    }
}

// y[b][h] = sum of the partial rows of the segments whose item holds token b.  The workgroup
// first lists those rows in segment order (workgroup-major) in LDS; 32 slices of the list are
// then added by a thread each, all of a slice's loads in flight together, and the slice sums are
// added in slice order.  grid (H / 32, B), 256 threads = 32 slices x 8 float4 columns;
// dynamic LDS: 2 * n_blocks * seg_max ints.
__global__ void __launch_bounds__(256) ffn_grouped_reduce_kernel(const float* __restrict__ part,
                                                                 const GroupItem* __restrict__ items,
                                                                 const int32_t* __restrict__ n_items, int tb, int I,
                                                                 int H, int n_blocks, int seg_max,
                                                                 float* __restrict__ y) {
    extern __shared__ __align__(16) int32_t s_rows[];  // partial row of each segment for this token, or -1
    __shared__ float s_sum[32][32];
    __shared__ int s_wbase[4];
    __shared__ int s_nv;
    const int n = n_blocks * seg_max;
    int32_t* s_list = s_rows + n;  // the rows that exist, in segment order
    const int b = blockIdx.y, tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const long total = (long)*n_items * I;
    for (int g = tid; g < n_blocks; g += 256) {
        long row = grouped_range_begin(total, g, n_blocks);
        const long R1 = grouped_range_begin(total, g + 1, n_blocks);
        for (int seg = 0; seg < seg_max; ++seg) {
            int entry = -1;
            if (row < R1) {
                const int item = (int)(row / I);
                const int r0 = (int)(row - (long)item * I);
                row += min((long)I, r0 + (R1 - row)) - r0;
                for (int j = 0; j < items[item].ntok; ++j)
                    if (items[item].tok[j] == b) entry = (g * seg_max + seg) * tb + j;
            }
            s_rows[g * seg_max + seg] = entry;
        }
    }
    __syncthreads();
    // compaction in list order: ballots inside a wavefront, running offsets across wavefronts and rounds
    int base = 0;
    for (int e0 = 0; e0 < n; e0 += 256) {
        const int e = e0 + tid;
        const int r = e < n ? s_rows[e] : -1;
        const unsigned long long mask = __ballot(r >= 0);
        if (lane == 0) s_wbase[wv] = __popcll(mask);
        __syncthreads();
        int before = base;
        for (int w = 0; w < wv; ++w) before += s_wbase[w];
        if (r >= 0) s_list[before + __popcll(mask & ((1ull << lane) - 1ull))] = r;
        base += s_wbase[0] + s_wbase[1] + s_wbase[2] + s_wbase[3];
        __syncthreads();
    }
    if (tid == 0) s_nv = base;
    __syncthreads();
    const int nv = s_nv;
    const int cq = tid & 7, sl = tid >> 3;
    const int h = blockIdx.x * 32 + cq * 4;
    const int per = (nv + 31) / 32;
    const int p0 = sl * per, p1 = min(nv, p0 + per);
    float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
    for (int p = p0; p < p1; p += 8) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
            v[u] = p + u < p1 ? *reinterpret_cast<const float4*>(part + (size_t)s_list[p + u] * H + h)
                              : make_float4(0.f, 0.f, 0.f, 0.f);
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            acc.x += v[u].x;
            acc.y += v[u].y;
            acc.z += v[u].z;
            acc.w += v[u].w;
        }
    }
    s_sum[sl][cq * 4 + 0] = acc.x;
    s_sum[sl][cq * 4 + 1] = acc.y;
    s_sum[sl][cq * 4 + 2] = acc.z;
    s_sum[sl][cq * 4 + 3] = acc.w;
    __syncthreads();
    if (tid < 32) {
        float t = 0.f;
#pragma unroll
        for (int k2 = 0; k2 < 32; ++k2) t += s_sum[k2][tid];
        y[(size_t)b * H + blockIdx.x * 32 + tid] = t;
    }
}

}  // namespace

int ffn_scratch_alloc(const moei_model_desc& d, int n_act_max, FfnScratch* out) {
    out->n_act_max = n_act_max;
    // the streaming kernels take one workgroup per compute unit; some units are left to the
    // side stream's match and priority kernels so that these never hold up a streaming workgroup
    // (the stream is bound by HBM, not by the number of units: measured per layer step on the
    // 64-expert shape, 42.9 us with 8 units left free, 41.1 us with 24, 43.4 us with 64)
    int reserve = env_int("MOEI_RESERVE_CUS", 24);
    if (reserve < 0 || reserve > compute_units() / 2) reserve = 0;
    out->n_part = compute_units() - reserve;
    float* unused = nullptr;  // the static scratch of expert_ffn_gemv_static: address looked up at set-up
    int rc = static_part_ptr(&unused);
    if (rc) return rc;
    hipError_t e = hipMalloc((void**)&out->d_part, (size_t)out->n_part * d.H * sizeof(float));
    if (e != hipSuccess) {
        out->d_part = nullptr;
        MOEI_FAIL(MOEI_ENOMEM, "FFN scratch allocation failed: %s", hipGetErrorString(e));
    }
    return MOEI_OK;
}

void ffn_scratch_free(FfnScratch* s) {
    (void)hipFree(s->d_part);
    s->d_part = nullptr;
}

// ------------------------------------------------------------------ scratch that is never allocated
// The workgroup partial rows of expert_ffn_gemv_static live in this array: one copy per GPU that
// the library runs on, held until the process ends.  Host code never uses the array's name as an
// address: its device address is looked up once per device and kept in g_static_part.
}  // namespace moei

static __device__ __align__(256) float scratch[moei::kStaticPartFloats];

namespace moei {

namespace {
constexpr int kMaxDevices = 64;
float* g_static_part[kMaxDevices] = {};
}  // namespace

// Device address of the static partial-row array on the current device (looked up at the
// first call on that device: cache creation, else the entry point itself).
int static_part_ptr(float** out) {
    int dev = -1;
    MOEI_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) MOEI_FAIL(MOEI_EINVAL, "device ordinal %d outside [0, %d)", dev, kMaxDevices);
    if (!g_static_part[dev]) {
        float* ptr = nullptr;
        MOEI_HIP(hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)));
        if (!ptr) MOEI_FAIL(MOEI_EHIP, "the static scratch array has no device address");
        g_static_part[dev] = ptr;
    }
    *out = g_static_part[dev];
    return MOEI_OK;
}

int launch_expert_ffn_static(const moei_model_desc& d, const void* d_pool, size_t slot_elems, int n_slots_total,
                             int n_part, const int32_t* d_slot_ids, const float* d_gate_w, int n_act, const void* d_x,
                             float* d_y, int32_t* d_flags, hipStream_t s) {
    if ((size_t)n_part * (size_t)d.H > kStaticPartFloats)
        MOEI_FAIL(MOEI_ECAPACITY,
                  "expert_ffn_gemv_static: %d partial rows of H = %d floats exceed the static scratch of %zu floats "
                  "(H <= %zu on this device)",
                  n_part, d.H, kStaticPartFloats, kStaticPartFloats / (size_t)n_part);
    FfnScratch scr;
    int rc = static_part_ptr(&scr.d_part);
    if (rc) return rc;
    scr.n_part = n_part;
    return launch_expert_ffn(d, d_pool, slot_elems, n_slots_total, scr, d_slot_ids, d_gate_w, n_act, d_x, d_y, d_flags, s);
}

int launch_expert_ffn(const moei_model_desc& d, const void* d_pool, size_t slot_elems, int n_slots_total,
                      const FfnScratch& scr, const int32_t* d_slot_ids, const float* d_gate_w, int n_act,
                      const void* d_x, float* d_y, int32_t* d_flags, hipStream_t s) {
    if (n_act == 0) {  // an empty sum: the reduction over zero partial rows writes zeros
        launch(K_FFN_REDUCE, ffn_reduce_kernel, dim3((d.H + 31) / 32), dim3(256), 0, s, (const float*)scr.d_part, 0, d.H,
               d_y);
        MOEI_LAUNCH_CHECK();
        return MOEI_OK;
    }
    FfnArgs a{};
    a.pool = d_pool;
    a.slot_elems = slot_elems;
    a.n_slots_total = n_slots_total;
    a.slot_ids = d_slot_ids;
    a.gate_w = d_gate_w;
    a.x = d_x;
    a.part = scr.d_part;
    a.H = d.H;
    a.I = d.I;
    a.n_act = n_act;
    a.flags = d_flags;
    const int wb = d.wdtype == MOEI_WDTYPE_BF16 ? 2 : 4;
    const int n = 16 / wb;
    static const bool force_generic = env_int("MOEI_FFN_GENERIC", 0) != 0;
    const bool fast = (d.H % (kWave * n) == 0) && ((uintptr_t)d_pool % 16 == 0) && ((slot_elems * wb) % 16 == 0) &&
                      !force_generic;
    if (d.wdtype == MOEI_WDTYPE_BF16) return launch_ffn_typed<uint16_t>(a, fast, scr.n_part, d_y, s);
    return launch_ffn_typed<float>(a, fast, scr.n_part, d_y, s);
}


int grouped_max_items(const moei_model_desc& d) { return kMaxBatch * d.k + d.n_shared * kMaxBatch; }
size_t grouped_item_bytes() { return sizeof(GroupItem); }
size_t grouped_part_floats(const moei_model_desc& d) {
    const int G = compute_units();
    return (size_t)G * grouped_seg_max(grouped_max_items(d), G) * kMaxGroup * d.H;
}

namespace {
template <typename WT>
int launch_grouped_typed(const moei_model_desc& d, GroupedFfnArgs ga, int B, float* d_y, hipStream_t s) {
    using V = WVec<WT>;
    const int nch = d.H / (kWave * V::N);
    const int grid = compute_units();
    ga.seg_max = grouped_seg_max(grouped_max_items(d), grid);
    int rc;
#define MOEI_GROUPED_CASE(N_)                                                                           \
    case N_: {                                                                                          \
        ga.grp.tb = GroupedShape<N_>::kTB;                                                              \
        const size_t smem = (size_t)(GroupedShape<N_>::kTB + kGroupedWaves) * d.H * sizeof(float) +     \
                            (size_t)ga.max_items * sizeof(GroupItem) + (size_t)B * d.k * 8;             \
        if (smem > kLdsBudget) MOEI_FAIL(MOEI_ECAPACITY, "expert_ffn_grouped: H = %d does not fit the LDS staging", d.H); \
        rc = allow_big_lds(ffn_grouped_kernel<WT, N_>, smem);                                           \
        if (rc) return rc;                                                                              \
        launch(K_FFN_FUSED, ffn_grouped_kernel<WT, N_>, dim3(grid), dim3(kGroupedWaves * kWave), smem, s, ga); \
        MOEI_LAUNCH_CHECK();                                                                            \
        break;                                                                                          \
    }
    switch (nch) {
        MOEI_GROUPED_CASE(1)
        MOEI_GROUPED_CASE(2)
        MOEI_GROUPED_CASE(4)
        MOEI_GROUPED_CASE(8)
        MOEI_GROUPED_CASE(10)
        default:
            MOEI_FAIL(MOEI_EINVAL, "expert_ffn_grouped: H = %d is not supported (needs H / %d in {1,2,4,8,10})", d.H,
                      kWave * V::N);
    }
#undef MOEI_GROUPED_CASE
    launch(K_FFN_REDUCE, ffn_grouped_reduce_kernel, dim3(d.H / 32, B), dim3(256),
           (size_t)2 * grid * ga.seg_max * sizeof(int32_t), s, (const float*)ga.part, (const GroupItem*)ga.grp.items,
           (const int32_t*)ga.grp.n_items, ga.grp.tb, d.I, d.H, grid, ga.seg_max, d_y);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}
}  // namespace

int launch_expert_ffn_grouped(const moei_model_desc& d, const void* d_pool, size_t slot_elems, void* d_items,
                              int32_t* d_n_items, float* d_part, const int32_t* d_slot_of_row, int shared_base,
                              const int32_t* d_idx, const float* d_w, int B, const void* d_x, float* d_y,
                              int32_t* d_flags, hipStream_t s) {
    if (B > kMaxBatch) MOEI_FAIL(MOEI_EINVAL, "expert_ffn_grouped: B = %d exceeds %d", B, kMaxBatch);
    // the item list is built by a thread per pick and per expert of a 256-thread group
    if (d.E > 256 || B * d.k > 512)
        MOEI_FAIL(MOEI_EINVAL, "expert_ffn_grouped: E = %d, B * k = %d exceed 256 experts or 512 picks", d.E, B * d.k);
    const int wb = d.wdtype == MOEI_WDTYPE_BF16 ? 2 : 4;
    const int n = 16 / wb;
    if (d.H % (kWave * n) != 0 || (uintptr_t)d_pool % 16 != 0 || (slot_elems * wb) % 16 != 0)
        MOEI_FAIL(MOEI_EINVAL, "expert_ffn_grouped: H = %d must be a multiple of %d", d.H, kWave * n);
    GroupArgs gr{d_idx, d_w, d_slot_of_row, B, d.k, d.E, d.n_shared, shared_base, 0,
                 reinterpret_cast<GroupItem*>(d_items), d_n_items, d_flags};
    GroupedFfnArgs ga{d_pool, slot_elems, gr, grouped_max_items(d), d_x, d_part, d.H, d.I, 0};
    if (d.wdtype == MOEI_WDTYPE_BF16) return launch_grouped_typed<uint16_t>(d, ga, B, d_y, s);
    return launch_grouped_typed<float>(d, ga, B, d_y, s);
}

}  // namespace moei

using namespace moei;

// Slot layout from the three plain matrices (host memory, desc->wdtype elements).
extern "C" int moei_expert_pack(const moei_model_desc* desc, const void* h_gate, const void* h_up, const void* h_down,
                                void* h_slot) {
    MOEI_REQUIRE(desc && h_gate && h_up && h_down && h_slot, "moei_expert_pack: null pointer");
    int rc = check_desc(desc);
    if (rc) return rc;
    const size_t H = desc->H, I = desc->I;
    const size_t wb = desc->wdtype == MOEI_WDTYPE_BF16 ? 2 : 4;
    const unsigned char* g = static_cast<const unsigned char*>(h_gate);
    const unsigned char* u = static_cast<const unsigned char*>(h_up);
    const unsigned char* dn = static_cast<const unsigned char*>(h_down);
    unsigned char* out = static_cast<unsigned char*>(h_slot);
    for (size_t i = 0; i < I; ++i) {
        unsigned char* row = out + i * 3 * H * wb;
        memcpy(row, g + i * H * wb, H * wb);
        memcpy(row + H * wb, u + i * H * wb, H * wb);
        unsigned char* dcol = row + 2 * H * wb;
        if (wb == 2) {
            const uint16_t* src = reinterpret_cast<const uint16_t*>(dn) + i;
            uint16_t* dst = reinterpret_cast<uint16_t*>(dcol);
            for (size_t h = 0; h < H; ++h) dst[h] = src[h * I];
        } else {
            const uint32_t* src = reinterpret_cast<const uint32_t*>(dn) + i;
            uint32_t* dst = reinterpret_cast<uint32_t*>(dcol);
            for (size_t h = 0; h < H; ++h) dst[h] = src[h * I];
        }
    }
    return MOEI_OK;
}
