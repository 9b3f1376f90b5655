// Step 4 of the layer step: PredictEAM aggregation + prefetch / eviction priorities.
//
// Prefetch score (Sec. 4.5 of the paper): the matched EAM's cell, normalised over
// its row, times the layer-proximity factor (1 - (i - l)/L) for future layers i > l.
// Eviction score (Alg. 1): (cell + eps)(1 - i/L) / row sum, lowest score evicted
// first.  Both are evaluated as one fp64 division of exact products so that equal
// rationals give equal keys; the orders are then produced by rank counting over the
// compacted candidate lists (a candidate's rank is the number of candidates that
// sort before it; ties go to the lower flat id, so ranks are unique).
#include "kernels.hpp"

namespace moei {

namespace {

typedef unsigned long long u64;
constexpr int kScoreThreads = 1024;
constexpr int kRankThreads = 1024;
constexpr u64 kNone = ~0ull;

struct ScoreArgs {
    const void* traces;  // [L][n_cap][E]
    int cell_bytes, n_cap, N, L, E;
    const int32_t* best;  // [B]
    int B, cur_layer;
    const int32_t* slot_of;  // [L*E]
    double eps;
    const int32_t* cur_idx;  // [B*k] or null
    int n_cur;
    float* P;  // [L*E]
    float* V;  // [L*E]
    u64* keys;     // [2][L*E]: prefetch keys, eviction keys (compacted in place)
    int32_t* ids;  // [2][L*E]
    int32_t* n_pf;
    int32_t* n_ev;
};

__device__ __forceinline__ uint32_t cell_at(const void* traces, int cell_bytes, size_t i) {
    return cell_bytes == 4 ? (uint32_t) reinterpret_cast<const int32_t*>(traces)[i]
                           : (uint32_t) reinterpret_cast<const uint16_t*>(traces)[i];
}

// Exclusive scan of one flag per thread over the workgroup; returns the total too.
__device__ __forceinline__ int block_scan_flags(bool flag, int* s_wave, int& total) {
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    u64 m = __ballot(flag);
    int in_wave = __popcll(m & ((1ull << lane) - 1ull));
    if (lane == 0) s_wave[wv] = __popcll(m);
    __syncthreads();
    int before = 0, tot = 0;
    for (int i = 0; i < kScoreThreads / kWave; ++i) {
        int c = s_wave[i];
        if (i < wv) before += c;
        tot += c;
    }
    total = tot;
    __syncthreads();
    return before + in_wave;
}

__global__ void __launch_bounds__(kScoreThreads) priority_score_kernel(ScoreArgs a) {
    __shared__ int s_wave[kScoreThreads / kWave];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wv = tid / kWave;
    const int L = a.L, E = a.E, l = a.cur_layer;
    const size_t LE = (size_t)L * E;
    u64* kp = a.keys;
    u64* kv = a.keys + LE;

    // phase A: one wavefront per layer row
    for (int i = wv; i < L; i += kScoreThreads / kWave) {
        u64 rsum = 0;
        for (int j = lane; j < E; j += kWave) {
            u64 t = 0;
            for (int b = 0; b < a.B; ++b) {
                int n = a.best[b];
                if (n >= 0 && n < a.N) t += cell_at(a.traces, a.cell_bytes, ((size_t)i * a.n_cap + n) * E + j);
            }
            rsum += t;
        }
        const u64 R = wave_sum_u64(rsum);
        const double den = (double)(R ? R : 1ull) * (double)L;
        for (int j = lane; j < E; j += kWave) {
            u64 t = 0;
            for (int b = 0; b < a.B; ++b) {
                int n = a.best[b];
                if (n >= 0 && n < a.N) t += cell_at(a.traces, a.cell_bytes, ((size_t)i * a.n_cap + n) * E + j);
            }
            const size_t f = (size_t)i * E + j;
            const double td = (double)t;
            const double v = ((td + a.eps) * (double)(L - i)) / den;
            double p = 0.0;
            if (i > l && R > 0) p = (td * (double)(L - i + l)) / den;
            a.P[f] = (float)p;
            a.V[f] = (float)v;
            const int slot = a.slot_of[f];
            bool excluded = false;
            if (i == l)
                for (int m = 0; m < a.n_cur; ++m) excluded |= (a.cur_idx[m] == j);
            // positive doubles order like their bit patterns; ~bits turns descending into ascending
            kp[f] = (i > l && p > 0.0 && slot < 0) ? ~(u64)__double_as_longlong(p) : kNone;
            kv[f] = (slot >= 0 && !excluded) ? (u64)__double_as_longlong(v) : kNone;
        }
    }
    __syncthreads();

    // phase B: compact both candidate lists in flat-id order, in place
    for (int which = 0; which < 2; ++which) {
        u64* keys = which == 0 ? kp : kv;
        int32_t* ids = a.ids + (size_t)which * LE;
        int count = 0;
        for (size_t c0 = 0; c0 < LE; c0 += kScoreThreads) {
            const size_t f = c0 + tid;
            const u64 key = f < LE ? keys[f] : kNone;
            const bool flag = key != kNone;
            int total;
            const int pos = block_scan_flags(flag, s_wave, total);  // its barriers order reads before writes
            if (flag) {
                keys[count + pos] = key;
                ids[count + pos] = (int32_t)f;
            }
            count += total;
            __syncthreads();
        }
        if (tid == 0) *(which == 0 ? a.n_pf : a.n_ev) = count;
    }
}

// grid (ceil(L*E/64), 2).  A workgroup ranks 64 candidates (one per lane); its 16
// wavefronts each count over a slice of the list, then the counts are added up.
__global__ void __launch_bounds__(kRankThreads)
    priority_rank_kernel(const u64* __restrict__ keys_all, const int32_t* __restrict__ ids_all, size_t LE,
                         const int32_t* __restrict__ n_pf, const int32_t* __restrict__ n_ev,
                         int32_t* __restrict__ pf_order, int32_t* __restrict__ ev_order) {
    __shared__ int s_cnt[kRankThreads / kWave][kWave];
    const int which = blockIdx.y;
    const int n = which == 0 ? *n_pf : *n_ev;
    const int c0 = blockIdx.x * kWave;
    if (c0 >= n) return;  // uniform over the workgroup
    const u64* keys = keys_all + (size_t)which * LE;
    const int32_t* ids = ids_all + (size_t)which * LE;
    int32_t* order = which == 0 ? pf_order : ev_order;
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    constexpr int kW = kRankThreads / kWave;
    const int mine = c0 + lane;
    const u64 my_key = mine < n ? keys[mine] : 0;
    const int per = (n + kW - 1) / kW;
    const int g0 = wv * per;
    const int g1 = min(g0 + per, n);
    int cnt = 0;
    for (int g = g0; g < g1; ++g) {
        const u64 kg = keys[g];  // same address in every lane
        cnt += (kg < my_key || (kg == my_key && g < mine)) ? 1 : 0;
    }
    s_cnt[wv][lane] = cnt;
    __syncthreads();
    if (wv == 0 && mine < n) {
        int rank = 0;
        for (int i = 0; i < kW; ++i) rank += s_cnt[i][lane];
        order[rank] = ids[mine];
    }
}

}  // namespace

}  // namespace moei

using namespace moei;

extern "C" int expert_priority(const moei_eamc* c, const int32_t* d_best, int32_t B, int32_t cur_layer,
                               const int32_t* d_slot_of, float eps, const int32_t* d_cur_idx, int32_t k,
                               float* d_prefetch, float* d_evict, int32_t* d_pf_order, int32_t* d_n_pf,
                               int32_t* d_ev_order, int32_t* d_n_ev, void* stream) {
    MOEI_REQUIRE(c && d_best && d_slot_of && d_prefetch && d_evict && d_pf_order && d_n_pf && d_ev_order && d_n_ev,
                 "expert_priority: null pointer");
    MOEI_REQUIRE(B >= 1 && B <= kMaxMatchBatch, "expert_priority: B = %d outside [1, %d]", B, kMaxMatchBatch);
    MOEI_REQUIRE(cur_layer >= -1 && cur_layer < c->d.L, "expert_priority: cur_layer = %d outside [-1, %d)", cur_layer,
                 c->d.L);
    MOEI_REQUIRE(eps >= 0.f, "expert_priority: eps must not be negative");
    MOEI_REQUIRE(!d_cur_idx || (k >= 1 && k <= c->d.E), "expert_priority: k = %d outside [1, E]", k);
    hipStream_t s = as_stream(stream);
    const size_t LE = (size_t)c->d.L * c->d.E;
    ScoreArgs a{c->d_traces, c->cell_bytes, c->n_cap, c->N, c->d.L, c->d.E, d_best, B, cur_layer, d_slot_of,
                (double)eps, d_cur_idx, d_cur_idx ? B * k : 0, d_prefetch, d_evict, c->d_keys, c->d_ids, d_n_pf, d_n_ev};
    launch(K_PRIO_SCORE, priority_score_kernel, dim3(1), dim3(kScoreThreads), 0, s, a);
    MOEI_LAUNCH_CHECK();
    dim3 grid((unsigned)((LE + kWave - 1) / kWave), 2);
    launch(K_PRIO_RANK, priority_rank_kernel, grid, dim3(kRankThreads), 0, s, (const u64*)c->d_keys,
           (const int32_t*)c->d_ids, LE, (const int32_t*)d_n_pf, (const int32_t*)d_n_ev, d_pf_order, d_ev_order);
    MOEI_LAUNCH_CHECK();
    return MOEI_OK;
}
