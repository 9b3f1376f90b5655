// Scoring of every (layer, expert) cell from the matched traces: shared by the stand-alone
// priority kernel and by the match kernel's finishing workgroup (fused layer step).
#pragma once

#include "kernels.hpp"

namespace moei {

#if defined(__HIPCC__)

typedef unsigned long long u64;
constexpr int kScoreThreads = 1024;
constexpr u64 kNone = ~0ull;

struct ScoreArgs {
    const void* traces;  // [L][n_cap][E]
    int cell_bytes, n_cap, N, L, E;
    const int32_t* best;  // [B]
    int B, cur_layer;
    const int32_t* slot_of;  // [L*E]
    double eps;
    const int32_t* cur_idx;  // [n_cur] experts of the current layer that are about to run, or null
    int n_cur;
    float* P;  // [L*E]
    float* V;  // [L*E]
    u64* keys;     // [2][L*E]: prefetch keys, eviction keys; kNone = not a candidate
    int32_t* n_pf;
    int32_t* n_ev;
};

__device__ __forceinline__ uint32_t cell_at(const void* traces, int cell_bytes, size_t i) {
    return cell_bytes == 4 ? (uint32_t) reinterpret_cast<const int32_t*>(traces)[i]
                           : (uint32_t) reinterpret_cast<const uint16_t*>(traces)[i];
}

// Called by all kScoreThreads threads of ONE workgroup: scores for every cell, a 64-bit sort
// key per cell and list (kNone where the cell is not a candidate) and the two candidate
// counts.  One wavefront per layer row.  s_n[2] and s_best[kMaxMatchBatch] are LDS; with
// best_in_lds the caller has already put the matched trace indices (-1 = none) there.
__device__ __forceinline__ void score_cells(const ScoreArgs& a, int* s_n, int* s_best, bool best_in_lds) {
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1), wv = tid / kWave;
    const int L = a.L, E = a.E, l = a.cur_layer;
    const size_t LE = (size_t)L * E;
    u64* kp = a.keys;
    u64* kv = a.keys + LE;
    if (tid < 2) s_n[tid] = 0;
    if (!best_in_lds && tid < a.B) {
        const int n = a.best[tid];
        s_best[tid] = (n >= 0 && n < a.N) ? n : -1;
    }
    __syncthreads();
    constexpr int kPerLane = 4;  // cells of a row held in registers (rows up to 256 wide)
    int my_ev = 0, my_pf = 0;
    for (int i = wv; i < L; i += kScoreThreads / kWave) {
        // all of the row's loads go out together: matched cells, residency, current picks
        u64 tv[kPerLane];
        int sv[kPerLane];
        u64 rsum = 0;
        for (int r = 0; r * kWave < E; ++r) {
            const int j = lane + r * kWave;
            u64 t = 0;
            int slot = -1;
            if (j < E) {
                for (int b = 0; b < a.B; ++b) {
                    const int n = s_best[b];
                    if (n >= 0) t += cell_at(a.traces, a.cell_bytes, ((size_t)i * a.n_cap + n) * E + j);
                }
                if (r < kPerLane) slot = a.slot_of[(size_t)i * E + j];
            }
            if (r < kPerLane) {
                tv[r] = t;
                sv[r] = slot;
            }
            rsum += t;
        }
        int cur = -1;  // lane m holds pick m of the current layer (used for row l only)
        if (i == l && lane < a.n_cur) cur = a.cur_idx[lane];
        const u64 R = wave_sum_u64_dpp(rsum);
        const double den = (double)(R ? R : 1ull) * (double)L;
        for (int r = 0; r * kWave < E; ++r) {
            const int j = lane + r * kWave;
            u64 t = 0;
            int slot = -1;
            if (r < kPerLane) {
                t = tv[r];
                slot = sv[r];
            } else if (j < E) {
                for (int b = 0; b < a.B; ++b) {
                    const int n = s_best[b];
                    if (n >= 0) t += cell_at(a.traces, a.cell_bytes, ((size_t)i * a.n_cap + n) * E + j);
                }
                slot = a.slot_of[(size_t)i * E + j];
            }
            // is expert j one of the current picks?  (all 64 lanes take part in the shuffles)
            bool excluded = false;
            if (i == l) {
                for (int m0 = 0; m0 < a.n_cur; m0 += kWave) {
                    int c = cur;
                    if (m0 > 0) c = (m0 + lane < a.n_cur) ? a.cur_idx[m0 + lane] : -1;
                    const int lim = min(kWave, a.n_cur - m0);
                    for (int m = 0; m < lim; ++m) excluded |= (__shfl(c, m, kWave) == j);
                }
            }
            if (j >= E) continue;
            const size_t f = (size_t)i * E + j;
            const double td = (double)t;
            const double v = ((td + a.eps) * (double)(L - i)) / den;
            double p = 0.0;
            if (i > l && R > 0) p = (td * (double)(L - i + l)) / den;
            a.P[f] = (float)p;
            a.V[f] = (float)v;
            // positive doubles order like their bit patterns; ~bits turns descending into ascending
            const bool is_pf = i > l && p > 0.0 && slot < 0;
            const bool is_ev = slot >= 0 && !excluded;
            kp[f] = is_pf ? ~(u64)__double_as_longlong(p) : kNone;
            kv[f] = is_ev ? (u64)__double_as_longlong(v) : kNone;
            my_pf += is_pf;
            my_ev += is_ev;
        }
    }
    if (my_pf) atomicAdd(&s_n[0], my_pf);
    if (my_ev) atomicAdd(&s_n[1], my_ev);
    __syncthreads();
    if (tid == 0) {
        *a.n_pf = s_n[0];
        *a.n_ev = s_n[1];
    }
}


#endif

// priority.hip
ScoreArgs make_score_args(const moei_eamc* c, const int32_t* d_best, int B, int cur_layer, const int32_t* d_slot_of,
                          float eps, const int32_t* d_cur_idx, int n_cur, float* d_prefetch, float* d_evict,
                          int32_t* d_n_pf, int32_t* d_n_ev);
int launch_priority_rank(const moei_eamc* c, const int32_t* d_n_pf, const int32_t* d_n_ev, int32_t* d_pf_order,
                         int32_t* d_ev_order, hipStream_t s);
// match.hip: the match, and - if `score` is given (B must be 1) - the scoring of the matched
// trace by the workgroup that finishes the match, in the same launch
int launch_match(const moei_eamc* c, const int32_t* d_eam, int B, int layer_hi, int32_t* d_best, float* d_best_sim,
                 float* d_sims, const ScoreArgs* score, hipStream_t s);
// the m most similar traces of one query; `score` (with B = m) scores their aggregate
int launch_match_topm(const moei_eamc* c, const int32_t* d_eam, int layer_hi, int m, int32_t* d_top, float* d_top_sim,
                      float* d_sims, const ScoreArgs* score, hipStream_t s);

}  // namespace moei
