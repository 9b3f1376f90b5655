/*
 * cpu_step.c -- a plain CPU baseline of one MoE decode layer step, for timing.
 *
 * TEST / BENCHMARK INFRASTRUCTURE ONLY: the benchmark's CPU-baseline leg times it on the host
 * cores (one thread, then all of them) and a CPU test checks it against the Python oracle.  It
 * shares no code with the HIP sources or with moei_oracle.py: the same steps of the paper
 * (arXiv 2401.14361) written once more as scalar C loops -
 *   Sec. 2     router logits, softmax, the k most probable experts, gate weights
 *   Sec. 4.3   EAM update: M[l][j] += 1 per pick
 *   Sec. 4.5   cosine match of the flattened EAM against every stored trace (the paper runs this
 *              search on the CPU, App. B.1), best = largest similarity, ties to the lowest index
 *   Sec. 4.5 / Alg. 1   prefetch score T/R (1 - (i-l)/L) for future layers, eviction score
 *              (T + eps)(1 - i/L)/R, both orders
 *   Sec. 2     the activated experts' SwiGLU FFN, y = sum_e w_e W_down (silu(W_gate x) * (W_up x))
 * with OpenMP over traces (match) and over weight rows (FFN, router) and nothing else: no
 * blocking, no SIMD intrinsics, fp64 accumulation, integers in 64 bits.  Alg. 1's cache
 * bookkeeping is host logic in every implementation and is not part of this timing loop: the
 * caller passes the residency mask.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

static inline double elem(const void* p, size_t i, int bf16) {
    if (bf16) {
        uint32_t u = (uint32_t)((const uint16_t*)p)[i] << 16;
        float f;
        memcpy(&f, &u, 4);
        return (double)f;
    }
    return (double)((const float*)p)[i];
}

typedef unsigned __int128 u128;

/* is candidate a = (dot_a, nt_a) more similar than b?  sim^2 ~ dot^2 / nt with a common |q|;
 * exact in 128 bits for dot < 2^40, nt < 2^46 (checked by the caller) */
static inline int more_similar(uint64_t da, uint64_t na, uint64_t db, uint64_t nb) {
    if (na == 0) da = 0, na = 1;
    if (nb == 0) db = 0, nb = 1;
    u128 l = (u128)da * da * nb, r = (u128)db * db * na;
    return l > r;
}

typedef struct {
    double key;
    int32_t id;
} keyed;

static int by_key_then_id(const void* a, const void* b) {
    const keyed *x = (const keyed*)a, *y = (const keyed*)b;
    if (x->key < y->key) return -1;
    if (x->key > y->key) return 1;
    return (x->id > y->id) - (x->id < y->id);
}

int cpu_threads_available(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* One layer step.  Returns 0, or a negative code: -1 bad argument, -2 counts too large for the
 * exact 128-bit comparison, -3 out of memory.
 * traces [N][L][E] int32 (trace-major); eam [L][E] int64, row `layer` updated in place;
 * W_r [E][H], x [H], expert matrices in wdtype (0 = fp32, 1 = bf16 bit patterns);
 * experts[e][0..2] = W_gate [I][H], W_up [I][H], W_down [H][I] of routed expert e of this layer,
 * shared[s][0..2] likewise; resident [L*E] bytes (1 = in the cache).
 * Outputs: idx[k], w[k], best, best_sim, P[L*E], V[L*E], pf_order / ev_order [L*E] with lengths,
 * y[H]. */
int cpu_decode_step(const int32_t* traces, int N, int L, int E, int64_t* eam, int layer, const void* W_r,
                    const float* bias, const void* x, int H, int I, int wdtype, int k, int renorm, double eps,
                    const void* const* experts, const void* const* shared, int n_shared, const uint8_t* resident,
                    int threads, int32_t* idx, double* w, int32_t* best, double* best_sim, double* P, double* V,
                    int32_t* pf_order, int32_t* n_pf, int32_t* ev_order, int32_t* n_ev, double* y) {
    if (N < 0 || L < 1 || E < 1 || H < 1 || I < 1 || k < 1 || k > E || layer < 0 || layer >= L || threads < 1) return -1;
    const int bf = wdtype == 1;
    const size_t LE = (size_t)L * E;
    double* logit = (double*)malloc(sizeof(double) * (size_t)E);
    double* xv = (double*)malloc(sizeof(double) * (size_t)H);
    double* act = (double*)malloc(sizeof(double) * (size_t)I);
    keyed* keys = (keyed*)malloc(sizeof(keyed) * LE);
    uint8_t* taken = (uint8_t*)calloc((size_t)E, 1);
    if (!logit || !xv || !act || !keys || !taken) {
        free(logit); free(xv); free(act); free(keys); free(taken);
        return -3;
    }
    for (int h = 0; h < H; ++h) xv[h] = elem(x, (size_t)h, bf);

    /* ---- Sec. 2: router logits, softmax, top-k */
#pragma omp parallel for num_threads(threads) schedule(static)
    for (int e = 0; e < E; ++e) {
        double s = 0.0;
        for (int h = 0; h < H; ++h) s += elem(W_r, (size_t)e * H + h, bf) * xv[h];
        logit[e] = s + (bias ? (double)bias[e] : 0.0);
    }
    double zmax = logit[0];
    for (int e = 1; e < E; ++e) zmax = logit[e] > zmax ? logit[e] : zmax;
    double zsum = 0.0;
    for (int e = 0; e < E; ++e) zsum += exp(logit[e] - zmax);
    double wsum = 0.0;
    for (int j = 0; j < k; ++j) {
        int arg = -1;
        for (int e = 0; e < E; ++e)
            if (!taken[e] && (arg < 0 || logit[e] > logit[arg])) arg = e; /* ties: the lower index stays */
        taken[arg] = 1;
        idx[j] = arg;
        w[j] = exp(logit[arg] - zmax) / zsum;
        wsum += w[j];
    }
    if (renorm)
        for (int j = 0; j < k; ++j) w[j] /= wsum;

    /* ---- Sec. 4.3: EAM update */
    for (int j = 0; j < k; ++j) eam[(size_t)layer * E + idx[j]] += 1;

    /* ---- Sec. 4.5: cosine match over the whole collection */
    uint64_t nq = 0;
    for (size_t i = 0; i < LE; ++i) nq += (uint64_t)eam[i] * (uint64_t)eam[i];
    int32_t win = -1;
    uint64_t win_dot = 0, win_nt = 1;
    int overflow = 0;
#pragma omp parallel num_threads(threads)
    {
        int32_t my = -1;
        uint64_t my_dot = 0, my_nt = 1;
#pragma omp for schedule(static) nowait
        for (int t = 0; t < N; ++t) {
            const int32_t* T = traces + (size_t)t * LE;
            uint64_t dot = 0, nt = 0;
            for (size_t i = 0; i < LE; ++i) {
                dot += (uint64_t)T[i] * (uint64_t)eam[i];
                nt += (uint64_t)T[i] * (uint64_t)T[i];
            }
            if (dot >= (1ull << 40) || nt >= (1ull << 46)) overflow = 1;
            if (nq == 0) dot = 0;
            if (my < 0 || more_similar(dot, nt, my_dot, my_nt)) { /* ascending t: an equal one never replaces */
                my = t;
                my_dot = dot;
                my_nt = nt;
            }
        }
#pragma omp critical
        {
            if (my >= 0 && (win < 0 || more_similar(my_dot, my_nt, win_dot, win_nt) ||
                            (!more_similar(win_dot, win_nt, my_dot, my_nt) && my < win))) {
                win = my;
                win_dot = my_dot;
                win_nt = my_nt;
            }
        }
    }
    if (overflow) {
        free(logit); free(xv); free(act); free(keys); free(taken);
        return -2;
    }
    *best = win;
    *best_sim = (win >= 0 && nq > 0 && win_nt > 0) ? (double)win_dot / (sqrt((double)nq) * sqrt((double)win_nt)) : 0.0;

    /* ---- Sec. 4.5 steps 2-3 and Alg. 1: scores from the matched trace, both orders */
    const int32_t* Tm = win >= 0 ? traces + (size_t)win * LE : NULL;
    int np = 0, ne = 0;
    for (int i = 0; i < L; ++i) {
        int64_t R = 0;
        for (int j = 0; j < E; ++j) R += Tm ? Tm[(size_t)i * E + j] : 0;
        const double den = (double)(R > 0 ? R : 1) * (double)L;
        for (int j = 0; j < E; ++j) {
            const double t = Tm ? (double)Tm[(size_t)i * E + j] : 0.0;
            const size_t f = (size_t)i * E + j;
            V[f] = ((t + eps) * (double)(L - i)) / den;
            P[f] = (i > layer && R > 0) ? (t * (double)(L - i + layer)) / den : 0.0;
        }
    }
    for (size_t f = 0; f < LE; ++f)
        if ((int)(f / E) > layer && P[f] > 0.0 && !resident[f]) keys[np++] = (keyed){-P[f], (int32_t)f};
    qsort(keys, (size_t)np, sizeof(keyed), by_key_then_id);
    for (int i = 0; i < np; ++i) pf_order[i] = keys[i].id;
    for (size_t f = 0; f < LE; ++f) {
        if (!resident[f]) continue;
        int running = 0;
        for (int j = 0; j < k; ++j) running |= ((size_t)layer * E + idx[j] == f);
        if (!running) keys[ne++] = (keyed){V[f], (int32_t)f};
    }
    qsort(keys, (size_t)ne, sizeof(keyed), by_key_then_id);
    for (int i = 0; i < ne; ++i) ev_order[i] = keys[i].id;
    *n_pf = np;
    *n_ev = ne;

    /* ---- Sec. 2: the activated experts' FFN, routed picks with their gate weights, shared with 1 */
    for (int h = 0; h < H; ++h) y[h] = 0.0;
    for (int a = 0; a < k + n_shared; ++a) {
        const void* const* m3 = a < k ? experts + (size_t)idx[a] * 3 : shared + (size_t)(a - k) * 3;
        const double gw = a < k ? w[a] : 1.0;
        const void *Wg = m3[0], *Wu = m3[1], *Wd = m3[2];
#pragma omp parallel for num_threads(threads) schedule(static)
        for (int i = 0; i < I; ++i) {
            double g = 0.0, u = 0.0;
            for (int h = 0; h < H; ++h) {
                g += elem(Wg, (size_t)i * H + h, bf) * xv[h];
                u += elem(Wu, (size_t)i * H + h, bf) * xv[h];
            }
            act[i] = g / (1.0 + exp(-g)) * u;
        }
#pragma omp parallel for num_threads(threads) schedule(static)
        for (int h = 0; h < H; ++h) {
            double s = 0.0;
            for (int i = 0; i < I; ++i) s += elem(Wd, (size_t)h * I + i, bf) * act[i];
            y[h] += gw * s;
        }
    }
    free(logit); free(xv); free(act); free(keys); free(taken);
    return 0;
}
