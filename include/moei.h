/*
 * moei.h -- C ABI of the MI355X (gfx950) decode hot path of a sparsity-aware
 * MoE expert cache (arXiv 2401.14361, "MoE-Infinity").
 *
 * One batch-1 decode iteration runs, per MoE layer: router top-k, EAM update,
 * EAMC cosine match, prefetch/eviction priorities, Alg. 1 cache retrieval and
 * the activated experts' FFN over weights held in HBM cache slots.
 *
 * Conventions
 *   - Every function returns 0 (MOEI_OK) or a negative MOEI_E* code and never
 *     aborts; moei_last_error() returns a message for the calling thread's last
 *     failure.
 *   - Pointer names: d_* = device memory, h_* = host memory.  The caller owns
 *     every buffer it passes in; the library owns what *_create allocates and
 *     frees it in *_destroy.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *     Calls are asynchronous on it unless they fill h_* outputs, in which case
 *     they synchronise as documented per function.
 *   - A moei_eamc and a moei_cache each hold device scratch (partial sums, arrival
 *     counters, sort keys, partial rows) that their calls reuse: calls that name
 *     the same object must be ordered by the caller (one stream, or events
 *     between streams); calls on different objects are independent.  A cache's
 *     layer step uses the EAMC it is handed on the cache's own side stream:
 *     moei_cache_join / moei_cache_sync order that work before other uses of it.
 *   - Matrices are row-major and dense.  Layer indices are 0-based.
 *   - Notation (Sec. 4.3 of the paper): L MoE layers, E routed experts per
 *     layer, k experts per token, EAM = L x E matrix of token counts; H hidden
 *     width, I expert intermediate width, N traces in the EAMC, S cache slots.
 */
#ifndef MOEI_H
#define MOEI_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOEI_OK          0
#define MOEI_EINVAL    (-1)   /* bad argument: null pointer, shape or range */
#define MOEI_ENOMEM    (-2)   /* host or device allocation failed */
#define MOEI_EHIP      (-3)   /* a HIP runtime call failed */
#define MOEI_ESTATE    (-4)   /* object not in a state that allows the call */
#define MOEI_ECAPACITY (-5)   /* a fixed capacity would be exceeded */

#define MOEI_WDTYPE_FP32 0
#define MOEI_WDTYPE_BF16 1

/* Largest count an EAM cell may hold anywhere in this library (2^24 - 1). */
#define MOEI_MAX_COUNT 16777215

typedef struct moei_model_desc {
    int32_t L, E, k, n_shared;  /* MoE layers, routed experts/layer, top-k, always-on shared experts/layer */
    int32_t H, I;               /* hidden width, expert intermediate width */
    int32_t wdtype;             /* MOEI_WDTYPE_*: storage type of expert/router weights and of x */
    int32_t renorm_topk;        /* 1: gate weights are renormalised over the k picks */
    float   eps;                /* epsilon of Alg. 1's priority score */
} moei_model_desc;

typedef struct moei_eamc  moei_eamc;   /* the EAM collection on the device */
typedef struct moei_cache moei_cache;  /* HBM slot pool + slot table + per-layer scratch */

const char* moei_last_error(void);
const char* moei_version(void);

/* ------------------------------------------------------------------ EAMC (Sec. 4.5)
 * Expert Activation Matrix Collection: up to n_cap request-level EAMs kept on the
 * device, stored layer-major [L][n_cap][E] in cells of `cell_bytes` (4 = int32,
 * 2 = uint16) together with each trace's squared norm.
 */
int moei_eamc_create(const moei_model_desc* desc, int32_t n_cap, int32_t cell_bytes, moei_eamc** out);
/* Replaces the contents with N traces given trace-major, h_traces[N][L][E] (host).
 * Cells must lie in [0, MOEI_MAX_COUNT] (and <= 65535 for 2-byte cells), else
 * MOEI_EINVAL and the collection is left empty.  N = 0 empties it.  Synchronous. */
int moei_eamc_load(moei_eamc* c, const int32_t* h_traces, int32_t N);
/* Sec. B.1 replacement rule: stores one finished request-level EAM (host, [L][E]).
 * While N < n_cap it is appended; at capacity it overwrites trace `victim`, which
 * the caller obtains from eamc_match on that EAM (the most similar stored trace).
 * victim is ignored while not full.  Synchronous. */
int moei_eamc_insert(moei_eamc* c, const int32_t* h_eam, int32_t victim);
/* Failure recovery (Sec. B.2): trace-major dump of the collection to host memory,
 * h_traces[N][L][E]; pass the result to moei_eamc_load to restore.  Synchronous. */
int moei_eamc_export(const moei_eamc* c, int32_t* h_traces, int32_t max_traces);
/* The same through a file (the EAMC is checkpointed with the model, Sec. B.2): a 32-byte
 * header (magic "MOEIEAMC", version, L, E, N) and the traces as int32 [N][L][E].  Restoring
 * replaces the contents; a file of another shape, with more traces than the capacity, with
 * a cell the collection cannot hold, truncated or not a checkpoint is refused and leaves
 * the collection as it was (MOEI_EINVAL; MOEI_ESTATE if the file cannot be opened).  Synchronous. */
int moei_eamc_save(const moei_eamc* c, const char* path);
int moei_eamc_restore(moei_eamc* c, const char* path);
int moei_eamc_size(const moei_eamc* c);            /* N, or MOEI_EINVAL */
int moei_eamc_destroy(moei_eamc* c);

/* -------------------------------------------------------- hot-path steps, one by one */

/* Step 1, router decision (Sec. 2): per token softmax over the E logits, the k most
 * probable experts in descending order (ties to the lower index), and their gate
 * weights (softmax probabilities; divided by their sum if renorm != 0).
 * d_logits[B][E] fp32 -> d_idx[B][k] int32, d_w[B][k] fp32.  Needs 1 <= k <= E <= 4096.
 * A token whose logits admit no softmax - a NaN among them, or no finite maximum (all
 * -inf, or a +inf) - gets no picks: all k indices -1, all k weights 0 (-inf entries beside a
 * finite maximum are fine: probability 0).  eam_update and expert_ffn_grouped pass over
 * indices of -1. */
int moe_route_topk(const float* d_logits, int32_t B, int32_t E, int32_t k, int32_t renorm,
                   int32_t* d_idx, float* d_w, void* stream);

/* Step 2, EAM update (Sec. 4.3): d_eam[b][layer][d_idx[b][j]] += 1 for every pick.
 * d_eam[B][L][E] int32 in place; picks of one token must be distinct; indices outside
 * [0,E) are ignored. */
int eam_update(int32_t* d_eam, int32_t B, int32_t L, int32_t E, int32_t layer,
               const int32_t* d_idx, int32_t k, void* stream);

/* Step 3, EAMC match (Sec. 4.5): cosine similarity between each of the B flattened
 * EAMs d_eam[B][L][E] (int32, cells in [0, MOEI_MAX_COUNT]) and every stored trace;
 * d_best[b] = index of the most similar trace (smallest cosine distance; equal
 * similarities go to the lowest index; decided in exact integer arithmetic),
 * d_best_sim[b] = its similarity (fp32), d_sims[B][N] = all similarities (may be NULL).
 * A zero vector has similarity 0 to everything.  Empty collection: best = -1, sim = 0.
 * layer_hi: the caller promises rows > layer_hi of every query are zero, so only
 * layers 0..layer_hi are scanned (L-1 scans everything); norms are always those of
 * the full matrices.  B <= 16.  The device does not check the queries' cells: a cell
 * outside [0, MOEI_MAX_COUNT] gives an unspecified (but in-bounds, finite) result for
 * that query. */
int eamc_match(const moei_eamc* c, const int32_t* d_eam, int32_t B, int32_t layer_hi,
               int32_t* d_best, float* d_best_sim, float* d_sims, void* stream);

/* Step 3 with several matches (Sec. 4.5: the match may return several EAMs, which the
 * prediction aggregates): d_top[m] = the m most similar traces to the single query
 * d_eam[L][E], most similar first, equal similarities by ascending index (the total
 * order whose first element eamc_match returns; exact integer arithmetic);
 * d_top_sim[m] (may be NULL) their similarities, d_sims[N] (may be NULL) all of them.
 * Entries beyond the stored traces are -1 / 0.  1 <= m <= 16; MOEI_ECAPACITY when
 * ceil(N / 1024) * m exceeds 4096.  Feed d_top to expert_priority with B = m. */
int eamc_match_topm(const moei_eamc* c, const int32_t* d_eam, int32_t layer_hi, int32_t m,
                    int32_t* d_top, float* d_top_sim, float* d_sims, void* stream);

/* Step 4, PredictEAM + priorities (Sec. 4.5 steps 2-3; Alg. 1 priority score).
 * T = sum over b of trace d_best[b] (entries < 0 skipped), R_i = row sums of T.
 *   prefetch  P[i][j] = T[i][j] (L - i + l) / (R_i L)   for l < i < L, else 0 (0 if R_i = 0)
 *   eviction  V[i][j] = (T[i][j] + eps)(L - i) / (R_i L)  (R_i := 1 for an empty row)
 * with l = cur_layer in [-1, L-1]; each is one fp64 division of exact products,
 * written out in fp32 to d_prefetch[L][E] / d_evict[L][E].
 * d_pf_order: flat ids i*E+j with i > l, P > 0 and d_slot_of[i*E+j] < 0, by P
 *   descending; d_ev_order: flat ids with d_slot_of >= 0, except the n_cur experts
 *   d_cur_idx[n_cur] of layer l that are about to run (may be NULL; a list, repeats
 *   allowed: one query's k picks, or all picks of a batch), by V ascending; ties to the lowest
 *   flat id in both.  Counts go to d_n_pf / d_n_ev; each order buffer holds L*E ints. */
int expert_priority(const moei_eamc* c, const int32_t* d_best, int32_t B, int32_t cur_layer,
                    const int32_t* d_slot_of, float eps, const int32_t* d_cur_idx, int32_t n_cur,
                    float* d_prefetch, float* d_evict,
                    int32_t* d_pf_order, int32_t* d_n_pf, int32_t* d_ev_order, int32_t* d_n_ev,
                    void* stream);

/* --------------------------------------------------------- expert cache (Sec. 4.7, Alg. 1)
 * A pool of n_slots cache slots in HBM for routed experts plus L*n_shared pinned
 * slots for the always-on shared experts.  One slot holds one expert of 3*H*I elements
 * in desc->wdtype, interleaved by intermediate unit so that the FFN is one stream:
 *   for i in 0..I-1:  W_gate[i][0..H) | W_up[i][0..H) | W_down[0..H)[i]
 * (moei_expert_pack builds this from the three plain matrices).
 * Slot ids: 0..n_slots-1 routed, n_slots + layer*n_shared + s shared.
 * h_experts: host copy of the routed experts in slot layout (pinned memory for
 *   asynchronous fills), n_host_experts rows of 3*H*I elements; expert (l, j) is row (l*E + j) %
 *   n_host_experts.  NULL = no host copy: slots are filled by the caller
 *   (moei_cache_slot_ptr) and a miss is an error.
 * h_shared: [L*n_shared][3*H*I] or NULL (then shared slots are left for the caller).
 * Needs n_slots >= k, else MOEI_ECAPACITY. */
int moei_cache_create(const moei_model_desc* desc, int32_t n_slots,
                      const void* h_experts, int32_t n_host_experts, const void* h_shared,
                      moei_cache** out);
int moei_cache_destroy(moei_cache* c);
/* Slot layout of one expert from W_gate[I][H], W_up[I][H], W_down[H][I] (all host memory,
 * desc->wdtype elements); h_slot receives 3*H*I elements.  Pure data movement. */
int moei_expert_pack(const moei_model_desc* desc, const void* h_gate, const void* h_up, const void* h_down,
                     void* h_slot);
/* Initial residency: n_resident (<= n_slots, <= L*E) experts with flat ids
 * 0..n_resident-1 in slots of the same number, the rest free.  Copies them from
 * h_experts when there is one.  Synchronous. */
int moei_cache_reset(moei_cache* c, int32_t n_resident);
/* Device address of a slot's weights (any slot id, shared included). */
int moei_cache_slot_ptr(moei_cache* c, int32_t slot, void** d_ptr);
/* Device slot table d_slot_of[L*E] (-1 = not resident), for expert_priority. */
int moei_cache_slot_table(moei_cache* c, const int32_t** d_slot_of);
/* Host copy of the slot table, h_slot_of[L*E]. */
int moei_cache_get_slots(const moei_cache* c, int32_t* h_slot_of);
/* Alg. 1 for one layer's picks, in order: a hit keeps its slot; otherwise the
 * expert goes to the lowest free slot or, when full, to the slot of the first entry
 * of h_ev_order that is resident and not one of these picks (if the order runs out:
 * the lowest slot whose owner is not one of these picks).  Misses are copied from
 * h_experts on the cache's copy stream; `stream` then waits for them.  Per pick:
 * h_slots[n] = slot, h_victims[n] = evicted flat id or -1; *h_n_miss = misses.
 * The device slot table is updated on `stream`. */
int moei_cache_retrieve(moei_cache* c, int32_t layer, const int32_t* h_idx, int32_t n,
                        const int32_t* h_ev_order, int32_t n_ev,
                        int32_t* h_slots, int32_t* h_victims, int32_t* h_n_miss, void* stream);

/* Step 5, expert FFN (Sec. 2; SwiGLU):
 *   y = sum_e w_e * W_down,e ( silu(W_gate,e x) * (W_up,e x) ),  silu(g) = g / (1 + exp(-g))
 * over the n_act slots d_slot_ids[n_act] with weights d_gate_w[n_act]; weights are
 * streamed once from the slot pool, sums are fp32 and bit-reproducible run to run.  d_x[H] in desc->wdtype, d_y[H] fp32.
 * A slot id outside the pool contributes nothing and raises the cache's error flag.
 * n_act <= k + n_shared. */
int expert_ffn_gemv(moei_cache* c, const int32_t* d_slot_ids, const float* d_gate_w,
                    int32_t n_act, const void* d_x, float* d_y, void* stream);
/* expert_ffn_gemv for callers that cannot allocate device memory: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, same kernels
 * and bit-identical results, but the workgroup partial rows live in a static device array of
 * 256 x 5120 floats (5 MiB per GPU the library runs on, held until the process ends) instead of
 * the cache's own scratch, and the call itself allocates nothing.  MOEI_ECAPACITY when
 * (compute units - 24) x H exceeds that array (H <= 5649 on a 256-unit part).  Every call on a
 * GPU shares that GPU's array: calls that overlap on one GPU - other streams, other caches,
 * other threads - race; order them on one stream or with events.  Nothing in the array has
 * to be cleared between calls (every row that is read is written first by the same call). */
int expert_ffn_gemv_static(moei_cache* c, const int32_t* d_slot_ids, const float* d_gate_w,
                           int32_t n_act, const void* d_x, float* d_y, void* stream);
/* Step 5 for a decode batch of B independent requests (B <= 16): for every token b,
 *   y[b] = sum_j d_w[b][j] * expert(layer, d_idx[b][j])(x[b]) + sum over the layer's shared experts,
 * with the picks' slots looked up in the device slot table.  Tokens are grouped per activated
 * expert on the device and an expert's weights are streamed once per group of up to 4 of its
 * tokens, so bytes read grow with the number of distinct experts, not with B.
 * d_idx[B][k] int32, d_w[B][k] fp32, d_x[B][H] in desc->wdtype, d_y[B][H] fp32.  A pick that is
 * not resident contributes nothing and raises error flag bit 1; a pick outside [0, E) (a token
 * that got no picks) is passed over.  Needs H to be a multiple of 64 lanes x 16 bytes, E <= 256
 * and B * k <= 512 (MOEI_EINVAL otherwise).  Results are bit-reproducible run to run. */
int expert_ffn_grouped(moei_cache* c, int32_t layer, const int32_t* d_idx, const float* d_w, int32_t B,
                       const void* d_x, float* d_y, void* stream);
/* Device-side error flags raised by kernels since the last call (bit 0: bad slot id,
 * bit 1: a routed expert was not resident in a step without host retrieval, bit 2: the
 * router logits of a token admitted no softmax - NaN or no finite maximum - so the token
 * got no picks: its EAM row is unchanged and only the shared experts contribute to its
 * output; the asynchronous moe_decode_layer also raises bit 0 for the empty slots then).
 * Synchronises `stream`. */
int moei_cache_error_flags(moei_cache* c, int32_t* h_flags, void* stream);

/* ------------------------------------------------------------------ the fused layer step
 * One MoE layer of one decode iteration for one request:
 *   logits = W_r x + b -> top-k -> EAM row update -> (EAMC match -> priorities) on a
 *   side stream, while Alg. 1 retrieval and the expert FFNs run on `stream`.
 * d_router_w[E][H] in wdtype, d_router_bias[E] fp32 or NULL, d_eam[L][E] int32.
 * The eviction order used for this layer's misses is the one computed from the EAM
 * that already contains this layer's routing.
 * If all three h_* outputs are NULL the call is fully asynchronous: slots are looked
 * up on the device and a non-resident pick raises error flag bit 1.  Otherwise the
 * call waits for the routing decision, serves misses from the host copy, and fills
 * h_topk_idx[k], *h_best (matched trace, waits for the side stream) and *h_n_miss
 * (each may be NULL).  Router logits that admit no softmax (NaN, no finite maximum): the
 * synchronous call returns MOEI_ESTATE before any expert runs; the asynchronous one
 * raises error flag bit 2 (see moei_cache_error_flags). */
int moe_decode_layer(moei_cache* c, const moei_eamc* eamc, int32_t* d_eam, int32_t layer,
                     const void* d_router_w, const float* d_router_bias,
                     const void* d_x, float* d_y,
                     int32_t* h_topk_idx, int32_t* h_best, int32_t* h_n_miss, void* stream);
/* Eviction rule of moei_cache_retrieve / moe_decode_layer when the cache is full:
 * MOEI_POLICY_EAM (default) is Alg. 1, driven by the eviction order; the other two are the
 * rules the paper compares against (Sec. 4.7 example, Sec. 6), for hit-rate comparisons:
 * MOEI_POLICY_LRU evicts the slot used least recently (every pick stamps its slot; never
 * used = oldest; ties to the lowest slot), MOEI_POLICY_COUNT the resident expert activated
 * least often since the last reset (ties to the lowest id).  A victim is never one of the
 * current picks.  Under these two the eviction order is ignored. */
#define MOEI_POLICY_EAM 0
#define MOEI_POLICY_LRU 1
#define MOEI_POLICY_COUNT 2
int moei_cache_set_policy(moei_cache* c, int32_t policy);

/* Prefetching into the cache (Sec. 4.6).  The first `depth` (<= 32) entries of
 * h_pf_order[n_pf] are considered in turn; one that is not resident goes to the lowest
 * free slot or, when the cache is full, displaces the first entry of h_ev_order[n_ev]
 * that is still resident and not in h_protect[n_protect] - but only if its own eviction
 * score h_V[fid] exceeds that victim's (fp32 compare; h_V[L*E] as written by
 * expert_priority); otherwise it is skipped and the victim is offered to the next one.
 * Copies run on the cache's prefetch stream after everything already queued on `stream`;
 * they are NOT waited for here: moei_cache_retrieve and the synchronous moe_decode_layer
 * make the reading stream wait when a prefetched expert is picked or replaced, an
 * asynchronous moe_decode_layer waits for all of them, and so does moei_cache_join (needed
 * before expert_ffn_gemv / expert_ffn_grouped / moe_prefill_layer touch such a slot).  The slot tables name the new owners at once.
 * Outputs (each may be NULL): h_fids / h_victims (-1 = free slot) / h_slots [depth],
 * *h_n_issued.  All arrays are host memory.  MOEI_ESTATE without a host copy. */
int moei_cache_prefetch(moei_cache* c, const int32_t* h_pf_order, int32_t n_pf,
                        const int32_t* h_ev_order, int32_t n_ev, const float* h_V, int32_t depth,
                        const int32_t* h_protect, int32_t n_protect,
                        int32_t* h_fids, int32_t* h_victims, int32_t* h_slots, int32_t* h_n_issued,
                        void* stream);
/* Prefetch candidates moe_decode_layer considers after each layer's retrieval (0 = off, the
 * default; needs MOEI_POLICY_EAM): moei_cache_prefetch with the step's own orders and scores,
 * protecting the layer's picks.  The synchronous step does this before it returns.  The
 * asynchronous step computes the plan on the device (heads of both orders and the scores, into
 * pinned memory) and the host carries it out at the next call that names this cache -
 * moe_decode_layer of either kind, or moei_cache_join - after waiting for that step's match and
 * scoring; nothing changes the cache in between, so the prefetches are the ones the synchronous
 * step would have issued.  Such steps cannot be recorded in a stream capture (MOEI_ESTATE). */
int moei_cache_set_prefetch(moei_cache* c, int32_t depth);
/* What the last layer step prefetched (for an asynchronous step: once its plan has been carried
 * out, see moei_cache_set_prefetch): h_fids[cap] / h_victims[cap], *h_n. */
int moei_cache_last_prefetch(moei_cache* c, int32_t* h_fids, int32_t* h_victims, int32_t cap, int32_t* h_n);
/* Number of most-similar traces the layer step's prediction aggregates (default 1; Sec. 4.5
 * step 2).  Takes effect from the next moe_decode_layer; *h_best stays the most similar. */
int moei_cache_set_match_count(moei_cache* c, int32_t m);
/* The matched traces of the last layer step, most similar first, after both streams have
 * drained: h_top[cap] / h_top_sim[cap] (either may be NULL), *h_m = how many. */
int moei_cache_last_matches(moei_cache* c, int32_t* h_top, float* h_top_sim, int32_t cap,
                            int32_t* h_m, void* stream);
/* The prefill iteration of one MoE layer (Sec. 4.3: an iteration routes n tokens; each adds its
 * k picks to row `layer` of the EAM): for the n prompt tokens d_X[n][H] (bf16), routing as in
 * moe_decode_layer, d_eam[layer][e] += number of tokens that picked e, and
 * d_Y[n][H] (fp32) = sum over the token's picks of gate weight x expert FFN, plus the layer's
 * shared experts with weight 1.  Tokens are grouped per expert and the groups run on the
 * matrix cores (activations rounded to bf16 between the two projections: the stated 2e-2 bar
 * applies, not the tighter fp32 one of the decode path).  Every picked expert must be
 * resident (the cache is not consulted or changed; a non-resident pick raises error flag
 * bit 1 and contributes zero).  Optional outputs d_idx_out[n][k], d_w_out[n][k] (device).
 * bf16 weights, H a multiple of 128 and <= 4096, I a multiple of 8, E <= 2048, n <= 8192; scratch for the
 * longest prompt so far is kept in the cache (allocated on a first or longer call, which
 * drains the device).  All work is queued on `stream`. */
int moe_prefill_layer(moei_cache* c, int32_t* d_eam, int32_t layer,
                      const void* d_router_w, const float* d_router_bias,
                      const void* d_X, int32_t n, float* d_Y,
                      int32_t* d_idx_out, float* d_w_out, void* stream);
/* Makes `stream` wait for the match/priority work that the last moe_decode_layer put on
 * the cache's side stream (the next moe_decode_layer does this by itself) and for every
 * prefetch copy that no stream has waited for yet; carries out the prefetch plan of an
 * asynchronous step first (then it waits for that step's side stream on the host).  Call it
 * before ending a stream capture that contains asynchronous layer steps, so that the
 * side stream has joined `stream` again. */
int moei_cache_join(moei_cache* c, void* stream);
/* Waits on the host for the cache's own streams (match/priority work, miss fills) and
 * forgets any pending cross-stream dependency.  Call it before beginning and after
 * ending a stream capture, so that no wait inside the capture refers to work outside
 * it and vice versa. */
int moei_cache_sync(moei_cache* c);
/* Results of the most recent moe_decode_layer on this cache, copied to the host
 * (any pointer may be NULL): gate weights [k], best similarity, score matrices [L*E],
 * orders [L*E] and their lengths.  Synchronises both streams.
 * A layer step itself selects only the heads of the two orders - Alg. 1 takes at most one victim
 * per pick from the front of the eviction order, prefetching looks at `depth` candidates - and
 * keeps the sort keys of every cell; the complete orders are ranked from those keys here, on
 * demand (one more kernel per call that asks for an order). */
int moei_cache_last_step(moei_cache* c, float* h_gate_w, float* h_best_sim,
                         float* h_prefetch, float* h_evict,
                         int32_t* h_pf_order, int32_t* h_n_pf, int32_t* h_ev_order, int32_t* h_n_ev,
                         void* stream);

/* The heads of the two orders as the most recent moe_decode_layer selected them itself:
 * h_ev_head[min(k + depth, n_ev)] (what Alg. 1's retrieval consumes) and h_pf_head[min(depth, n_pf)]
 * (prefetch candidates; depth as set by moei_cache_set_prefetch), their lengths in *h_n_ev_head /
 * *h_n_pf_head; cap_* = room in the arrays (MOEI_ECAPACITY if too small).  They are the leading
 * entries of the complete orders.  Synchronises both streams. */
int moei_cache_last_heads(moei_cache* c, int32_t* h_pf_head, int32_t cap_pf, int32_t* h_n_pf_head,
                          int32_t* h_ev_head, int32_t cap_ev, int32_t* h_n_ev_head, void* stream);

/* ------------------------------------------------------------------ kernel timing (diagnostic)
 * While enabled, every kernel launch of the library carries a start and a stop HIP event
 * that the runtime stamps with the kernel's own begin and end on its stream (at most
 * max_samples launches are recorded, later ones are not timed).  moei_profile_read
 * synchronises the device and returns, for kernel `id` (0 <= id <
 * moei_profile_kernels()), the number of recorded launches and the sum of their
 * start-to-stop durations in milliseconds.  Not thread-safe. */
int moei_profile_enable(int32_t max_samples);
int moei_profile_disable(void);
int moei_profile_kernels(void);
const char* moei_profile_kernel_name(int32_t id);
int moei_profile_read(int32_t id, double* total_ms, int32_t* count);
/* The recorded launches of one kernel one by one, in launch order: h_ms[min(cap, *count)]
 * milliseconds each; *count = launches recorded (may exceed cap). */
int moei_profile_samples(int32_t id, float* h_ms, int32_t cap, int32_t* count);

#ifdef __cplusplus
}
#endif
#endif /* MOEI_H */
