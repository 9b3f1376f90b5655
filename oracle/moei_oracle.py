"""CPU oracle for the batch-1 MoE decode layer step of the sparsity-aware expert cache.

TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition the HIP path
is checked against.  Only tests, the smoke check and the benchmark's CPU-baseline
leg may import it; the product path never does.  It shares no code, tables or
helpers with the HIP sources and imports nothing from the GPU package.

Arithmetic: integers are Python ints / int64, reals are fp64, one thread, no
blocking, no fusion.  Every function cites the passage of the paper
(arXiv 2401.14361) it follows.  Readings taken where the paper is silent or
garbled are marked "reading:".

Pin status (tests marked "not gpu" under tests/): every function below is pinned
to something other than itself -- brute force with exact fractions, library
routines, closed forms, invariants, or the worked example of Sec. 4.7.  The
composite ``decode_layer``, which the paper prints no value for, is pinned through
its parts and through one layer step worked by hand.
"""
from __future__ import annotations

import math
from fractions import Fraction

import numpy as np

__all__ = [
    "to_f64", "router_logits", "softmax", "route_topk", "eam_update", "eamc_match",
    "eamc_match_topm", "aggregate_matches", "expert_priority", "swiglu_expert", "expert_ffn",
    "ExpertCache", "decode_layer", "prefill_layer",
]


# --------------------------------------------------------------------- storage
def to_f64(a) -> np.ndarray:
    """Stored values -> fp64, exactly. uint16 arrays hold bfloat16 bit patterns."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


# ---------------------------------------------------------- step 1: router, top-k
def router_logits(W_r, x, bias=None) -> np.ndarray:
    """logit_j = sum_h W_r[j][h] x[h] (+ b_j): the router scores of one token (Sec. 2)."""
    z = to_f64(W_r) @ to_f64(x)
    if bias is not None:
        z = z + to_f64(bias)
    return z


def softmax(z) -> np.ndarray:
    z = np.asarray(z, dtype=np.float64)
    e = np.exp(z - z.max())
    return e / e.sum()


def route_topk(logits, k: int, renorm: bool):
    """Router decision for each token (Sec. 2; e.g. 2 of 8 experts, or 1 of 128).

    reading: softmax over all E experts, then the k most probable; the order is
    by descending logit with ties going to the lower expert index; gate weight =
    softmax probability, divided by the sum over the k picks when ``renorm``.
    Returns (idx [B][k] int64, w [B][k] fp64).
    """
    z = np.atleast_2d(np.asarray(logits, dtype=np.float64))
    B, E = z.shape
    if not (1 <= k <= E):
        raise ValueError("need 1 <= k <= E")
    idx = np.empty((B, k), dtype=np.int64)
    w = np.empty((B, k), dtype=np.float64)
    for b in range(B):
        order = sorted(range(E), key=lambda j: (-z[b, j], j))[:k]
        p = softmax(z[b])
        idx[b] = order
        w[b] = p[order]
        if renorm:
            w[b] = w[b] / w[b].sum()
    return idx, w


# ------------------------------------------------------------ step 2: EAM update
def eam_update(eam, layer: int, idx) -> None:
    """M[l][j] += 1 for every expert j a token was routed to at layer l (Sec. 4.3).

    ``eam`` is one request's L x E matrix; ``idx`` holds the picks of one token
    ([k]) or of several tokens ([n][k]).  Rows above l are left untouched, which
    gives the iteration-level property of Sec. 4.3 (rows > l stay zero).
    """
    L, E = eam.shape
    if not (0 <= layer < L):
        raise ValueError("layer out of range")
    for j in np.asarray(idx, dtype=np.int64).reshape(-1):
        if not (0 <= j < E):
            raise ValueError("expert index out of range")
        eam[layer, j] += 1


# ------------------------------------------------------------ step 3: EAMC match
def eamc_match(traces, q):
    """Most similar stored EAM by cosine distance of the flattened matrices (Sec. 4.5).

    sim_t = <q, T_t> / (|q| |T_t|), 0 when either vector is all zero (reading:
    never NaN).  The winner is the trace of largest similarity (= smallest cosine
    distance); equal similarities go to the lowest trace index.  The ranking is
    decided in exact integer arithmetic: all dots are >= 0, |q| is common to all
    traces, so sim_a > sim_b  <=>  dot_a^2 |T_b|^2 > dot_b^2 |T_a|^2.
    Returns (best, sim_best, sims[N]) with sims in fp64; (-1, 0.0, []) if N = 0.
    """
    T = np.asarray(traces)
    N = T.shape[0]
    if N == 0:
        return -1, 0.0, np.zeros(0, dtype=np.float64)
    qv = np.asarray(q).reshape(-1).astype(np.int64)
    Tv = T.reshape(N, -1).astype(np.int64)
    if Tv.shape[1] != qv.shape[0]:
        raise ValueError("shape mismatch")
    if (qv < 0).any() or (Tv < 0).any():
        raise ValueError("EAM counts are non-negative")
    dots = Tv @ qv
    nts = (Tv * Tv).sum(axis=1)
    nq = int((qv * qv).sum())
    sims = np.zeros(N, dtype=np.float64)
    for t in range(N):
        if nq > 0 and nts[t] > 0:
            sims[t] = float(dots[t]) / (math.sqrt(nq) * math.sqrt(int(nts[t])))
    best, best_key = 0, None
    for t in range(N):
        d, n = int(dots[t]), int(nts[t])
        key = Fraction(d * d, n) if (n > 0 and nq > 0) else Fraction(0)
        if best_key is None or key > best_key:
            best, best_key = t, key
    return best, float(sims[best]), sims


def eamc_match_topm(traces, q, m: int):
    """The m most similar stored EAMs (Sec. 4.5: the match may hand back several EAMs,
    which PredictEAM then aggregates).

    reading: the paper does not say how many matches are returned or by what rule;
    here the caller fixes m and the m traces of largest cosine similarity are taken,
    most similar first, equal similarities by ascending trace index -- the same total
    order whose first element ``eamc_match`` returns.  Decided with exact fractions
    (dot^2 / |T|^2).  Returns (idx list, sims list) of length min(m, N).
    """
    if m < 0:
        raise ValueError("m must be >= 0")
    T = np.asarray(traces)
    N = T.shape[0]
    if N == 0 or m == 0:
        return [], []
    qv = np.asarray(q).reshape(-1).astype(np.int64)
    Tv = T.reshape(N, -1).astype(np.int64)
    nq = int((qv * qv).sum())
    dots = Tv @ qv
    nts = (Tv * Tv).sum(axis=1)
    keyed = []
    for t in range(N):
        d, n = int(dots[t]), int(nts[t])
        key = Fraction(d * d, n) if (n > 0 and nq > 0) else Fraction(0)
        sim = d / (math.sqrt(nq) * math.sqrt(n)) if (n > 0 and nq > 0) else 0.0
        keyed.append((key, t, sim))
    keyed.sort(key=lambda e: (-e[0], e[1]))
    top = keyed[:m]
    return [t for _, t, _ in top], [s for _, _, s in top]


# -------------------------------------------------------- step 4: PredictEAM
def aggregate_matches(traces, best_list) -> np.ndarray:
    """PredictEAM step 2 (Sec. 4.5): cells of the matched EAMs are summed (rows are
    normalised later, inside the scores).  One match per request of the batch;
    an index of -1 (empty EAMC) contributes nothing."""
    T = np.asarray(traces)
    L, E = T.shape[1], T.shape[2]
    out = np.zeros((L, E), dtype=np.int64)
    for b in np.asarray(best_list).reshape(-1):
        if b >= 0:
            out += T[int(b)].astype(np.int64)
    return out


def expert_priority(tstar, cur_layer: int, resident, eps: float, exclude=()):
    """Prefetch and eviction priorities from the matched EAM.

    Prefetch (Sec. 4.5, PredictEAM steps 2-3): row-normalised cell times the layer
    proximity factor, P[i][j] = (T[i][j] / R_i) (1 - (i - l)/L) for future layers
    l < i < L, else 0; R_i = sum_j T[i][j]; P = 0 where R_i = 0.
    Eviction (Sec. 4.7, Alg. 1 priority score with layer decay):
    V[i][j] = (T[i][j] + eps) (1 - i/L) / R_i, layers 0-based (reading), R_i := 1
    where the row is empty.
    Both are evaluated as ONE fp64 division of exactly representable products,
    P = T (L - i + l) / (R_i L),  V = (T + eps)(L - i) / (R_i L),
    so equal rationals give equal keys and ties are decided by index alone.

    pf_order: flat ids i*E+j with i > l, P > 0, not resident, by P descending,
              ties to the lowest flat id (what to prefetch first).
    ev_order: flat ids of resident experts not in ``exclude`` (the experts the
              current layer is about to run), by V ascending, ties to the lowest
              flat id (what Alg. 1 evicts first: the argmin).
    ``cur_layer`` may be -1 (before the first layer).
    Returns (P [L][E] fp64, V [L][E] fp64, pf_order list, ev_order list).
    """
    T = np.asarray(tstar).astype(np.int64)
    L, E = T.shape
    if not (-1 <= cur_layer < L):
        raise ValueError("cur_layer out of range")
    res = np.asarray(resident).astype(bool).reshape(L, E)
    excl = set(int(e) for e in exclude)
    l = cur_layer
    P = np.zeros((L, E), dtype=np.float64)
    V = np.zeros((L, E), dtype=np.float64)
    for i in range(L):
        R = int(T[i].sum())
        Rv = R if R > 0 else 1
        den = float(Rv) * float(L)
        for j in range(E):
            t = float(int(T[i, j]))
            V[i, j] = ((t + float(eps)) * float(L - i)) / den
            if i > l and R > 0:
                P[i, j] = (t * float(L - i + l)) / den
    pf = [i * E + j for i in range(L) for j in range(E)
          if i > l and P[i, j] > 0.0 and not res[i, j]]
    pf.sort(key=lambda f: (-P[f // E, f % E], f))
    ev = [i * E + j for i in range(L) for j in range(E)
          if res[i, j] and (i * E + j) not in excl]
    ev.sort(key=lambda f: (V[f // E, f % E], f))
    return P, V, pf, ev


# ------------------------------------------------------------- step 5: expert FFN
def swiglu_expert(x, W_g, W_u, W_dn) -> np.ndarray:
    """One expert FFN (Sec. 2: experts are feed-forward networks), SwiGLU form:
    o = W_dn ( silu(W_g x) * (W_u x) ), silu(g) = g / (1 + exp(-g)).  fp64 throughout;
    the intermediate is not rounded to the storage type."""
    xv = to_f64(x)
    g = to_f64(W_g) @ xv
    u = to_f64(W_u) @ xv
    a = g / (1.0 + np.exp(-g)) * u
    return to_f64(W_dn) @ a


def expert_ffn(x, experts, gates) -> np.ndarray:
    """y = sum_e w_e * expert_e(x) over the activated experts (routed picks with their
    gate weights, always-on shared experts with weight 1).  ``experts`` is a list of
    (W_g [I][H], W_u [I][H], W_dn [H][I])."""
    y = None
    for (Wg, Wu, Wd), w in zip(experts, gates):
        o = float(w) * swiglu_expert(x, Wg, Wu, Wd)
        y = o if y is None else y + o
    if y is None:
        return np.zeros(np.asarray(x).shape[0], dtype=np.float64)
    return y


# ---------------------------------------------------------- cache retrieval (Alg. 1)
class ExpertCache:
    """Expert cache of Sec. 4.7 / Alg. 1 as a slot table: S slots, expert id = l*E + j.

    reading: the cache starts full of the experts with flat ids 0..S-1 in slots
    0..S-1 (``warm=True``) or empty.  ``retrieve`` serves one layer's picks in
    router order: a hit returns the slot; with a free slot the expert is fetched
    into the lowest free slot; otherwise a victim chosen by the policy gives up its
    slot.  The victim is never one of this layer's picks.

    policy "eam" (the paper's, Alg. 1): the first entry of ``ev_order`` (lowest
    eviction priority first) that is still resident; if ``ev_order`` runs out, the
    lowest slot whose owner is not a current pick.
    The two policies the paper compares against (Sec. 4.7, the example with three
    caches; Sec. 6), as plain eviction rules, for the hit-rate comparison only:
    policy "lru": the slot used least recently; every pick, hit or miss, stamps
      its slot with a running clock; slots never used (warm start) carry stamp 0;
      ties to the lowest slot.
    policy "count": the resident expert activated least often so far (a
      model-level count over everything this cache has served); ties to the lowest
      flat id.
    """

    POLICIES = ("eam", "lru", "count")

    def __init__(self, L: int, E: int, S: int, warm: bool = True, policy: str = "eam"):
        if policy not in self.POLICIES:
            raise ValueError("unknown policy")
        self.L, self.E, self.S, self.policy = L, E, S, policy
        self.slot_of = np.full(L * E, -1, dtype=np.int64)
        self.owner = np.full(S, -1, dtype=np.int64)
        self.stamp = np.zeros(S, dtype=np.int64)
        self.clock = 0
        self.count = np.zeros(L * E, dtype=np.int64)
        if warm:
            for s in range(min(S, L * E)):
                self.slot_of[s] = s
                self.owner[s] = s

    def resident(self) -> np.ndarray:
        return (self.slot_of >= 0).reshape(self.L, self.E)

    def _victim(self, needed, ev, pos):
        """(victim flat id, new position in ev) for a full cache."""
        if self.policy == "lru":
            best = None
            for s in range(self.S):
                if int(self.owner[s]) in needed:
                    continue
                if best is None or self.stamp[s] < self.stamp[best]:
                    best = s
            return int(self.owner[best]), pos
        if self.policy == "count":
            best = None
            for s in range(self.S):
                f = int(self.owner[s])
                if f in needed:
                    continue
                if best is None or (self.count[f], f) < (self.count[best], best):
                    best = f
            return best, pos
        while pos < len(ev):
            c = int(ev[pos]); pos += 1
            if self.slot_of[c] >= 0 and c not in needed:
                return c, pos
        for s2 in range(self.S):
            if int(self.owner[s2]) not in needed:
                return int(self.owner[s2]), pos
        raise AssertionError("no victim")

    def retrieve(self, layer: int, picks, ev_order=()):
        """Returns a list of (flat id, hit, victim flat id or -1, slot), one per pick."""
        picks = [int(p) for p in picks]
        needed = set(layer * self.E + p for p in picks)
        if len(needed) > self.S:
            raise ValueError("cache smaller than one layer's picks")
        ev = list(ev_order)
        pos = 0
        out = []
        for p in picks:
            fid = layer * self.E + p
            self.count[fid] += 1
            s = int(self.slot_of[fid])
            hit = s >= 0
            victim = -1
            if not hit:
                free = np.nonzero(self.owner < 0)[0]
                if free.size:
                    s = int(free[0])
                else:
                    victim, pos = self._victim(needed, ev, pos)
                    s = int(self.slot_of[victim])
                    self.slot_of[victim] = -1
                self.slot_of[fid] = s
                self.owner[s] = fid
            self.clock += 1
            self.stamp[s] = self.clock
            out.append((fid, hit, victim, s))
        return out

    def prefetch(self, pf_order, ev_order, V, depth: int, protect=()):
        """Prefetching into the cache (Sec. 4.6: the cache is extended by prefetching).

        reading (the paper leaves the mechanism out): after a layer's retrieval the
        first ``depth`` entries of ``pf_order`` (most likely future experts first)
        are considered in turn.  A candidate that is not resident takes the lowest
        free slot; with a full cache it may displace the cheapest victim -- the
        first entry of ``ev_order`` that is still resident and not in ``protect``
        -- but only if that improves the cache by Alg. 1's own measure: the
        candidate's eviction score must exceed the victim's, compared in fp32 (the
        precision the scores are handed over in).  A candidate that is not
        admitted is skipped and the same victim is offered to the next one.
        A prefetched expert counts as a use for the "lru" stamps, not for the
        activation counts.  Returns a list of (flat id, victim or -1, slot).
        """
        Vf = np.asarray(V, dtype=np.float64).reshape(-1).astype(np.float32)
        ev = [int(e) for e in ev_order]
        prot = set(int(p) for p in protect)
        pos = 0
        out = []
        for c in [int(c) for c in list(pf_order)[:max(depth, 0)]]:
            if self.slot_of[c] >= 0:
                continue
            free = np.nonzero(self.owner < 0)[0]
            victim = -1
            if free.size:
                s = int(free[0])
            else:
                while pos < len(ev) and (self.slot_of[ev[pos]] < 0 or ev[pos] in prot):
                    pos += 1
                if pos >= len(ev):
                    break
                if not (Vf[c] > Vf[ev[pos]]):
                    continue
                victim = ev[pos]; pos += 1
                s = int(self.slot_of[victim])
                self.slot_of[victim] = -1
            self.slot_of[c] = s
            self.owner[s] = c
            self.clock += 1
            self.stamp[s] = self.clock
            out.append((c, victim, s))
        return out


# ----------------------------------------------------------------- whole layer step
def decode_layer(traces, eam, cache: ExpertCache, layer: int, W_r, bias, x, expert_of, shared_of,
                 k: int, renorm: bool, eps: float, m: int = 1, prefetch_depth: int = 0):
    """One MoE layer of one decode iteration, in the order of Sec. 4.3-4.7:
    routing decision, EAM update, EAMC match, priorities, Alg. 1 retrieval, expert FFNs.

    ``expert_of(flat_id)`` / ``shared_of(layer)`` hand back weight triples.  The
    eviction order used for this layer's misses is the one computed from the EAM
    that already holds this layer's routing (Alg. 1 calls PredictEAM with the
    current EAM).  With m > 1 the m most similar traces are aggregated; with
    prefetch_depth > 0 the layer's retrieval is followed by ``ExpertCache.prefetch``.
    Composite: pinned through its parts and through a step worked by hand (tests).
    """
    L, E = eam.shape
    z = router_logits(W_r, x, bias)
    idx, w = route_topk(z, k, renorm)
    idx, w = idx[0], w[0]
    eam_update(eam, layer, idx)
    best, sim, _ = eamc_match(traces, eam)
    matched = [best] if m == 1 else eamc_match_topm(traces, eam, m)[0]
    tstar = aggregate_matches(traces, matched)
    excl = [layer * E + int(j) for j in idx]
    P, V, pf, ev = expert_priority(tstar, layer, cache.resident(), eps, excl)
    events = cache.retrieve(layer, idx, ev)
    prefetched = cache.prefetch(pf, ev, V, prefetch_depth, excl) if prefetch_depth > 0 else []
    experts = [expert_of(layer * E + int(j)) for j in idx]
    gates = [float(v) for v in w]
    for sh in shared_of(layer):
        experts.append(sh)
        gates.append(1.0)
    y = expert_ffn(x, experts, gates)
    return dict(logits=z, idx=idx, w=w, best=best, sim=sim, matched=list(matched), P=P, V=V, pf_order=pf,
                ev_order=ev, events=events, prefetched=prefetched, y=y)


# ------------------------------------------------------------- prefill iteration
def prefill_layer(eam, layer: int, W_r, bias, X, expert_of, shared_of, k: int, renorm: bool):
    """One MoE layer of the prefill iteration: all n prompt tokens pass the layer together
    (Sec. 4.3: an iteration routes n tokens, every token adds its k picks to row l of the EAM).

    Token by token: routing decision, EAM update, the picked experts' FFNs weighted by
    the gate weights plus the shared experts with weight 1.  Every expert is taken to be
    available (the cache is not consulted: the prompt pass decides nothing about
    eviction here).  Returns (idx [n][k], w [n][k], Y [n][H] fp64); ``eam`` is updated in place.
    """
    X = to_f64(X)
    n = X.shape[0]
    L, E = eam.shape
    idx = np.zeros((n, k), dtype=np.int64)
    w = np.zeros((n, k), dtype=np.float64)
    Y = np.zeros((n, X.shape[1]), dtype=np.float64)
    shared = list(shared_of(layer))
    for t in range(n):
        z = router_logits(W_r, X[t], bias)
        i_t, w_t = route_topk(z, k, renorm)
        idx[t], w[t] = i_t[0], w_t[0]
        eam_update(eam, layer, idx[t])
        experts = [expert_of(layer * E + int(j)) for j in idx[t]] + shared
        gates = [float(v) for v in w[t]] + [1.0] * len(shared)
        Y[t] = expert_ffn(X[t], experts, gates)
    return idx, w, Y
