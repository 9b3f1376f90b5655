"""Seeded generators. Draws only; no routing, matching, scoring or FFN maths here.

Stream ids: ``BASE_SEED + 1000*cid + purpose`` with purpose 0 = expert weights,
1 = router weights, 2 = EAMC traces, 3 = request, 4 = hidden states; further
integers (layer, trace id, request id) are appended to the SeedSequence entropy
so that every object can be regenerated on its own.
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass

import numpy as np

from .configs import BASE_SEED, Config

P_WEIGHTS, P_ROUTER, P_TRACES, P_REQUEST, P_HIDDEN = range(5)


def stream(cfg: Config, purpose: int, *extra: int) -> np.random.Generator:
    ent = [BASE_SEED + 1000 * cfg.cid + purpose] + [int(e) for e in extra]
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(ent)))


# ---------------------------------------------------------------- storage types
def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    return ((u + np.uint32(0x7FFF) + lsb) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def store_dtype(cfg: Config):
    return np.float32 if cfg.wdtype == "fp32" else np.uint16


def to_store(cfg: Config, a: np.ndarray) -> np.ndarray:
    """Round float32 data to the configuration's storage type (fp32 or bf16 bits)."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a if cfg.wdtype == "fp32" else f32_to_bf16_bits(a)


def store_to_f32(cfg: Config, a: np.ndarray) -> np.ndarray:
    return np.asarray(a, dtype=np.float32) if cfg.wdtype == "fp32" else bf16_bits_to_f32(a)


# ---------------------------------------------------------------------- weights
def expert_weights(cfg: Config, uid: int, out: np.ndarray | None = None) -> np.ndarray:
    """One expert, flat: W_gate[I][H], W_up[I][H], W_down[H][I], i.i.d. N(0, w_std)."""
    rng = stream(cfg, P_WEIGHTS, uid)
    w = rng.standard_normal(cfg.expert_elems, dtype=np.float32)
    w *= np.float32(cfg.w_std)
    s = to_store(cfg, w)
    if out is not None:
        out[...] = s
        return out
    return s


def expert_bank(cfg: Config, n_unique: int, out: np.ndarray | None = None, threads: int = 8) -> np.ndarray:
    """``n_unique`` distinct experts, shape [n_unique][3*H*I] in storage dtype.

    Expert (layer l, index e) maps to bank row ``(l*E + e) % n_unique`` wherever a
    full L*E bank would not fit or would take too long to draw.
    """
    if out is None:
        out = np.empty((n_unique, cfg.expert_elems), dtype=store_dtype(cfg))
    assert out.shape == (n_unique, cfg.expert_elems)
    with ThreadPoolExecutor(max_workers=max(1, threads)) as ex:
        list(ex.map(lambda u: expert_weights(cfg, u, out[u]), range(n_unique)))
    return out


def router_weights(cfg: Config, layer: int) -> np.ndarray:
    """Router matrix of one layer, [E][H] in storage dtype, i.i.d. N(0, r_std)."""
    rng = stream(cfg, P_ROUTER, layer)
    w = rng.standard_normal((cfg.E, cfg.H), dtype=np.float32) * np.float32(cfg.r_std)
    return to_store(cfg, w)


# ------------------------------------------------------------------ preferences
def _zipf(E: int, s: float) -> np.ndarray:
    r = np.arange(1, E + 1, dtype=np.float64)
    z = r ** (-s)
    return z / z.sum()


def cluster_preferences(cfg: Config) -> np.ndarray:
    """[n_clusters][L][E]: Zipf(s) over a seeded per-(cluster, layer) expert permutation."""
    rng = stream(cfg, P_TRACES, 0)
    z = _zipf(cfg.E, cfg.zipf_s)
    C = max(cfg.n_clusters, 1)
    out = np.empty((C, cfg.L, cfg.E), dtype=np.float64)
    for c in range(C):
        for l in range(cfg.L):
            out[c, l, rng.permutation(cfg.E)] = z
    return out


def _own_permuted_zipf(cfg: Config, rng: np.random.Generator) -> np.ndarray:
    z = _zipf(cfg.E, cfg.zipf_s)
    out = np.empty((cfg.L, cfg.E), dtype=np.float64)
    for l in range(cfg.L):
        out[l, rng.permutation(cfg.E)] = z
    return out


def trace_preferences(cfg: Config, t: int, clusters: np.ndarray | None = None):
    """Preference rows p[L][E] of trace ``t`` and its cluster id (-1 if it has its own)."""
    rng = stream(cfg, P_TRACES, 1, t)
    if cfg.n_clusters > 0:
        if clusters is None:
            clusters = cluster_preferences(cfg)
        c = int(rng.integers(cfg.n_clusters))
        base = clusters[c]
    else:
        c = -1
        base = _own_permuted_zipf(cfg, rng)
    noise = rng.dirichlet(np.full(cfg.E, cfg.dirichlet_alpha), size=cfg.L)
    p = (1.0 - cfg.mix_noise) * base + cfg.mix_noise * noise
    return p / p.sum(axis=1, keepdims=True), c, rng


def counts_from_preferences(rng: np.random.Generator, p: np.ndarray, n_tokens, k: int) -> np.ndarray:
    """Token counts per expert for rows of preferences ``p[R][E]``.

    Each row gets ``n_tokens*k`` activations in total and no expert more than
    ``n_tokens`` (a token picks k *distinct* experts): a multinomial draw whose
    excess over the per-expert cap is redrawn among the experts still below it.
    """
    p = np.asarray(p, dtype=np.float64)
    R, E = p.shape
    n = np.broadcast_to(np.asarray(n_tokens, dtype=np.int64), (R,)).copy()
    assert k <= E
    counts = rng.multinomial(n * k, p).astype(np.int64)
    for _ in range(64):
        cap = n[:, None]
        excess = np.maximum(counts - cap, 0).sum(axis=1)
        if not excess.any():
            break
        counts = np.minimum(counts, cap)
        room = (counts < cap)
        p2 = np.where(room, np.maximum(p, 1e-300), 0.0)
        s = p2.sum(axis=1, keepdims=True)
        p2 = np.where(s > 0, p2 / np.where(s > 0, s, 1.0), 1.0 / E)
        counts += rng.multinomial(excess, p2)
    else:  # pragma: no cover - cannot happen for k <= E
        raise RuntimeError("cap redistribution did not converge")
    assert (counts.sum(axis=1) == n * k).all() and (counts <= n[:, None]).all()
    return counts.astype(np.int32)


# ------------------------------------------------------------------------- EAMC
def _one_trace(cfg: Config, t: int, clusters):
    p, c, rng = trace_preferences(cfg, t, clusters)
    r = int(rng.integers(32, 513))
    return counts_from_preferences(rng, p, r, cfg.k), c, r


def eamc_traces(cfg: Config, N: int | None = None, threads: int = 8):
    """EAMC contents: int32 [N][L][E] request-level EAMs, plus (cluster id, tokens) per trace.

    Trace t covers r_t ~ U{32..512} tokens, so every row of it sums to r_t*k and
    no cell exceeds 512.
    """
    N = cfg.N if N is None else N
    clusters = cluster_preferences(cfg) if cfg.n_clusters > 0 else None
    traces = np.empty((N, cfg.L, cfg.E), dtype=np.int32)
    cl = np.empty(N, dtype=np.int32)
    rt = np.empty(N, dtype=np.int32)

    def work(t):
        traces[t], cl[t], rt[t] = _one_trace(cfg, t, clusters)

    if threads > 1 and N >= 64:
        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, range(N)))
    else:
        for t in range(N):
            work(t)
    return traces, cl, rt


# ---------------------------------------------------------------------- request
@dataclass
class Request:
    rid: int
    source: int                 # cluster id, or planted trace id when traces own their permutations
    p_req: np.ndarray           # [L][E] float64 preference of this request
    bias: np.ndarray            # [L][E] float32 = log p_req, added to the router logits
    prefill_eam: np.ndarray     # [L][E] int32 counts of the prompt tokens (zeros if no prompt)
    x: np.ndarray               # [T][L][H] storage dtype, teacher-forced layer inputs


def make_request(cfg: Config, rid: int = 0, decode: int | None = None, clusters: np.ndarray | None = None) -> Request:
    """One request: its own skewed preference, the prompt's EAM and per-(token, layer) inputs.

    The preference is a cluster's (or, when every trace has its own permutation,
    one planted trace's) permuted Zipf mixed with fresh Dirichlet noise.  Decode
    routing is *not* drawn here: it comes out of the router under test, fed with
    ``x`` and ``bias = log p_req``.
    """
    T = cfg.decode if decode is None else decode
    rng = stream(cfg, P_REQUEST, rid)
    if cfg.n_clusters > 0:
        if clusters is None:
            clusters = cluster_preferences(cfg)
        src = int(rng.integers(cfg.n_clusters))
        base = clusters[src]
    else:
        src = int(rng.integers(cfg.N))
        # the planted trace's own permutations, redrawn from that trace's stream
        base = _own_permuted_zipf(cfg, stream(cfg, P_TRACES, 1, src))
    noise = rng.dirichlet(np.full(cfg.E, cfg.dirichlet_alpha), size=cfg.L)
    p = (1.0 - cfg.mix_noise) * base + cfg.mix_noise * noise
    p = p / p.sum(axis=1, keepdims=True)
    bias = np.log(np.maximum(p, 1e-30)).astype(np.float32)
    if cfg.prompt > 0:
        prefill = counts_from_preferences(rng, p, cfg.prompt, cfg.k)
    else:
        prefill = np.zeros((cfg.L, cfg.E), dtype=np.int32)
    xr = stream(cfg, P_HIDDEN, rid)
    x = to_store(cfg, xr.standard_normal((T, cfg.L, cfg.H), dtype=np.float32))
    return Request(rid, src, p, bias, prefill, x)
