"""Pins for the CPU oracle: each check ties an oracle function to something other
than itself -- exact fractions on tiny inputs, library routines, closed forms,
invariants, and the worked example of Sec. 4.7 (tests/golden/).  No GPU needed.
"""
import itertools
import json
import math
import os
from fractions import Fraction

import numpy as np
import pytest
import scipy.special
import torch

from oracle import moei_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


# =============================================================== O1 router / top-k
def test_topk_matches_stable_argsort_library():
    rng = np.random.default_rng(1)
    for E, k in [(8, 2), (64, 6), (160, 6), (5, 5), (7, 1)]:
        z = rng.standard_normal((9, E))
        idx, w = O.route_topk(z, k, renorm=False)
        ref = np.argsort(-z, axis=1, kind="stable")[:, :k]
        assert (idx == ref).all()
        p = scipy.special.softmax(z, axis=1)
        np.testing.assert_allclose(w, np.take_along_axis(p, ref, 1), rtol=1e-13)


def test_topk_ties_go_to_lowest_index():
    z = np.array([[1.0, 3.0, 3.0, 0.5, 3.0, 1.0]])
    idx, _ = O.route_topk(z, 4, renorm=False)
    assert idx.tolist() == [[1, 2, 4, 0]]
    idx, _ = O.route_topk(np.zeros((1, 6)), 3, renorm=True)
    assert idx.tolist() == [[0, 1, 2]]


def test_topk_special_cases():
    rng = np.random.default_rng(2)
    z = rng.standard_normal((4, 11))
    idx, w = O.route_topk(z, 11, renorm=False)      # k = E: a permutation, weights = softmax
    for b in range(4):
        assert sorted(idx[b].tolist()) == list(range(11))
        assert abs(w[b].sum() - 1.0) < 1e-14
        assert (np.diff(z[b, idx[b]]) <= 0).all()
    idx1, w1 = O.route_topk(z, 1, renorm=True)      # k = 1: argmax, renormalised weight is 1
    assert (idx1[:, 0] == z.argmax(axis=1)).all()
    assert (w1 == 1.0).all()
    _, wr = O.route_topk(z, 3, renorm=True)
    np.testing.assert_allclose(wr.sum(axis=1), 1.0, rtol=1e-14)
    with pytest.raises(ValueError):
        O.route_topk(z, 12, False)


def test_topk_brute_force_subsets():
    # the chosen set maximises the sum of logits over all k-subsets
    rng = np.random.default_rng(3)
    z = rng.standard_normal(7)
    idx, _ = O.route_topk(z, 3, False)
    best = max(itertools.combinations(range(7), 3), key=lambda c: sum(z[list(c)]))
    assert sorted(idx[0].tolist()) == sorted(best)


def test_softmax_closed_form_and_shift_invariance():
    p = O.softmax([0.0, math.log(3.0)])
    np.testing.assert_allclose(p, [0.25, 0.75], rtol=1e-15)
    z = np.array([1000.0, 1001.0, 999.0])      # would overflow without max subtraction
    np.testing.assert_allclose(O.softmax(z), O.softmax(z - 1000.0), rtol=1e-15)


def test_router_logits_is_a_matvec_and_bf16_decode_is_exact():
    rng = np.random.default_rng(4)
    W = rng.standard_normal((6, 16)).astype(np.float32)
    x = rng.standard_normal(16).astype(np.float32)
    b = rng.standard_normal(6).astype(np.float32)
    ref = torch.from_numpy(W).double() @ torch.from_numpy(x).double() + torch.from_numpy(b).double()
    np.testing.assert_allclose(O.router_logits(W, x, b), ref.numpy(), rtol=1e-14)
    # bf16 bit patterns decode exactly: compare with torch's own bfloat16
    tb = torch.from_numpy(W).to(torch.bfloat16)
    bits = tb.view(torch.int16).numpy().view(np.uint16)
    assert (O.to_f64(bits) == tb.double().numpy()).all()
    # asymmetric W: a transposed operand would fail the shape or the value
    assert O.router_logits(W, x).shape == (6,)


# ==================================================================== O2 EAM update
def test_eam_update_row_sums_and_partial_rows():
    L, E, k, n_tok = 5, 9, 3, 7
    rng = np.random.default_rng(5)
    eam = np.zeros((L, E), dtype=np.int64)
    for t in range(n_tok):
        for l in range(L):
            idx = rng.choice(E, size=k, replace=False)
            before = eam.copy()
            O.eam_update(eam, l, idx)
            assert eam[l].sum() == before[l].sum() + k          # each token adds k to row l
            assert (np.delete(eam, l, 0) == np.delete(before, l, 0)).all()
            assert (eam[l, idx] == before[l, idx] + 1).all()
    assert (eam.sum(axis=1) == n_tok * k).all()                  # Sec. 4.3 row-sum property
    assert eam.sum() == k * L * n_tok
    assert eam.max() <= n_tok                                    # M[i][j] in {0..n}


def test_eam_update_iteration_level_rows_above_current_layer_stay_zero():
    L, E = 4, 6
    eam = np.zeros((L, E), dtype=np.int64)
    for l in range(L):
        O.eam_update(eam, l, [l % E, (l + 1) % E])
        assert (eam[l + 1:] == 0).all() and (eam[:l + 1].sum(axis=1) == 2).all()
    with pytest.raises(ValueError):
        O.eam_update(eam, L, [0])
    with pytest.raises(ValueError):
        O.eam_update(eam, 0, [E])


# ==================================================================== O3 EAMC match
def _brute_cosine(a, b):
    a = [int(v) for v in np.asarray(a).reshape(-1)]
    b = [int(v) for v in np.asarray(b).reshape(-1)]
    d = sum(x * y for x, y in zip(a, b))
    na = sum(x * x for x in a)
    nb = sum(y * y for y in b)
    if na == 0 or nb == 0:
        return Fraction(0), 0.0
    return Fraction(d * d, na * nb), d / math.sqrt(na * nb)


def test_match_brute_force_tiny_exact():
    rng = np.random.default_rng(6)
    for trial in range(200):
        N, L, E = rng.integers(1, 9), rng.integers(1, 4), rng.integers(1, 4)
        T = rng.integers(0, 4, size=(N, L, E))
        q = rng.integers(0, 4, size=(L, E))
        best, sim, sims = O.eamc_match(T, q)
        keys = [_brute_cosine(q, T[t]) for t in range(N)]
        want = max(range(N), key=lambda t: (keys[t][0], -t))   # ties -> lowest index
        assert best == want
        for t in range(N):
            assert abs(sims[t] - keys[t][1]) <= 1e-15
        assert sim == sims[best]


def test_match_known_values():
    T = np.array([[[1, 1]], [[0, 5]], [[2, 0]], [[0, 0]]])
    best, sim, sims = O.eamc_match(T, np.array([[3, 0]]))
    np.testing.assert_allclose(sims, [1 / math.sqrt(2), 0.0, 1.0, 0.0], rtol=1e-15)
    assert best == 2 and sim == 1.0


def test_match_self_similarity_scale_invariance_and_ties():
    rng = np.random.default_rng(7)
    T = rng.integers(0, 50, size=(12, 3, 5))
    q = T[7].copy()
    best, sim, _ = O.eamc_match(T, q)
    assert best == 7 and abs(sim - 1.0) < 1e-15
    T2 = T.copy()
    T2[3] = 4 * T[7]                        # a scaled copy ties exactly; lowest index wins
    best, sim, sims = O.eamc_match(T2, q)
    assert best == 3 and abs(sims[3] - sims[7]) < 1e-15
    T3 = T.copy()
    T3[5] *= 9                              # scaling any trace leaves every similarity unchanged
    _, _, s_a = O.eamc_match(T, T[1] + 1)
    _, _, s_b = O.eamc_match(T3, T[1] + 1)
    np.testing.assert_allclose(s_a, s_b, rtol=1e-15)
    # scaling the query changes nothing either
    assert O.eamc_match(T, 3 * q)[0] == 7


def test_match_degenerate_inputs():
    assert O.eamc_match(np.zeros((0, 2, 3), dtype=np.int32), np.ones((2, 3)))[:2] == (-1, 0.0)
    T = np.ones((3, 2, 2), dtype=np.int32)
    best, sim, sims = O.eamc_match(T, np.zeros((2, 2), dtype=np.int32))    # empty query
    assert best == 0 and sim == 0.0 and (sims == 0).all() and not np.isnan(sims).any()
    T[0] = 0                                                               # empty trace
    best, sim, sims = O.eamc_match(T, np.ones((2, 2), dtype=np.int32))
    assert best == 1 and sims[0] == 0.0


def test_match_equals_dense_matvec_of_normalised_rows():
    # App. B.1 describes the search as a matrix multiplication: check against torch in fp64
    rng = np.random.default_rng(8)
    T = rng.integers(0, 300, size=(50, 6, 16))
    q = rng.integers(0, 40, size=(6, 16))
    _, _, sims = O.eamc_match(T, q)
    Tn = torch.nn.functional.normalize(torch.from_numpy(T.reshape(50, -1)).double(), dim=1)
    qn = torch.nn.functional.normalize(torch.from_numpy(q.reshape(-1)).double(), dim=0)
    np.testing.assert_allclose(sims, (Tn @ qn).numpy(), rtol=1e-13)


def test_match_exact_rank_agrees_with_fp64_and_finds_planted_group():
    from moei_inputs import get_config, eamc_traces, make_request
    cfg = get_config("C2").scaled(N=200)
    T, cl, _ = eamc_traces(cfg, threads=4)
    req = make_request(cfg, rid=3, decode=1)
    best, sim, sims = O.eamc_match(T, req.prefill_eam)
    top = sims.max()
    assert sims[best] == top and best == int(np.nonzero(sims == top)[0][0])
    assert cl[best] == req.source          # soft structure check: same activation group
    assert sim > 0.9


def test_match_topm_against_library_sort_and_brute_force():
    rng = np.random.default_rng(81)
    # distinct similarities: the order is that of a library cosine + stable sort
    T = rng.integers(0, 300, size=(40, 4, 8))
    q = rng.integers(0, 40, size=(4, 8))
    Tn = torch.nn.functional.normalize(torch.from_numpy(T.reshape(40, -1)).double(), dim=1)
    qn = torch.nn.functional.normalize(torch.from_numpy(q.reshape(-1)).double(), dim=0)
    lib = (Tn @ qn).numpy()
    assert np.unique(lib).size == 40
    order = np.argsort(-lib, kind="stable")
    for m in (1, 2, 5, 16, 40, 64):
        idx, sims = O.eamc_match_topm(T, q, m)
        assert idx == order[:m].tolist()
        np.testing.assert_allclose(sims, lib[order[:m]], rtol=1e-13)
    assert O.eamc_match_topm(T, q, 1)[0] == [O.eamc_match(T, q)[0]]
    # tiny cases with many exact ties: exact fractions, ties by ascending index
    for trial in range(150):
        N, L, E = rng.integers(1, 9), rng.integers(1, 3), rng.integers(1, 4)
        T = rng.integers(0, 3, size=(N, L, E))
        q = rng.integers(0, 3, size=(L, E))
        keys = [_brute_cosine(q, T[t])[0] for t in range(N)]
        want = sorted(range(N), key=lambda t: (-keys[t], t))
        for m in (1, 3, N, N + 2):
            assert O.eamc_match_topm(T, q, m)[0] == want[:m]


def test_match_topm_ties_prefix_and_degenerate_inputs():
    rng = np.random.default_rng(82)
    T = rng.integers(1, 50, size=(10, 2, 6))
    q = T[6].copy()
    T[2] = 3 * T[6]                          # scaled copies tie exactly at similarity 1
    T[9] = 5 * T[6]
    idx, sims = O.eamc_match_topm(T, q, 4)
    assert idx[:3] == [2, 6, 9] and all(abs(s - 1.0) < 1e-15 for s in sims[:3])
    for m in range(1, 10):                   # each list is a prefix of the next
        assert O.eamc_match_topm(T, q, m + 1)[0][:m] == O.eamc_match_topm(T, q, m)[0]
    assert sorted(O.eamc_match_topm(T, q, 99)[0]) == list(range(10))
    assert O.eamc_match_topm(np.zeros((0, 2, 3), dtype=np.int32), np.ones((2, 3)), 3) == ([], [])
    assert O.eamc_match_topm(T, q, 0) == ([], [])
    # an all-zero query: every similarity is 0, the order is the index order
    assert O.eamc_match_topm(T, np.zeros((2, 6), dtype=np.int64), 3) == ([0, 1, 2], [0.0, 0.0, 0.0])


def test_aggregated_matches_hand_worked_priorities():
    # two matched EAMs, cells summed, rows normalised, proximity applied (Sec. 4.5, steps 2-3)
    Ta = np.array([[1, 0], [1, 1], [4, 0]])
    Tb = np.array([[1, 2], [0, 2], [0, 4]])
    agg = O.aggregate_matches(np.stack([Ta, Tb]), [0, 1])
    assert agg.tolist() == [[2, 2], [1, 3], [4, 4]]
    P, V, pf, ev = O.expert_priority(agg, 0, np.zeros((3, 2), dtype=bool), 0.0)
    # layer 1: (1/4, 3/4) * (1 - 1/3); layer 2: (1/2, 1/2) * (1 - 2/3)
    np.testing.assert_allclose(P, [[0, 0], [1 / 6, 1 / 2], [1 / 6, 1 / 6]], rtol=1e-15)
    assert pf == [3, 2, 4, 5]                # 1/2 first; the three equal 1/6 cells by flat id


# ==================================================================== O4 priorities
def test_priority_worked_example_from_the_paper():
    g = json.load(open(os.path.join(GOLD, "alg1_worked_example.json")))
    eam = np.array(g["eam"])
    L, E = g["L"], g["E"]
    eps = 2.0 ** g["eps_log2"]
    res = np.ones((L, E), dtype=bool)
    P, V, pf, ev = O.expert_priority(eam, 0, res, eps)
    assert ev == g["evict_order_all_resident"]
    for key, (an, ad, bn, bd) in ((k, v) for k, v in g["evict_scores_fraction_of_eps"].items() if k != "comment"):
        i, j = map(int, key.split(","))
        want = Fraction(an, ad) + Fraction(bn, bd) * Fraction(1, 2 ** 20)
        assert abs(V[i, j] - float(want)) <= 1e-16 + 2e-16 * float(want)
    # the narrative: E[2,2] is kept, E[2,1]/E[3,1] go first
    keep = g["paper_retained_0based"][0] * E + g["paper_retained_0based"][1]
    cands = sorted(i * E + j for i, j in g["paper_evict_candidates_0based"])
    assert sorted(ev[:2]) == cands and ev.index(keep) >= 4
    # prefetch at l = 0 with nothing resident
    P, V, pf, ev = O.expert_priority(eam, 0, np.zeros((L, E), dtype=bool), eps)
    want = [[0.0, 0.0], [0.0, 2 / 3], [0.0, 1 / 3]]
    np.testing.assert_allclose(P, want, rtol=1e-15)
    assert pf == g["prefetch_order_l0_none_resident"] and ev == []


def _exact_orders(T, l, res, eps_frac, excl):
    L, E = T.shape
    Pk, Vk = {}, {}
    for i in range(L):
        R = int(T[i].sum())
        for j in range(E):
            f = i * E + j
            Vk[f] = (int(T[i, j]) + eps_frac) * Fraction(L - i, L) / (R if R else 1)
            Pk[f] = Fraction(int(T[i, j]), R) * (1 - Fraction(i - l, L)) if (i > l and R) else Fraction(0)
    pf = sorted((f for f in Pk if f // E > l and Pk[f] > 0 and not res.reshape(-1)[f]), key=lambda f: (-Pk[f], f))
    ev = sorted((f for f in Vk if res.reshape(-1)[f] and f not in excl), key=lambda f: (Vk[f], f))
    return Pk, Vk, pf, ev


def test_priority_orders_equal_exact_rational_orders():
    rng = np.random.default_rng(9)
    eps = 2.0 ** -20
    for trial in range(150):
        L, E = int(rng.integers(1, 7)), int(rng.integers(1, 7))
        T = rng.integers(0, 5, size=(L, E)) * rng.integers(0, 2, size=(L, 1))   # some empty rows
        l = int(rng.integers(-1, L))
        res = rng.integers(0, 2, size=(L, E)).astype(bool)
        excl = set(int(v) for v in rng.choice(L * E, size=min(2, L * E), replace=False))
        P, V, pf, ev = O.expert_priority(T, l, res, eps, excl)
        Pk, Vk, pf_x, ev_x = _exact_orders(T, l, res, Fraction(1, 2 ** 20), excl)
        assert pf == pf_x and ev == ev_x
        for f in range(L * E):
            assert abs(P[f // E, f % E] - float(Pk[f])) <= 2e-16 * float(Pk[f])
            assert abs(V[f // E, f % E] - float(Vk[f])) <= 2e-16 * float(Vk[f])


def test_priority_monotone_in_layer_distance_and_scale_free():
    L, E = 8, 4
    T = np.tile(np.array([5, 3, 0, 2]), (L, 1))          # identical rows: only the layer term varies
    eps = 2.0 ** -20
    P, V, pf, ev = O.expert_priority(T, 2, np.zeros((L, E), bool), eps)
    assert (P[:3] == 0).all()                             # nothing to prefetch at or below l
    for j in (0, 1, 3):
        assert (np.diff(P[3:, j]) < 0).all()              # strictly decreasing in i - l
        assert (np.diff(V[:, j]) < 0).all()               # layer decay starts at the first layer
    assert (P[:, 2] == 0).all() and all(f % E != 2 for f in pf)   # zero = predicted inactive
    np.testing.assert_allclose(P[3, 0], (5 / 10) * (1 - 1 / 8), rtol=1e-15)
    np.testing.assert_allclose(V[7, 1], (3 + eps) * (1 - 7 / 8) / 10, rtol=1e-15)
    P2, V2, pf2, _ = O.expert_priority(7 * T, 2, np.zeros((L, E), bool), eps)
    np.testing.assert_array_equal(P2, P)                  # row normalisation removes the scale
    assert pf2 == pf
    np.testing.assert_allclose(V2, V, rtol=0, atol=eps)   # up to the eps term
    # residents are not prefetch candidates, non-residents are not eviction candidates
    res = np.zeros((L, E), bool); res[4, 0] = True
    _, _, pf3, ev3 = O.expert_priority(T, 2, res, eps)
    assert 4 * E not in pf3 and ev3 == [4 * E]
    assert O.expert_priority(T, 2, res, eps, exclude=[4 * E])[3] == []


def test_aggregate_matches_sums_cells():
    T = np.arange(24).reshape(4, 2, 3)
    assert (O.aggregate_matches(T, [1]) == T[1]).all()
    assert (O.aggregate_matches(T, [1, 3, -1, 1]) == 2 * T[1] + T[3]).all()
    assert (O.aggregate_matches(T, [-1]) == 0).all()


# ========================================================================== O5 FFN
def test_ffn_closed_form_scalar():
    # H = I = 1: g = 1, silu(1) = 1/(1+e^-1), u = 6, o = 4 * silu(1) * 6
    y = O.swiglu_expert(np.array([2.0]), np.array([[0.5]]), np.array([[3.0]]), np.array([[4.0]]))
    np.testing.assert_allclose(y, [24.0 / (1.0 + math.exp(-1.0))], rtol=1e-15)


def test_ffn_matches_torch_fp64_library_ops():
    rng = np.random.default_rng(10)
    H, I = 24, 40                               # H != I: a transposed operand cannot pass
    x = rng.standard_normal(H)
    ex = [(rng.standard_normal((I, H)), rng.standard_normal((I, H)), rng.standard_normal((H, I))) for _ in range(3)]
    gates = [0.5, 0.25, 1.0]
    y = O.expert_ffn(x, ex, gates)
    xt = torch.from_numpy(x)
    ref = sum(w * (torch.from_numpy(Wd) @ (torch.nn.functional.silu(torch.from_numpy(Wg) @ xt) * (torch.from_numpy(Wu) @ xt)))
              for (Wg, Wu, Wd), w in zip(ex, gates))
    np.testing.assert_allclose(y, ref.numpy(), rtol=1e-12, atol=1e-12)
    # gate and up are not interchangeable: swapping them changes the result
    y_sw = O.expert_ffn(x, [(Wu, Wg, Wd) for Wg, Wu, Wd in ex], gates)
    assert np.abs(y - y_sw).max() > 1e-3


def test_ffn_special_cases():
    rng = np.random.default_rng(11)
    H, I = 8, 12
    x = rng.standard_normal(H)
    Wg, Wu, Wd = rng.standard_normal((I, H)), rng.standard_normal((I, H)), rng.standard_normal((H, I))
    assert (O.expert_ffn(x, [(np.zeros((I, H)), Wu, Wd)], [1.0]) == 0).all()     # silu(0) = 0
    y1 = O.expert_ffn(x, [(Wg, Wu, Wd)], [1.0])
    np.testing.assert_allclose(O.expert_ffn(x, [(Wg, Wu, Wd)], [0.3]), 0.3 * y1, rtol=1e-14)  # linear in w_e
    np.testing.assert_allclose(O.expert_ffn(x, [(Wg, Wu, Wd)] * 2, [0.3, 0.7]), y1, rtol=1e-14)
    assert (O.expert_ffn(x, [], []) == 0).all()
    # stored bf16 inputs: decoded exactly, then plain fp64
    from moei_inputs import f32_to_bf16_bits, bf16_bits_to_f32
    xb = f32_to_bf16_bits(x.astype(np.float32))
    Wb = [f32_to_bf16_bits(w.astype(np.float32)) for w in (Wg, Wu, Wd)]
    yb = O.expert_ffn(xb, [tuple(Wb)], [1.0])
    yf = O.expert_ffn(bf16_bits_to_f32(xb).astype(np.float64), [tuple(bf16_bits_to_f32(w).astype(np.float64) for w in Wb)], [1.0])
    np.testing.assert_array_equal(yb, yf)


# ============================================================== O6 cache retrieval
def _simulate_dict(L, E, S, steps):
    """Independent dictionary-based replay of Alg. 1 (cache: id -> slot)."""
    cache = {f: f for f in range(min(S, L * E))}
    log = []
    for layer, picks, ev in steps:
        need = {layer * E + p for p in picks}
        evq = list(ev)
        for p in picks:
            fid = layer * E + p
            if fid in cache:                                   # Alg. 1 steps 1-3
                log.append((fid, True, -1, cache[fid])); continue
            used = set(cache.values())
            if len(cache) < S:                                 # steps 4-7
                slot = min(s for s in range(S) if s not in used); victim = -1
            else:                                              # steps 8-19
                victim = next((c for c in evq if c in cache and c not in need), None)
                if victim is None:
                    victim = next(o for o in (next(k for k, v in cache.items() if v == s) for s in range(S)) if o not in need)
                else:
                    evq = evq[evq.index(victim) + 1:]
                slot = cache.pop(victim)
            cache[fid] = slot
            log.append((fid, False, victim, slot))
    return log, cache


def test_cache_retrieval_against_independent_simulation_and_invariants():
    rng = np.random.default_rng(12)
    for S, warm in [(12, True), (5, False), (3, True)]:
        L, E, k = 4, 8, 2
        c = O.ExpertCache(L, E, S, warm=warm)
        steps, got = [], []
        for it in range(40):
            for layer in range(L):
                picks = rng.choice(E, size=k, replace=False).tolist()
                resident = [f for f in range(L * E) if c.slot_of[f] >= 0 and f not in {layer * E + p for p in picks}]
                ev = rng.permutation(resident).tolist()
                if it % 7 == 3:
                    ev = ev[:1]                                # exhausted order -> fallback rule
                steps.append((layer, picks, ev))
                ev_now = c.retrieve(layer, picks, ev)
                got += ev_now
                # invariants: capacity, inverse maps, picks resident, victim never a current pick
                assert (c.slot_of >= 0).sum() <= S
                for f in range(L * E):
                    if c.slot_of[f] >= 0:
                        assert c.owner[c.slot_of[f]] == f
                for s in range(S):
                    if c.owner[s] >= 0:
                        assert c.slot_of[c.owner[s]] == s
                for p in picks:
                    assert c.slot_of[layer * E + p] >= 0
                for fid, hit, victim, slot in ev_now:
                    assert victim not in {layer * E + p for p in picks}
        if warm:                                               # the dictionary replay starts full too
            log, _ = _simulate_dict(L, E, S, steps)
            assert log == got
    with pytest.raises(ValueError):
        O.ExpertCache(2, 4, 1).retrieve(0, [0, 1], [])


def test_lru_policy_equals_textbook_ordered_dict_lru():
    # one pick per call: no pick protection comes into play and the rule is the textbook one
    from collections import OrderedDict
    rng = np.random.default_rng(21)
    L, E, S = 3, 6, 5
    c = O.ExpertCache(L, E, S, warm=False, policy="lru")
    book = OrderedDict()
    for step in range(600):
        layer = step % L
        p = int(rng.integers(0, E)) if rng.random() < 0.7 else int(rng.integers(0, 2))
        fid = layer * E + p
        hit_book = fid in book
        if hit_book:
            book.move_to_end(fid)
        else:
            if len(book) == S:
                book.popitem(last=False)
            book[fid] = True
        (f, hit, victim, slot), = c.retrieve(layer, [p])
        assert hit == hit_book
        assert set(np.nonzero(c.slot_of >= 0)[0].tolist()) == set(book.keys())
    # several picks per call: a resident later pick is never the victim of an earlier one
    c = O.ExpertCache(2, 4, 2, warm=False, policy="lru")
    c.retrieve(0, [0, 1])                      # slots: 0 -> e0, 1 -> e1; e0 is the older
    ev = c.retrieve(0, [2, 0])                 # e2 misses; the LRU slot holds e0, a current pick -> e1 goes
    assert ev[0][2] == 1 and ev[1][1] is True
    # warm start: all stamps equal, ties to the lowest slot
    c = O.ExpertCache(2, 4, 3, warm=True, policy="lru")
    assert c.retrieve(1, [3])[0][2:] == (0, 0)


def test_count_policy_hand_worked_and_brute_force():
    c = O.ExpertCache(1, 6, 3, warm=False, policy="count")
    for p in (0, 0, 0, 1, 2, 2):
        c.retrieve(0, [p])
    assert c.retrieve(0, [3])[0][2] == 1        # counts 3, 1, 2 -> expert 1 leaves
    assert c.retrieve(0, [4])[0][2] == 3        # counts 3, 2, 1(new) -> the newcomer leaves
    c.retrieve(0, [4])                          # now e4 has count 2 = e2's: tie -> lowest id
    assert c.retrieve(0, [5])[0][2] == 2
    rng = np.random.default_rng(22)
    L, E, S, k = 3, 5, 4, 2
    c = O.ExpertCache(L, E, S, warm=True, policy="count")
    counts = {}
    res = set(range(S))
    for step in range(300):
        layer = step % L
        picks = rng.choice(E, size=k, replace=False).tolist()
        need = {layer * E + p for p in picks}
        want = []
        for p in picks:
            f = layer * E + p
            counts[f] = counts.get(f, 0) + 1
            if f in res:
                want.append(-1); continue
            v = min((x for x in res if x not in need), key=lambda x: (counts.get(x, 0), x))
            res.remove(v); res.add(f); want.append(v)
        assert [e[2] for e in c.retrieve(layer, picks)] == want
        assert set(np.nonzero(c.slot_of >= 0)[0].tolist()) == res
    with pytest.raises(ValueError):
        O.ExpertCache(1, 2, 1, policy="fifo")


def test_prefetch_hand_worked_admission_rule():
    # 3 layers x 2 experts, 3 slots holding experts 0, 1 and 4
    c = O.ExpertCache(3, 2, 3, warm=False)
    for layer, p in ((0, 0), (0, 1), (2, 0)):
        c.retrieve(layer, [p], [])
    V = np.array([0.9, 0.1, 0.5, 0.3, 0.2, 0.6])
    # candidates 5 then 2 then 3; victims cheapest first: 1 (0.1), 4 (0.2), 0 (0.9)
    got = c.prefetch([5, 2, 3], [1, 4, 0], V, depth=3)
    #  5 (0.6) > 1 (0.1): takes slot of 1.  2 (0.5) > 4 (0.2): takes slot of 4.  3 (0.3) < 0 (0.9): skipped
    assert got == [(5, 1, 1), (2, 4, 2)]
    assert sorted(np.nonzero(c.slot_of >= 0)[0].tolist()) == [0, 2, 5]
    # depth limits the candidates considered; a resident candidate is passed over
    c2 = O.ExpertCache(3, 2, 3, warm=True)                   # holds 0, 1, 2
    assert c2.prefetch([2, 5, 4], [1, 0], V, depth=2) == [(5, 1, 1)]
    # a protected victim and a victim that has left are passed over
    c3 = O.ExpertCache(3, 2, 3, warm=True)
    c3.retrieve(1, [1], [1])                                 # expert 3 replaces expert 1 in slot 1
    assert c3.prefetch([5], [1, 0, 2], V, depth=1, protect=[0]) == [(5, 2, 2)]
    # free slots are used first, lowest first, and need no admission
    c4 = O.ExpertCache(3, 2, 3, warm=False)
    assert c4.prefetch([1, 0], [], np.zeros(6), depth=5) == [(1, -1, 0), (0, -1, 1)]
    # scores that differ only below fp32 resolution do not admit (compared as handed over, in fp32)
    Vt = np.array([0.5, 0.5 + 1e-12, 0.0, 0.0, 0.0, 0.0])
    c5 = O.ExpertCache(3, 2, 1, warm=True)                   # holds expert 0
    assert c5.prefetch([1], [0], Vt, depth=1) == []
    assert O.ExpertCache(3, 2, 1, warm=True).prefetch([1], [0], np.array([0.5, 0.5001, 0, 0, 0, 0]), 1) == [(1, 0, 0)]


def test_prefetch_invariants_random():
    rng = np.random.default_rng(23)
    L, E, S, k = 4, 6, 7, 2
    c = O.ExpertCache(L, E, S, warm=True)
    for step in range(300):
        layer = step % L
        picks = rng.choice(E, size=k, replace=False).tolist()
        need = [layer * E + p for p in picks]
        V = rng.random(L * E)
        res = [f for f in range(L * E) if c.slot_of[f] >= 0 and f not in need]
        ev = sorted(res, key=lambda f: (V[f], f))
        c.retrieve(layer, picks, ev)
        pf = [f for f in rng.permutation(L * E).tolist() if f // E > layer and c.slot_of[f] < 0]
        before = set(np.nonzero(c.slot_of >= 0)[0].tolist())
        out = c.prefetch(pf, ev, V, depth=3, protect=need)
        after = set(np.nonzero(c.slot_of >= 0)[0].tolist())
        assert len(out) <= 3 and len(after) <= S and all(f in after for f in need)
        for fid, victim, slot in out:
            assert fid not in before and c.owner[slot] == fid and victim not in need
            if victim >= 0:
                assert np.float32(V[fid]) > np.float32(V[victim]) and victim not in after
        for f in after:
            assert c.owner[c.slot_of[f]] == f


def test_cache_cold_start_fills_lowest_free_slots():
    c = O.ExpertCache(2, 4, 3, warm=False)
    ev = c.retrieve(0, [2, 0], [])
    assert ev == [(2, False, -1, 0), (0, False, -1, 1)]
    ev = c.retrieve(1, [1, 3], [2, 0])
    assert ev == [(5, False, -1, 2), (7, False, 2, 0)]       # one free slot, then evict the order's head
    ev = c.retrieve(1, [1, 2], [0, 7])
    assert ev == [(5, True, -1, 2), (6, False, 0, 1)]


def test_retrieval_passes_over_needed_and_departed_eviction_candidates():
    # Alg. 1 by hand on 2 layers x 3 experts; 3 slots, holding experts 0, 1, 2 (flat ids) at the start
    c = O.ExpertCache(2, 3, 3, warm=True)
    assert c.retrieve(0, [1], [1, 2, 0]) == [(1, True, -1, 1)]
    # layer 1 needs flat ids 3 and 4, both misses; the order's head (3) is not resident: passed over
    assert c.retrieve(1, [0, 1], [3, 2, 0, 1]) == [(3, False, 2, 2), (4, False, 0, 0)]
    # slots now hold 4, 1, 3; the order's head (4) is needed by this very call and stays
    assert c.retrieve(1, [1, 2], [4, 3, 1]) == [(4, True, -1, 0), (5, False, 3, 2)]
    # slots hold 4, 1, 5; expert 2 left long ago and nobody needs it: a stale entry, passed over
    assert c.retrieve(0, [0], [2, 1]) == [(0, False, 1, 1)]
    assert sorted(np.nonzero(c.slot_of >= 0)[0].tolist()) == [0, 4, 5]
    for f in (0, 4, 5):
        assert c.owner[c.slot_of[f]] == f


def test_a_prefetched_expert_is_the_most_recent_use_under_lru():
    c = O.ExpertCache(1, 4, 2, warm=False, policy="lru")
    c.retrieve(0, [0], [])                                      # slot 0, stamp 1
    assert c.prefetch([1], [], np.zeros(4), depth=1) == [(1, -1, 1)]   # slot 1, stamp 2
    c.retrieve(0, [0], [])                                      # expert 0 used again: stamp 3
    # the least recently used is now the prefetched expert 1, not expert 0
    assert c.retrieve(0, [2], []) == [(2, False, 1, 1)]
    c2 = O.ExpertCache(1, 4, 2, warm=False, policy="lru")
    c2.retrieve(0, [0], [])
    c2.retrieve(0, [1], [])
    assert c2.prefetch([2], [0], np.array([0.0, 0.0, 1.0, 0.0]), depth=1) == [(2, 0, 0)]   # takes expert 0's slot
    # expert 2 was brought in after expert 1 was used: expert 1 is the older one
    assert c2.retrieve(0, [3], []) == [(3, False, 1, 1)]


# ============================================================ composite (via parts)
def test_decode_layer_composes_its_parts():
    from moei_inputs import get_config, eamc_traces, make_request, router_weights, expert_weights
    cfg = get_config("C1")
    T, _, _ = eamc_traces(cfg, threads=1)
    req = make_request(cfg, 0)
    eam = req.prefill_eam.astype(np.int64).copy()
    cache = O.ExpertCache(cfg.L, cfg.E, cfg.S)
    H, I = cfg.H, cfg.I

    def expert_of(fid):
        w = expert_weights(cfg, fid)
        return w[:I * H].reshape(I, H), w[I * H:2 * I * H].reshape(I, H), w[2 * I * H:].reshape(H, I)

    row0 = eam[0].sum()
    out = O.decode_layer(T, eam, cache, 0, router_weights(cfg, 0), req.bias[0], req.x[0, 0], expert_of,
                         lambda l: [], cfg.k, bool(cfg.renorm), 2.0 ** -20)
    assert eam[0].sum() == row0 + cfg.k
    idx, w = O.route_topk(out["logits"], cfg.k, True)
    assert (idx[0] == out["idx"]).all()
    y = O.expert_ffn(req.x[0, 0], [expert_of(int(j)) for j in idx[0]], w[0])
    np.testing.assert_array_equal(y, out["y"])
    assert out["best"] == O.eamc_match(T, eam)[0]


def _hand_step(m):
    """A layer step small enough to follow by hand: 3 layers x 4 experts, top-2 without
    renormalisation, an identity router, one-unit experts that only touch y[0]."""
    L, E = 3, 4
    T = np.array([[[4, 4, 0, 0], [0, 8, 0, 0], [0, 0, 0, 8]],
                  [[0, 0, 4, 4], [8, 0, 0, 0], [0, 0, 8, 0]]])
    cache = O.ExpertCache(L, E, 3, warm=False)
    cache.retrieve(0, [0, 2])                                   # slots 0, 1 hold flat ids 0 and 2
    cache.retrieve(1, [1])                                      # slot 2 holds flat id 5
    par = {0: (0.5, 1.0), 1: (-0.25, 2.0)}                      # expert -> (g, d); o = d silu(g x0) x1 e_0

    def mk(g, d):
        return (np.array([[g, 0.0, 0.0, 0.0]]), np.array([[0.0, 1.0, 0.0, 0.0]]), np.array([[d], [0.0], [0.0], [0.0]]))

    eam = np.zeros((L, E), dtype=np.int64)
    out = O.decode_layer(T, eam, cache, 0, np.eye(4), None, np.array([4.0, 3.0, 0.0, 0.0]),
                         lambda f: mk(*par.get(f, (9.0, 9.0))), lambda l: [mk(1.0, -1.0)], 2, False, 2.0 ** -20, m=m)
    return out, eam, cache


def test_decode_layer_hand_worked_step():
    out, eam, cache = _hand_step(1)
    silu = lambda t: t / (1.0 + math.exp(-t))
    z = np.array([4.0, 3.0, 0.0, 0.0])
    p = np.exp(z) / np.exp(z).sum()
    assert out["idx"].tolist() == [0, 1]
    np.testing.assert_allclose(out["w"], p[:2], rtol=1e-15)
    assert eam.tolist() == [[1, 1, 0, 0], [0, 0, 0, 0], [0, 0, 0, 0]]
    # the query (1, 1, 0, ...) meets trace 0 in <q, T> = 8, trace 1 in 0; |q|^2 = 2, |T_0|^2 = 160
    assert out["best"] == 0 and out["matched"] == [0]
    assert out["sim"] == pytest.approx(1.0 / math.sqrt(5.0), rel=1e-15)
    # prefetch scores from trace 0 at layer 0: (row-normalised cell) x (1 - (i - 0)/3)
    P = np.zeros((3, 4)); P[1, 1] = 2.0 / 3.0; P[2, 3] = 1.0 / 3.0
    np.testing.assert_allclose(out["P"], P, rtol=1e-15)
    assert out["pf_order"] == [11]                              # (1, 1) is resident already
    # eviction: residents 0, 2, 5 without the experts running now (0 and 1): V[2] ~ eps/8 < V[5] ~ 2/3
    assert out["ev_order"] == [2, 5]
    assert out["V"][0, 0] == pytest.approx((4 + 2.0 ** -20) / 8.0, rel=1e-15)
    assert out["V"][1, 1] == pytest.approx((8 + 2.0 ** -20) * (2.0 / 3.0) / 8.0, rel=1e-15)
    # Alg. 1: expert 0 hits slot 0; expert 1 misses, the cache is full, the order's head (2) gives up slot 1
    assert out["events"] == [(0, True, -1, 0), (1, False, 2, 1)]
    assert sorted(np.nonzero(cache.slot_of >= 0)[0].tolist()) == [0, 1, 5]
    # y[0] = p_0 silu(0.5 * 4) 3 + p_1 2 silu(-0.25 * 4) 3 - silu(4) 3 (the shared expert enters with weight 1)
    want = p[0] * silu(2.0) * 3.0 + p[1] * 2.0 * silu(-1.0) * 3.0 - silu(4.0) * 3.0
    np.testing.assert_allclose(out["y"], [want, 0.0, 0.0, 0.0], rtol=1e-14, atol=0)


def test_decode_layer_hand_worked_step_with_two_matches():
    out, _, _ = _hand_step(2)
    # both traces are returned (similarities 1/sqrt(5) and 0) and their cells are summed:
    # rows (4,4,4,4), (8,8,0,0), (0,0,8,8)
    assert out["matched"] == [0, 1] and out["best"] == 0
    P = np.zeros((3, 4)); P[1, 0] = P[1, 1] = 0.5 * 2.0 / 3.0; P[2, 2] = P[2, 3] = 0.5 / 3.0
    np.testing.assert_allclose(out["P"], P, rtol=1e-15)
    assert out["pf_order"] == [4, 10, 11]                       # 5 is resident; equal scores by ascending id
    assert out["ev_order"] == [2, 5]                            # V[2] = (4 + eps)/16 < V[5] = (8 + eps)(2/3)/16


def test_decode_layer_hand_worked_step_with_prefetch():
    """Layer 1 of a 4-layer x 4-expert model, top-2, identity router, prefetch depth 2.  The numbers are
    chosen so that the prefetch order (by P) and the admission measure (V, Alg. 1's score) disagree:
    the first candidate has the larger P but the smaller V and is turned down, the second is admitted.
    Everything below is worked out by hand in fractions (eps = 2^-20 only breaks exact zeros)."""
    L, E = 4, 4
    T = np.array([[[2, 2, 0, 0], [3, 2, 3, 0], [0, 0, 6, 4], [0, 5, 0, 0]],      # row sums 4, 8, 10, 5
                  [[0, 0, 5, 5], [0, 0, 0, 7], [7, 0, 0, 0], [0, 0, 0, 3]]])     # orthogonal to the query
    cache = O.ExpertCache(L, E, 4, warm=False)
    cache.retrieve(0, [0, 2])                                   # slots 0, 1: flat ids 0 and 2
    cache.retrieve(1, [1, 2])                                   # slots 2, 3: flat ids 5 and 6
    par = {5: (0.5, 1.0), 4: (-0.25, 2.0)}                      # expert -> (g, d); o = d silu(g x0) x1 e_0

    def mk(g, d):
        return (np.array([[g, 0.0, 0.0, 0.0]]), np.array([[0.0, 1.0, 0.0, 0.0]]), np.array([[d], [0.0], [0.0], [0.0]]))

    def run(depth):
        c = O.ExpertCache(L, E, 4, warm=False)
        c.retrieve(0, [0, 2])
        c.retrieve(1, [1, 2])
        eam = np.zeros((L, E), dtype=np.int64)
        eam[0, :2] = 1                                          # this iteration's layer 0 picked experts 0 and 1
        out = O.decode_layer(T, eam, c, 1, np.eye(4), None, np.array([3.0, 4.0, 0.0, 0.0]),
                             lambda f: mk(*par.get(f, (9.0, 9.0))), lambda l: [mk(1.0, -1.0)], 2, False, 2.0 ** -20,
                             prefetch_depth=depth)
        return out, eam, c

    out, eam, c = run(2)
    assert out["idx"].tolist() == [1, 0]                        # logits (3, 4, 0, 0)
    assert eam.tolist() == [[1, 1, 0, 0], [1, 1, 0, 0], [0, 0, 0, 0], [0, 0, 0, 0]]
    # <q, T_0> = 2 + 2 + 3 + 2 = 9, |q|^2 = 4, |T_0|^2 = 107; <q, T_1> = 0
    assert out["best"] == 0 and out["sim"] == pytest.approx(9.0 / (2.0 * math.sqrt(107.0)), rel=1e-15)
    # prefetch scores at l = 1: cell / row sum x (L - i + l) / L for i > 1
    P = np.zeros((L, E)); P[2, 2] = 0.6 * 0.75; P[2, 3] = 0.4 * 0.75; P[3, 1] = 1.0 * 0.5
    np.testing.assert_allclose(out["P"], P, rtol=1e-15)
    assert out["pf_order"] == [13, 10, 11]                      # 0.5 > 0.45 > 0.3, none of them resident
    # eviction scores (cell + eps)(L - i) / (row sum x L): V[6] = 9/32, V[10] = 3/10, V[13] = 1/4
    e = 2.0 ** -20
    assert out["V"][1, 2] == pytest.approx((3 + e) * 3 / 32, rel=1e-15)
    assert out["V"][2, 2] == pytest.approx((6 + e) * 2 / 40, rel=1e-15)
    assert out["V"][3, 1] == pytest.approx((5 + e) * 1 / 20, rel=1e-15)
    # residents 0, 2, 5, 6 without the experts that run now (5 and 4): V[2] ~ eps/4 < V[6] = 9/32 < V[0] = 1/2
    assert out["ev_order"] == [2, 6, 0]
    # Alg. 1: pick 1 (flat 5) hits slot 2; pick 0 (flat 4) misses, the cache is full, flat 2 gives up slot 1
    assert out["events"] == [(5, True, -1, 2), (4, False, 2, 1)]
    # prefetch: candidate 13 (P = 1/2) meets the cheapest remaining victim 6 (2 has left): V[13] = 1/4 is not
    # above V[6] = 9/32 -> turned down; candidate 10 (P = 0.45): V[10] = 3/10 > 9/32 -> takes slot 3 from 6
    assert out["prefetched"] == [(10, 6, 3)]
    assert c.owner.tolist() == [0, 4, 5, 10]
    assert sorted(np.nonzero(c.slot_of >= 0)[0].tolist()) == [0, 4, 5, 10]
    silu = lambda t: t / (1.0 + math.exp(-t))
    p = np.exp([3.0, 4.0, 0.0, 0.0]) / np.exp([3.0, 4.0, 0.0, 0.0]).sum()
    want = p[1] * silu(1.5) * 4.0 + p[0] * 2.0 * silu(-0.75) * 4.0 - silu(3.0) * 4.0
    np.testing.assert_allclose(out["y"], [want, 0.0, 0.0, 0.0], rtol=1e-14, atol=0)
    # depth 1 considers only candidate 13 and prefetches nothing; depth 3 adds candidate 11, whose
    # V = 1/5 is not above the next victim's (flat 0, V = 1/2); depth 0 never prefetches
    out1, _, c1 = run(1)
    assert out1["prefetched"] == [] and c1.owner.tolist() == [0, 4, 5, 6]
    out3, _, c3 = run(3)
    assert out3["prefetched"] == [(10, 6, 3)] and c3.owner.tolist() == [0, 4, 5, 10]
    out0, _, c0 = run(0)
    assert out0["prefetched"] == [] and c0.owner.tolist() == [0, 4, 5, 6]


# ================================================================ prefill iteration
def test_prefill_layer_against_dense_all_expert_formulation():
    # every expert applied to every token with dense library matmuls, then masked by the routing:
    # a different formulation of the same sum (torch, fp64)
    rng = np.random.default_rng(41)
    L, E, k, H, I, n = 3, 6, 2, 16, 12, 23
    Wr = rng.standard_normal((E, H))
    bias = rng.standard_normal(E)
    X = rng.standard_normal((n, H))
    Wg, Wu = rng.standard_normal((E, I, H)) * 0.3, rng.standard_normal((E, I, H)) * 0.3
    Wd = rng.standard_normal((E, H, I)) * 0.3
    Sg, Su, Sd = rng.standard_normal((I, H)) * 0.3, rng.standard_normal((I, H)) * 0.3, rng.standard_normal((H, I)) * 0.3
    layer = 1
    for renorm in (False, True):
        eam = rng.integers(0, 5, size=(L, E)).astype(np.int64)
        before = eam.copy()
        idx, w, Y = O.prefill_layer(eam, layer, Wr, bias, X, lambda f: (Wg[f % E], Wu[f % E], Wd[f % E]),
                                    lambda l: [(Sg, Su, Sd)], k, renorm)
        tX = torch.from_numpy(X)
        logits = tX @ torch.from_numpy(Wr).T + torch.from_numpy(bias)
        prob = torch.softmax(logits, dim=1)
        top = torch.topk(logits, k, dim=1)
        assert (top.indices.numpy() == idx).all()
        gate = torch.zeros((n, E), dtype=torch.float64)
        sel = prob.gather(1, top.indices)
        if renorm:
            sel = sel / sel.sum(dim=1, keepdim=True)
        gate.scatter_(1, top.indices, sel)
        np.testing.assert_allclose(w, sel.numpy(), rtol=1e-12)
        dense = torch.zeros((n, H), dtype=torch.float64)
        for e in range(E):
            g = tX @ torch.from_numpy(Wg[e]).T
            u = tX @ torch.from_numpy(Wu[e]).T
            dense += gate[:, e:e + 1] * ((torch.nn.functional.silu(g) * u) @ torch.from_numpy(Wd[e]).T)
        g = tX @ torch.from_numpy(Sg).T
        dense += (torch.nn.functional.silu(g) * (tX @ torch.from_numpy(Su).T)) @ torch.from_numpy(Sd).T
        np.testing.assert_allclose(Y, dense.numpy(), rtol=1e-10, atol=1e-12)
        # Sec. 4.3: the n tokens add n*k to row l, nothing elsewhere; the row is the histogram of the picks
        delta = eam - before
        assert delta[layer].sum() == n * k and (np.delete(delta, layer, axis=0) == 0).all()
        assert (delta[layer] == np.bincount(idx.reshape(-1), minlength=E)).all()


def test_prefill_layer_token_order_does_not_matter():
    rng = np.random.default_rng(42)
    L, E, k, H, I, n = 2, 5, 2, 8, 6, 11
    Wr, X = rng.standard_normal((E, H)), rng.standard_normal((n, H))
    ex = [(rng.standard_normal((I, H)), rng.standard_normal((I, H)), rng.standard_normal((H, I))) for _ in range(E)]
    e1, e2 = np.zeros((L, E), dtype=np.int64), np.zeros((L, E), dtype=np.int64)
    perm = rng.permutation(n)
    i1, w1, Y1 = O.prefill_layer(e1, 0, Wr, None, X, lambda f: ex[f % E], lambda l: [], k, True)
    i2, w2, Y2 = O.prefill_layer(e2, 0, Wr, None, X[perm], lambda f: ex[f % E], lambda l: [], k, True)
    assert (e1 == e2).all() and (i1[perm] == i2).all()
    np.testing.assert_array_equal(Y1[perm], Y2)
