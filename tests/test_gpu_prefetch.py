"""Cache policies and the prefetch step (Sec. 4.6-4.7) against the oracle: the sequences of
hits, victims, slots and prefetches must agree exactly, every slot must end up holding its
owner's weights, and FFN outputs computed from prefetched slots must be right (which is
what proves that readers wait for the copies).
"""
import numpy as np
import pytest
import torch

import moei_inputs as mi
from oracle import moei_oracle as O
from tests.helpers import EPS, dev, pack_bank, pick_clear_tokens, pinned, rel_max_err, split_expert

pytestmark = pytest.mark.gpu
FFN_TOL = 2e-4


@pytest.fixture(scope="module")
def m():
    import paper_2401_14361_amd as mod
    mod.lib()
    return mod


def _check_slot_contents(cache, ref, packed):
    torch.cuda.synchronize()
    for f in range(ref.slot_of.size):
        s = int(ref.slot_of[f])
        if s >= 0:
            assert (cache.slot_tensor(s).cpu().numpy() == packed[f % len(packed)]).all(), f


@pytest.mark.parametrize("policy", ["lru", "count"])
def test_comparison_policies_follow_the_oracle(m, policy):
    cfg = mi.get_config("C1").scaled(H=64, I=32)
    L, E, k, S = cfg.L, cfg.E, cfg.k, 7
    packed = pack_bank(m, cfg, mi.expert_bank(cfg, L * E, threads=2))
    cache = m.Cache(m.ModelDesc.from_config(cfg), S, pinned(packed))
    for warm in (True, False):
        cache.reset(S if warm else 0)
        cache.set_policy(policy)
        ref = O.ExpertCache(L, E, S, warm=warm, policy=policy)
        rng = np.random.default_rng(31)
        for it in range(40):
            for layer in range(L):
                picks = rng.choice(E, size=k, replace=False, p=np.arange(1, E + 1) / (E * (E + 1) / 2))
                want = ref.retrieve(layer, picks)
                slots, victims, n_miss = cache.retrieve(layer, picks, [])
                assert slots.tolist() == [w[3] for w in want]
                assert victims.tolist() == [w[2] for w in want]
                assert n_miss == sum(1 for w in want if not w[1])
        assert (cache.get_slots() == ref.slot_of).all()
        _check_slot_contents(cache, ref, packed)
    assert m.lib().moei_cache_set_policy(cache.h, 7) != 0          # unknown policy: refused
    assert b"unknown policy" in m.lib().moei_last_error()
    cache.close()


def test_a_prefetched_expert_is_the_most_recent_use_under_lru(m):
    # the hand-worked case of the oracle's pin, through the library
    cfg = mi.get_config("C1").scaled(H=64, I=32, L=1, E=4, k=1)
    packed = pack_bank(m, cfg, mi.expert_bank(cfg, 4, threads=2))
    cache = m.Cache(m.ModelDesc.from_config(cfg), 2, pinned(packed))
    cache.reset(0)
    cache.set_policy("lru")
    ref = O.ExpertCache(1, 4, 2, warm=False, policy="lru")
    V = np.array([0.0, 0.0, 1.0, 0.0], dtype=np.float32)
    for step in (("r", 0), ("p", 1), ("r", 0), ("r", 2), ("r", 1), ("p", 3), ("r", 0)):
        if step[0] == "r":
            want = ref.retrieve(0, [step[1]])
            slots, victims, n_miss = cache.retrieve(0, [step[1]], [])
            assert (slots.tolist(), victims.tolist()) == ([w[3] for w in want], [w[2] for w in want]), step
        else:
            ev = [int(f) for f in np.nonzero(ref.slot_of >= 0)[0]]
            want = ref.prefetch([step[1]], ev, np.where(np.arange(4) == step[1], 1.0, 0.0), depth=1)
            got = cache.prefetch([step[1]], ev, np.where(np.arange(4) == step[1], 1.0, 0.0).astype(np.float32), depth=1)
            assert [tuple(g) for g in got] == want, step
        assert (cache.get_slots() == ref.slot_of).all(), step
    cache.close()


def test_prefetch_step_follows_the_oracle_and_fills_the_slots(m):
    cfg = mi.get_config("C1").scaled(H=64, I=32, L=5)
    L, E, k, S = cfg.L, cfg.E, cfg.k, 9
    packed = pack_bank(m, cfg, mi.expert_bank(cfg, L * E, threads=2))
    cache = m.Cache(m.ModelDesc.from_config(cfg), S, pinned(packed))
    for warm in (True, False):
        cache.reset(S if warm else 0)
        ref = O.ExpertCache(L, E, S, warm=warm)
        rng = np.random.default_rng(32)
        n_issued = 0
        for it in range(40):
            for layer in range(L):
                picks = rng.choice(E, size=k, replace=False)
                need = [layer * E + int(p) for p in picks]
                V = (rng.integers(0, 12, size=L * E) / 8.0).astype(np.float32)   # many equal scores
                resident = [f for f in range(L * E) if ref.slot_of[f] >= 0 and f not in need]
                ev = sorted(resident, key=lambda f: (V[f], f))
                want = ref.retrieve(layer, picks, ev)
                slots, victims, _ = cache.retrieve(layer, picks, ev)
                assert slots.tolist() == [w[3] for w in want] and victims.tolist() == [w[2] for w in want]
                pf = [f for f in rng.permutation(L * E).tolist() if f // E > layer and ref.slot_of[f] < 0]
                depth = int(rng.integers(0, 6))
                want_pf = ref.prefetch(pf, ev, V, depth, need)
                got_pf = cache.prefetch(pf, ev, V, depth, need)
                assert got_pf == want_pf, (it, layer)
                n_issued += len(got_pf)
                assert (cache.get_slots() == ref.slot_of).all()
        assert n_issued > 20
        cache.join()
        _check_slot_contents(cache, ref, packed)
        cache.sync()
    # argument checks
    with pytest.raises(m.MoeiError):
        cache.prefetch([L * E], [], np.zeros(L * E), 1)
    with pytest.raises(m.MoeiError):
        cache.prefetch([1], [], np.zeros(L * E), 33)
    with pytest.raises(m.MoeiError):
        cache.set_prefetch(33)
    cache.close()
    nohost = m.Cache(m.ModelDesc.from_config(cfg), S)
    with pytest.raises(m.MoeiError):
        nohost.set_prefetch(2)
    with pytest.raises(m.MoeiError):
        nohost.prefetch([1], [], np.zeros(L * E), 1)
    nohost.close()


def _replay_prefetch(m, cfg, S, n_tokens, depth, match_m=1, rid=0):
    L, E, k = cfg.L, cfg.E, cfg.k
    T, _, _ = mi.eamc_traces(cfg, threads=4)
    req = mi.make_request(cfg, rid, decode=n_tokens + 8)
    tokens = pick_clear_tokens(cfg, req, n_tokens)
    bank = mi.expert_bank(cfg, L * E, threads=4)
    shared = mi.expert_bank(cfg.scaled(cid=cfg.cid + 50), max(L * cfg.n_shared, 1), threads=2)
    routers = [mi.router_weights(cfg, l) for l in range(L)]
    desc = m.ModelDesc.from_config(cfg)
    eamc = m.Eamc(desc, cfg.N, 4)
    eamc.load(T)
    cache = m.Cache(desc, S, pinned(pack_bank(m, cfg, bank)), pinned(pack_bank(m, cfg, shared)) if cfg.n_shared else None)
    cache.reset(min(S, L * E))
    cache.set_match_count(match_m)
    cache.set_prefetch(depth)
    d_eam = dev(req.prefill_eam.astype(np.int32))
    d_routers = [dev(w) for w in routers]
    d_bias, d_x = dev(req.bias), dev(req.x)
    y = torch.empty(cfg.H, dtype=torch.float32, device="cuda")
    ref_eam = req.prefill_eam.astype(np.int64).copy()
    ref_cache = O.ExpertCache(L, E, S)
    n_pf, n_miss_total, worst = 0, 0, 0.0
    for t in tokens:
        for l in range(L):
            idx, best, n_miss = m.moe_decode_layer(cache, eamc, d_eam, l, d_routers[l], d_bias[l], d_x[t, l], y)
            ref = O.decode_layer(T, ref_eam, ref_cache, l, routers[l], req.bias[l], req.x[t, l],
                                 lambda f: split_expert(cfg, bank[f]),
                                 lambda layer: [split_expert(cfg, shared[layer * cfg.n_shared + s]) for s in range(cfg.n_shared)],
                                 k, bool(cfg.renorm), EPS, m=match_m, prefetch_depth=depth)
            where = f"token {t} layer {l}"
            assert idx.tolist() == ref["idx"].tolist(), where
            assert best == ref["best"], where
            pf_head, ev_head = cache.last_heads()     # the heads the step selected: k + depth victims, depth candidates
            assert ev_head.tolist() == ref["ev_order"][:k + depth], where
            assert pf_head.tolist() == ref["pf_order"][:depth], where
            assert n_miss == sum(1 for e in ref["events"] if not e[1]), where
            assert cache.last_prefetch() == [(f, v) for f, v, _ in ref["prefetched"]], where
            assert (cache.get_slots() == ref_cache.slot_of).all(), where
            worst = max(worst, rel_max_err(y.cpu().numpy(), ref["y"]))
            n_pf += len(ref["prefetched"])
            n_miss_total += n_miss
    assert cache.error_flags() == 0
    assert worst <= FFN_TOL, worst
    eamc.close()
    cache.close()
    return n_pf, n_miss_total


def test_decode_request_with_prefetching(m):
    cfg = mi.get_config("C1")
    n_pf, n_miss = _replay_prefetch(m, cfg, cfg.S, 12, depth=2)
    assert n_pf > 0
    cfg = mi.get_config("C2").scaled(L=6, H=256, I=192, N=120, prompt=64)
    n_pf, n_miss = _replay_prefetch(m, cfg, (cfg.L * cfg.E) // 4, 8, depth=6, match_m=2)
    assert n_pf > 0


def test_prefetching_lowers_misses_on_the_same_request(m):
    cfg = mi.get_config("C2").scaled(L=6, H=256, I=192, N=120, prompt=64)
    S = (cfg.L * cfg.E) // 6
    _, base = _replay_prefetch(m, cfg, S, 10, depth=0, rid=3)
    _, with_pf = _replay_prefetch(m, cfg, S, 10, depth=8, rid=3)
    assert with_pf < base


def test_prefetches_planned_by_asynchronous_steps(m):
    # Device-driven (asynchronous) layer steps with prefetching: the step plans on the device, the host
    # carries the plan out at the next call on the cache.  All layers but the last are resident and are
    # stepped asynchronously (they cannot miss); the last layer's experts start out on the host, are
    # prefetched into the free slots as the prediction names them, and that layer is stepped synchronously
    # (it may still miss).  Every step's prefetches, the slot table and the outputs against the oracle,
    # whose decode_layer prefetches right after the step: nothing touches the cache in between, so the
    # one-call lag changes no state.
    cfg = mi.get_config("C2").scaled(L=5, H=256, I=192, N=120, prompt=64, E=32)
    L, E, k, depth = cfg.L, cfg.E, cfg.k, 4
    S = L * E - E // 2                                      # half of the last layer never fits: real evictions too
    T, _, _ = mi.eamc_traces(cfg, threads=4)
    req = mi.make_request(cfg, 9, decode=14)
    tokens = pick_clear_tokens(cfg, req, 6)
    bank = mi.expert_bank(cfg, L * E, threads=4)
    shared = mi.expert_bank(cfg.scaled(cid=cfg.cid + 50), L * cfg.n_shared, threads=2)
    routers = [mi.router_weights(cfg, l) for l in range(L)]
    desc = m.ModelDesc.from_config(cfg)
    eamc = m.Eamc(desc, cfg.N, 4)
    eamc.load(T)
    cache = m.Cache(desc, S, pinned(pack_bank(m, cfg, bank)), pinned(pack_bank(m, cfg, shared)))
    n_res = (L - 1) * E
    cache.reset(n_res)
    cache.set_prefetch(depth)
    ref_cache = O.ExpertCache(L, E, S, warm=False)
    for l in range(L - 1):
        ref_cache.retrieve(l, list(range(E)))               # flat ids 0 .. n_res-1 in slots of the same number
    assert (cache.get_slots() == ref_cache.slot_of).all()
    d_eam = dev(req.prefill_eam.astype(np.int32))
    ref_eam = req.prefill_eam.astype(np.int64).copy()
    d_routers, d_bias, d_x = [dev(w) for w in routers], dev(req.bias), dev(req.x)
    y = torch.empty(cfg.H, dtype=torch.float32, device="cuda")
    n_pf = n_miss_total = 0
    for t in tokens:
        for l in range(L):
            last_layer = l == L - 1
            ref = O.decode_layer(T, ref_eam, ref_cache, l, routers[l], req.bias[l], req.x[t, l],
                                 lambda f: split_expert(cfg, bank[f]),
                                 lambda layer: [split_expert(cfg, shared[layer * cfg.n_shared + s]) for s in range(cfg.n_shared)],
                                 k, bool(cfg.renorm), EPS, prefetch_depth=depth)
            where = f"token {t} layer {l}"
            if last_layer:
                idx, best, n_miss = m.moe_decode_layer(cache, eamc, d_eam, l, d_routers[l], d_bias[l], d_x[t, l], y)
                assert idx.tolist() == ref["idx"].tolist() and best == ref["best"], where
                assert n_miss == sum(1 for e in ref["events"] if not e[1]), where
                n_miss_total += n_miss
            else:
                assert all(e[1] for e in ref["events"]), where       # resident layers never miss
                m.moe_decode_layer(cache, eamc, d_eam, l, d_routers[l], d_bias[l], d_x[t, l], y, sync=False)
                cache.join()                                         # the host carries the step's plan out
            assert cache.last_prefetch() == [(f, v) for f, v, _ in ref["prefetched"]], where
            assert (cache.get_slots() == ref_cache.slot_of).all(), where
            torch.cuda.synchronize()
            assert (d_eam.cpu().numpy() == ref_eam).all(), where
            assert rel_max_err(y.cpu().numpy(), ref["y"]) <= FFN_TOL, where
            n_pf += len(ref["prefetched"])
    assert n_pf > 0
    assert cache.error_flags() == 0
    # the plan of an asynchronous step is also carried out by the next layer step itself (no join between)
    cache.reset(n_res)
    ref_cache = O.ExpertCache(L, E, S, warm=False)
    for l in range(L - 1):
        ref_cache.retrieve(l, list(range(E)))
    d_eam.copy_(dev(req.prefill_eam.astype(np.int32)))
    ref_eam = req.prefill_eam.astype(np.int64).copy()
    t = tokens[0]
    for l in range(L - 1):
        O.decode_layer(T, ref_eam, ref_cache, l, routers[l], req.bias[l], req.x[t, l], lambda f: split_expert(cfg, bank[f]),
                       lambda layer: [split_expert(cfg, shared[layer * cfg.n_shared + s]) for s in range(cfg.n_shared)],
                       k, bool(cfg.renorm), EPS, prefetch_depth=depth)
        m.moe_decode_layer(cache, eamc, d_eam, l, d_routers[l], d_bias[l], d_x[t, l], y, sync=False)
    cache.join()
    assert (cache.get_slots() == ref_cache.slot_of).all()
    eamc.close()
    cache.close()
