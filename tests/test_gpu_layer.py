"""Cache retrieval (Alg. 1) and the fused layer step against the oracle, state carried
across a whole request: routing, EAM, matched trace, both orders and the hit/miss/victim
sequence must agree exactly at every layer step; FFN outputs within tolerance.
Layer inputs are teacher-forced (each (token, layer) has its own pre-drawn x), so a
rounding difference in one FFN output cannot change a later routing decision.
"""
import numpy as np
import pytest
import torch

import moei_inputs as mi
from oracle import moei_oracle as O
from tests.helpers import EPS, dev, pack_bank, pick_clear_tokens, pinned, rel_max_err, split_expert

pytestmark = pytest.mark.gpu

FFN_TOL = 2e-2
FFN_TOL_FP32ACC = 2e-4


@pytest.fixture(scope="module")
def m():
    import paper_2401_14361_amd as mod
    mod.lib()
    return mod


def test_cache_retrieve_sequence_and_slot_contents(m):
    cfg = mi.get_config("C1").scaled(H=64, I=32)
    L, E, k, S = cfg.L, cfg.E, cfg.k, 6
    bank = mi.expert_bank(cfg, L * E, threads=2)
    packed = pack_bank(m, cfg, bank)
    host = pinned(packed)
    cache = m.Cache(m.ModelDesc.from_config(cfg), S, host)
    for warm in (True, False):
        cache.reset(S if warm else 0)
        ref = O.ExpertCache(L, E, S, warm=warm)
        rng = np.random.default_rng(11)
        for it in range(30):
            for layer in range(L):
                picks = rng.choice(E, size=k, replace=False)
                need = {layer * E + int(p) for p in picks}
                resident = [f for f in range(L * E) if ref.slot_of[f] >= 0 and f not in need]
                ev = rng.permutation(resident)[: (1 if it % 5 == 0 else len(resident))]
                if it % 3 == 1:  # an order with stale entries and experts needed now: both are passed over
                    ev = rng.permutation(L * E)
                want = ref.retrieve(layer, picks, ev)
                slots, victims, n_miss = cache.retrieve(layer, picks, ev)
                assert slots.tolist() == [w[3] for w in want]
                assert victims.tolist() == [w[2] for w in want]
                assert n_miss == sum(1 for w in want if not w[1])
                assert (cache.get_slots() == ref.slot_of).all()
        torch.cuda.synchronize()
        # every resident slot holds its owner's weights; the device table mirrors the host's
        for f in range(L * E):
            s = int(ref.slot_of[f])
            if s >= 0:
                got = cache.slot_tensor(s).cpu().numpy()
                assert (got == packed[f]).all()
    with pytest.raises(m.MoeiError):
        cache.retrieve(0, [1, 1], [])
    with pytest.raises(m.MoeiError):
        cache.retrieve(L, [0, 1], [])
    cache.close()
    # without a host copy a miss is an error, not a silent zero
    c2 = m.Cache(m.ModelDesc.from_config(cfg), S)
    c2.reset(S)
    with pytest.raises(m.MoeiError):
        c2.retrieve(L - 1, [0, 1], [0])
    c2.close()


def _weights_as_f64(cfg, flat):
    """(W_gate, W_up, W_down) of a drawn expert, converted to fp64 once (the conversion is exact; the
    oracle would repeat it at every use, which takes seconds for a 352 MB expert)."""
    return tuple(O.to_f64(w) for w in split_expert(cfg, flat))


def _replay(m, cfg, S, n_tokens, n_unique, cell_bytes, rid=0, match_m=1, f64_cache=False):
    L, E, k = cfg.L, cfg.E, cfg.k
    T, _, _ = mi.eamc_traces(cfg, threads=4)
    req = mi.make_request(cfg, rid, decode=n_tokens + 8)
    tokens = pick_clear_tokens(cfg, req, n_tokens)
    bank = mi.expert_bank(cfg, n_unique, threads=4)
    shared = mi.expert_bank(cfg.scaled(cid=cfg.cid + 50), max(L * cfg.n_shared, 1), threads=2)
    routers = [mi.router_weights(cfg, l) for l in range(L)]

    desc = m.ModelDesc.from_config(cfg)
    eamc = m.Eamc(desc, cfg.N, cell_bytes)
    eamc.load(T)
    cache = m.Cache(desc, S, pinned(pack_bank(m, cfg, bank)), pinned(pack_bank(m, cfg, shared)) if cfg.n_shared else None)
    cache.reset(min(S, L * E))
    cache.set_match_count(match_m)
    d_eam = dev(req.prefill_eam.astype(np.int32))
    d_routers = [dev(w) for w in routers]
    d_bias = dev(req.bias)
    d_x = dev(req.x)
    y = torch.empty(cfg.H, dtype=torch.float32, device="cuda")

    ref_eam = req.prefill_eam.astype(np.int64).copy()
    ref_cache = O.ExpertCache(L, E, S)

    f64 = [_weights_as_f64(cfg, bank[u]) for u in range(n_unique)] if f64_cache else None

    def expert_of(fid):
        return f64[fid % n_unique] if f64_cache else split_expert(cfg, bank[fid % n_unique])

    def shared_of(layer):
        return [split_expert(cfg, shared[layer * cfg.n_shared + s]) for s in range(cfg.n_shared)]

    n_miss_total, worst = 0, 0.0
    for t in tokens:
        for l in range(L):
            idx, best, n_miss = m.moe_decode_layer(cache, eamc, d_eam, l, d_routers[l], d_bias[l], d_x[t, l], y)
            pf_head, ev_head = cache.last_heads()      # what the step itself selected, before the full ranking
            last = cache.last_step()
            ref = O.decode_layer(T, ref_eam, ref_cache, l, routers[l], req.bias[l], req.x[t, l], expert_of, shared_of,
                                 k, bool(cfg.renorm), EPS, m=match_m)
            where = f"token {t} layer {l}"
            assert ev_head.tolist() == ref["ev_order"][:k] and pf_head.tolist() == [], where
            assert idx.tolist() == ref["idx"].tolist(), where
            np.testing.assert_allclose(last["w"], ref["w"], rtol=1e-4, err_msg=where)
            assert (d_eam.cpu().numpy() == ref_eam).all(), where
            assert best == ref["best"], where
            assert cache.last_matches()[0].tolist() == ref["matched"], where
            np.testing.assert_allclose(last["sim"], ref["sim"], rtol=1e-5, err_msg=where)
            assert last["ev_order"].tolist() == ref["ev_order"], where
            assert last["pf_order"].tolist() == ref["pf_order"], where
            np.testing.assert_allclose(last["P"], ref["P"], rtol=1e-6, err_msg=where)
            np.testing.assert_allclose(last["V"], ref["V"], rtol=1e-6, err_msg=where)
            assert n_miss == sum(1 for e in ref["events"] if not e[1]), where
            assert (cache.get_slots() == ref_cache.slot_of).all(), where
            worst = max(worst, rel_max_err(y.cpu().numpy(), ref["y"]))
            n_miss_total += n_miss
    assert cache.error_flags() == 0
    assert worst <= FFN_TOL_FP32ACC <= FFN_TOL, worst
    eamc.close()
    cache.close()
    return n_miss_total


def test_requests_in_sequence_starting_from_an_empty_collection(m):
    # the online loop (App. B.1): the first request meets an empty EAMC (no match: best = -1, all
    # prefetch scores zero, eviction by layer decay alone); its request-level EAM is inserted when
    # it ends; later requests match what their predecessors left
    cfg = mi.get_config("C1").scaled(H=64, I=32)
    L, E, k, S = cfg.L, cfg.E, cfg.k, 10
    bank = mi.expert_bank(cfg, L * E, threads=2)
    routers = [mi.router_weights(cfg, l) for l in range(L)]
    desc = m.ModelDesc.from_config(cfg)
    eamc = m.Eamc(desc, 8, 4)
    cache = m.Cache(desc, S, pinned(pack_bank(m, cfg, bank)))
    cache.reset(S)
    ref_cache = O.ExpertCache(L, E, S)
    d_routers = [dev(w) for w in routers]
    y = torch.empty(cfg.H, dtype=torch.float32, device="cuda")
    T = np.zeros((0, L, E), dtype=np.int32)
    bests = []
    for rid in range(3):
        req = mi.make_request(cfg, 40 + rid, decode=12)
        tokens = pick_clear_tokens(cfg, req, 4)
        d_eam = dev(req.prefill_eam.astype(np.int32))
        ref_eam = req.prefill_eam.astype(np.int64).copy()
        d_bias, d_x = dev(req.bias), dev(req.x)
        for t in tokens:
            for l in range(L):
                idx, best, n_miss = m.moe_decode_layer(cache, eamc, d_eam, l, d_routers[l], d_bias[l], d_x[t, l], y)
                last = cache.last_step()
                ref = O.decode_layer(T, ref_eam, ref_cache, l, routers[l], req.bias[l], req.x[t, l],
                                     lambda f: split_expert(cfg, bank[f]), lambda layer: [], k, bool(cfg.renorm), EPS)
                where = f"request {rid} token {t} layer {l}"
                assert idx.tolist() == ref["idx"].tolist(), where
                assert best == ref["best"], where
                assert last["ev_order"].tolist() == ref["ev_order"], where
                assert last["pf_order"].tolist() == ref["pf_order"], where
                np.testing.assert_allclose(last["V"], ref["V"], rtol=1e-6, err_msg=where)
                np.testing.assert_allclose(last["P"], ref["P"], rtol=1e-6, atol=0, err_msg=where)
                assert (cache.get_slots() == ref_cache.slot_of).all(), where
                assert rel_max_err(y.cpu().numpy(), ref["y"]) <= FFN_TOL_FP32ACC, where
                bests.append(best)
        assert (d_eam.cpu().numpy() == ref_eam).all()
        eamc.insert(ref_eam.astype(np.int32))
        T = np.concatenate([T, ref_eam.astype(np.int32)[None]], axis=0)
        assert eamc.size == rid + 1 and (eamc.export() == T).all()
    n_first = 4 * L
    assert all(b == -1 for b in bests[:n_first]) and all(b >= 0 for b in bests[n_first:])
    assert cache.error_flags() == 0
    eamc.close()
    cache.close()


def test_decode_request_tiny_config(m):
    # configuration 1 as specified: 4 layers x 8 experts, top-2, fp32, 12 of 32 slots, 16 decode tokens
    cfg = mi.get_config("C1")
    misses = _replay(m, cfg, cfg.S, cfg.decode, cfg.L * cfg.E, 4)
    assert misses > 0                                   # the capped cache really evicts


def test_decode_request_tiny_config_waiting_for_events_only(m, monkeypatch):
    # the synchronous step normally polls the pinned words its kernels write and falls back to the
    # events; the same replay with the polling switched off (read when the cache is created)
    monkeypatch.setenv("MOEI_SYNC_POLL", "0")
    cfg = mi.get_config("C1")
    misses = _replay(m, cfg, cfg.S, cfg.decode, cfg.L * cfg.E, 4)
    assert misses > 0


@pytest.mark.parametrize("cell_bytes", [4, 2])
def test_decode_request_reduced_deepseek_shape(m, cell_bytes):
    # DeepSeek-V2-Lite structure (top-6 of 64 + 2 shared, bf16, 25 % of experts cached), narrow matrices
    cfg = mi.get_config("C2").scaled(L=6, H=256, I=192, N=120, prompt=64)
    misses = _replay(m, cfg, (cfg.L * cfg.E) // 4, 10, 48, cell_bytes)
    assert misses > 0


def test_decode_request_reduced_mixtral_shape(m):
    cfg = mi.get_config("C3").scaled(L=5, H=512, I=1792, N=80, prompt=32)
    misses = _replay(m, cfg, 15, 10, cfg.L * cfg.E, 4)
    assert misses > 0


def test_decode_request_with_aggregated_matches(m):
    # PredictEAM over the 3 / 16 most similar traces (Sec. 4.5 step 2) inside the fused layer step
    cfg = mi.get_config("C2").scaled(L=6, H=256, I=192, N=120, prompt=64)
    assert _replay(m, cfg, (cfg.L * cfg.E) // 4, 6, 48, 4, match_m=3) > 0
    cfg = mi.get_config("C1")
    assert _replay(m, cfg, cfg.S, 8, cfg.L * cfg.E, 2, rid=1, match_m=16) > 0
    # more traces than one workgroup scans: the finishing workgroup merges the winners
    cfg = mi.get_config("C1").scaled(N=2300)
    _replay(m, cfg, cfg.S, 3, cfg.L * cfg.E, 4, rid=2, match_m=5)


def _resident_setup(m, cfg, n_unique, rid, n_decode):
    """Everything resident (the asynchronous step looks its slots up on the device and cannot miss)."""
    L, E = cfg.L, cfg.E
    T, _, _ = mi.eamc_traces(cfg, threads=4)
    req = mi.make_request(cfg, rid, decode=n_decode)
    bank = mi.expert_bank(cfg, n_unique, threads=4)
    shared = mi.expert_bank(cfg.scaled(cid=cfg.cid + 50), max(L * cfg.n_shared, 1), threads=2)
    desc = m.ModelDesc.from_config(cfg)
    eamc = m.Eamc(desc, cfg.N)
    eamc.load(T)
    packed, packed_sh = pack_bank(m, cfg, bank), pack_bank(m, cfg, shared)
    d_packed = [dev(packed[u]) for u in range(n_unique)]

    def fresh():
        c = m.Cache(desc, L * E)
        for s_ in range(L * E):
            t = c.slot_tensor(s_)
            t.copy_(d_packed[s_ % n_unique].view(t.dtype))
        for s_ in range(L * cfg.n_shared):
            t = c.slot_tensor(L * E + s_)
            t.copy_(dev(packed_sh[s_]).view(t.dtype))
        c.reset(L * E)
        return c

    def expert_of(fid):
        return split_expert(cfg, bank[fid % n_unique])

    def shared_of(layer):
        return [split_expert(cfg, shared[layer * cfg.n_shared + s_]) for s_ in range(cfg.n_shared)]

    return T, req, eamc, fresh, expert_of, shared_of


def _check_step(cfg, where, last, matched, ref, y, eam_now, ref_eam):
    """One layer step of the device-driven path against the oracle's: the EAM (hence the picks), gate
    weights, matched traces, similarity, both score tables and both orders, the output."""
    assert (eam_now == ref_eam).all(), where
    np.testing.assert_allclose(last["w"], ref["w"], rtol=1e-4, err_msg=where)
    assert matched == ref["matched"], where
    np.testing.assert_allclose(last["sim"], ref["sim"], rtol=1e-5, err_msg=where)
    assert last["ev_order"].tolist() == ref["ev_order"], where
    assert last["pf_order"].tolist() == ref["pf_order"], where
    np.testing.assert_allclose(last["P"], ref["P"], rtol=1e-6, err_msg=where)
    np.testing.assert_allclose(last["V"], ref["V"], rtol=1e-6, err_msg=where)
    err = rel_max_err(y, ref["y"])
    assert err <= FFN_TOL_FP32ACC <= FFN_TOL, (where, err)


def _async_against_oracle(m, cfg, n_unique, n_tokens, rid):
    """Asynchronous layer steps (no host outputs: slots looked up on the device, nothing waits for
    the side stream), each compared with the oracle's layer step."""
    L, E, k = cfg.L, cfg.E, cfg.k
    T, req, eamc, fresh, expert_of, shared_of = _resident_setup(m, cfg, n_unique, rid, n_tokens + 8)
    tokens = pick_clear_tokens(cfg, req, n_tokens)
    routers = [mi.router_weights(cfg, l) for l in range(L)]
    d_routers, d_bias, d_x = [dev(w) for w in routers], dev(req.bias), dev(req.x)
    cache = fresh()
    d_eam = dev(req.prefill_eam.astype(np.int32))
    ref_eam = req.prefill_eam.astype(np.int64).copy()
    ref_cache = O.ExpertCache(L, E, L * E)
    y = torch.empty(cfg.H, dtype=torch.float32, device="cuda")
    for t in tokens:
        for l in range(L):
            m.moe_decode_layer(cache, eamc, d_eam, l, d_routers[l], d_bias[l], d_x[t, l], y, sync=False)
            _, ev_head = cache.last_heads()
            last = cache.last_step()
            ref = O.decode_layer(T, ref_eam, ref_cache, l, routers[l], req.bias[l], req.x[t, l], expert_of, shared_of,
                                 k, bool(cfg.renorm), EPS)
            assert all(e[1] for e in ref["events"])
            assert ev_head.tolist() == ref["ev_order"][:k], (t, l)
            _check_step(cfg, f"async token {t} layer {l}", last, cache.last_matches()[0].tolist(), ref,
                        y.cpu().numpy(), d_eam.cpu().numpy(), ref_eam)
    assert cache.error_flags() == 0
    cache.close()
    eamc.close()


def _graph_against_oracle(m, cfg, n_unique, n_tokens, rid):
    """One token's L asynchronous layer steps captured in a HIP graph and replayed per token, with
    eager work and synchronisations between replays.  After every replay: each layer's output, the
    EAM, and the last layer's match, scores and orders against the oracle run over the same steps."""
    L, E, k = cfg.L, cfg.E, cfg.k
    T, req, eamc, fresh, expert_of, shared_of = _resident_setup(m, cfg, n_unique, rid, n_tokens + 8)
    tokens = pick_clear_tokens(cfg, req, n_tokens)
    routers = [mi.router_weights(cfg, l) for l in range(L)]
    d_routers, d_bias, d_x = [dev(w) for w in routers], dev(req.bias), dev(req.x)
    cache = fresh()
    d_eam = dev(req.prefill_eam.astype(np.int32))
    x_stage = torch.empty_like(d_x[0])
    y_all = torch.empty((L, cfg.H), dtype=torch.float32, device="cuda")
    cache.sync()
    cap = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=cap):
        for l in range(L):
            m.moe_decode_layer(cache, eamc, d_eam, l, d_routers[l], d_bias[l], x_stage[l], y_all[l], sync=False)
        cache.join()
    cache.sync()
    d_eam.copy_(dev(req.prefill_eam.astype(np.int32)))      # the capture itself did not run anything
    ref_eam = req.prefill_eam.astype(np.int64).copy()
    ref_cache = O.ExpertCache(L, E, L * E)
    for t in tokens:
        x_stage.copy_(d_x[t])
        graph.replay()
        torch.cuda.synchronize()
        got_y, got_eam = y_all.cpu().numpy(), d_eam.cpu().numpy()
        last, matched = cache.last_step(), cache.last_matches()[0].tolist()
        for l in range(L):
            ref = O.decode_layer(T, ref_eam, ref_cache, l, routers[l], req.bias[l], req.x[t, l], expert_of, shared_of,
                                 k, bool(cfg.renorm), EPS)
            err = rel_max_err(got_y[l], ref["y"])
            assert err <= FFN_TOL_FP32ACC, (t, l, err)
        _check_step(cfg, f"graph token {t}", last, matched, ref, got_y[L - 1], got_eam, ref_eam)
        # the program's own eager work between replays
        m.eamc_match(eamc, d_eam)
        y_all.zero_()
        torch.cuda.synchronize()
    assert cache.error_flags() == 0
    cache.close()
    eamc.close()


def test_async_layer_steps_against_the_oracle(m):
    cfg = mi.get_config("C2").scaled(L=3, H=128, I=64, N=40, prompt=16, E=16, k=3)
    _async_against_oracle(m, cfg, cfg.L * cfg.E, 4, rid=2)
    cfg = mi.get_config("C1")
    _async_against_oracle(m, cfg, cfg.L * cfg.E, 3, rid=3)


def test_async_layer_step_flags_a_miss(m):
    # a pick that is not resident cannot be served without the host: the flag says so
    cfg = mi.get_config("C2").scaled(L=3, H=128, I=64, N=40, prompt=16, E=16, k=3)
    L, E = cfg.L, cfg.E
    T, _, _ = mi.eamc_traces(cfg, threads=2)
    req = mi.make_request(cfg, 2, decode=4)
    bank = pack_bank(m, cfg, mi.expert_bank(cfg, L * E, threads=2))
    shared = pack_bank(m, cfg, mi.expert_bank(cfg.scaled(cid=77), L * cfg.n_shared, threads=2))
    desc = m.ModelDesc.from_config(cfg)
    eamc = m.Eamc(desc, cfg.N)
    eamc.load(T)
    cache = m.Cache(desc, cfg.k, pinned(bank), pinned(shared))
    cache.reset(0)
    y = torch.empty(cfg.H, dtype=torch.float32, device="cuda")
    m.moe_decode_layer(cache, eamc, dev(req.prefill_eam.astype(np.int32)), 0, dev(mi.router_weights(cfg, 0)),
                       dev(req.bias[0]), dev(req.x[0, 0]), y, sync=False)
    assert cache.error_flags() & 2
    cache.close()
    eamc.close()


def test_layer_step_with_router_logits_that_have_no_softmax(m):
    # error path: a NaN in the router bias.  Asynchronous step: flag bit 2, no picks, the EAM row
    # untouched, the output is the shared experts' alone; synchronous step: an error, nothing runs
    cfg = mi.get_config("C2").scaled(L=2, H=128, I=64, N=20, prompt=16, E=16, k=3)
    L, E = cfg.L, cfg.E
    T, req, eamc, fresh, expert_of, shared_of = _resident_setup(m, cfg, L * E, 6, 2)
    cache = fresh()
    eam0 = req.prefill_eam.astype(np.int32)
    d_eam = dev(eam0)
    bias = req.bias[1].astype(np.float32).copy()
    bias[5] = np.nan
    y = torch.empty(cfg.H, dtype=torch.float32, device="cuda")
    W = dev(mi.router_weights(cfg, 1))
    m.moe_decode_layer(cache, eamc, d_eam, 1, W, dev(bias), dev(req.x[0, 1]), y, sync=False)
    torch.cuda.synchronize()
    assert cache.error_flags() & 4
    assert (d_eam.cpu().numpy() == eam0).all()
    want = O.expert_ffn(req.x[0, 1], shared_of(1), [1.0] * cfg.n_shared)
    assert rel_max_err(y.cpu().numpy(), want) <= FFN_TOL_FP32ACC
    with pytest.raises(m.MoeiError) as e:
        m.moe_decode_layer(cache, eamc, d_eam, 1, W, dev(bias), dev(req.x[0, 1]), y, sync=True)
    assert e.value.code == -4 and "no finite" in str(e.value)
    cache.sync()
    # the cache still works afterwards
    cache.error_flags()
    m.moe_decode_layer(cache, eamc, d_eam, 1, W, dev(req.bias[1]), dev(req.x[0, 1]), y, sync=False)
    torch.cuda.synchronize()
    assert cache.error_flags() == 0 and int(d_eam.cpu().numpy()[1].sum() - eam0[1].sum()) == cfg.k
    cache.close()
    eamc.close()


def test_layer_steps_in_a_hip_graph_against_the_oracle(m):
    cfg = mi.get_config("C2").scaled(L=4, H=256, I=192, N=60, prompt=32)
    _graph_against_oracle(m, cfg, cfg.L * cfg.E, 5, rid=4)


# ------------------------------------------------------------------ full benchmark shapes
def test_full_size_deepseek_v2_lite_tokens_with_capped_cache(m):
    # configuration 2 at full size (26 x 64 experts of 2048 x 1408 bf16, 1,000 traces, 416 slots):
    # 12 decode tokens = 312 layer steps, every one compared in full while the cache keeps evicting
    cfg = mi.get_config("C2")
    misses = _replay(m, cfg, cfg.S, 12, 24, 4)
    assert misses > 12 * cfg.k


def test_full_size_deepseek_v2_lite_async_and_graph_steps(m):
    # the path the benchmark times, at the benchmark's width: all 1,664 experts resident, asynchronous
    # layer steps (one token, step by step) and the HIP-graph replay (two tokens of 26 layer steps)
    cfg = mi.get_config("C2")
    _async_against_oracle(m, cfg, 24, 1, rid=0)
    _graph_against_oracle(m, cfg, 24, 2, rid=0)


def test_full_size_mixtral_request_all_layers(m):
    # configuration 3 at full size: all 32 layers x 8 experts of 4096 x 14336 bf16 (352 MB each),
    # 96 of 256 slots, 1,000 traces; three decode tokens = 96 layer steps with misses from host memory
    cfg = mi.get_config("C3")
    misses = _replay(m, cfg, cfg.S, 3, 6, 4, f64_cache=True)
    assert misses > 0


def test_full_size_deepseek_v2_slice_steps(m):
    # configuration 4's shapes: 160 experts per layer top-6 + 2 shared, 5120 x 1536, 10,000 traces; the 12
    # layers whose 1,920 experts fill the 2,048-slot pool carry weights (the 59 x 160 match and priority
    # sizes are covered in test_gpu_steps.py), one token through all of them
    cfg = mi.get_config("C4")
    cfg = cfg.scaled(L=cfg.S // cfg.E)
    _replay(m, cfg, cfg.L * cfg.E, 1, 12, 2)
