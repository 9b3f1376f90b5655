"""Decode batches of independent requests (the batch-sweep configuration): the step-wise entry
points with B > 1 against the oracle applied request by request."""
import numpy as np
import pytest
import torch

import moei_inputs as mi
from oracle import moei_oracle as O
from tests.helpers import EPS, dev, pack_bank, rel_max_err, split_expert

pytestmark = pytest.mark.gpu

FFN_TOL_FP32ACC = 2e-4


@pytest.fixture(scope="module")
def m():
    import paper_2401_14361_amd as mod
    mod.lib()
    return mod


def _batch_case(m, cfg, n_unique, batches, cell_bytes=4):
    L, E, k = cfg.L, cfg.E, cfg.k
    T, _, _ = mi.eamc_traces(cfg, threads=8)
    bank = mi.expert_bank(cfg, n_unique, threads=8)
    shared = mi.expert_bank(cfg.scaled(cid=cfg.cid + 50), max(L * cfg.n_shared, 1), threads=2)
    routers = [mi.router_weights(cfg, l) for l in range(L)]
    desc = m.ModelDesc.from_config(cfg)
    eamc = m.Eamc(desc, cfg.N, cell_bytes)
    eamc.load(T)
    S = L * E
    cache = m.Cache(desc, S)
    packed, sh_packed = pack_bank(m, cfg, bank), pack_bank(m, cfg, shared)
    d_bank = [dev(packed[u]) for u in range(n_unique)]
    for s in range(S):
        t = cache.slot_tensor(s)
        t.copy_(d_bank[s % n_unique].view(t.dtype))
    for s in range(L * cfg.n_shared):
        t = cache.slot_tensor(S + s)
        t.copy_(dev(sh_packed[s]).view(t.dtype))
    cache.reset(S)
    slot_of = np.arange(S, dtype=np.int32)
    for B in batches:
        reqs = [mi.make_request(cfg, 100 + b, decode=1) for b in range(B)]
        eam = np.stack([r.prefill_eam for r in reqs]).astype(np.int32)
        d_eam = dev(eam)
        ref_eam = eam.astype(np.int64)
        for l in range(L):
            x = np.stack([r.x[0, l] for r in reqs])
            logits = np.stack([O.router_logits(routers[l], x[b], reqs[b].bias[l]) for b in range(B)]).astype(np.float32)
            idx, w = m.moe_route_topk(dev(logits), k, bool(cfg.renorm))
            ridx, rw = O.route_topk(logits, k, bool(cfg.renorm))
            assert (idx.cpu().numpy() == ridx).all()
            m.eam_update(d_eam, l, idx)
            for b in range(B):
                O.eam_update(ref_eam[b], l, ridx[b])
            assert (d_eam.cpu().numpy() == ref_eam).all()
            best, sim, _ = m.eamc_match(eamc, d_eam)
            rbest = [O.eamc_match(T, ref_eam[b])[0] for b in range(B)]
            assert best.cpu().numpy().tolist() == rbest
            out = m.expert_priority(eamc, best, l, cache.slot_table(), EPS, idx)
            P, V, pf, n_pf, ev, n_ev = [o.cpu().numpy() for o in out]
            excl = [l * E + int(j) for j in ridx.reshape(-1)]
            rP, rV, rpf, rev = O.expert_priority(O.aggregate_matches(T, rbest), l, slot_of.reshape(L, E) >= 0, EPS, excl)
            assert ev[:int(n_ev[0])].tolist() == rev and pf[:int(n_pf[0])].tolist() == rpf
            np.testing.assert_allclose(V, rV, rtol=1e-6)
            y = m.expert_ffn_grouped(cache, l, idx, w, dev(x)).cpu().numpy()
            for b in range(B):
                ex = [split_expert(cfg, bank[(l * E + int(j)) % n_unique]) for j in ridx[b]]
                ex += [split_expert(cfg, shared[l * cfg.n_shared + s]) for s in range(cfg.n_shared)]
                ref = O.expert_ffn(x[b], ex, list(rw[b]) + [1.0] * cfg.n_shared)
                assert rel_max_err(y[b], ref) <= FFN_TOL_FP32ACC, (B, l, b)
        assert cache.error_flags() == 0
    # deterministic: the same batch twice gives identical bits
    y2 = m.expert_ffn_grouped(cache, L - 1, idx, w, dev(x)).cpu().numpy()
    assert (y2 == y).all()
    # a pick that is not resident contributes nothing and is flagged
    cache.reset(0)
    m.expert_ffn_grouped(cache, 0, idx, w, dev(x))
    assert cache.error_flags() & 2
    eamc.close()
    cache.close()


def test_batch_sweep_on_the_deepseek_v2_lite_shape(m):
    # batch sizes 1..16 on the DeepSeek-V2-Lite shape (two of its layers carry weights here)
    cfg = mi.get_config("C5").scaled(L=2, N=400, prompt=64)
    _batch_case(m, cfg, 24, [1, 2, 4, 8, 16])


@pytest.mark.parametrize("wdtype,H,I", [("fp32", 256, 96), ("bf16", 1024, 72), ("bf16", 4096, 40), ("fp32", 1024, 130),
                                          ("fp32", 2048, 37), ("bf16", 2048, 3)])
def test_batched_ffn_other_shapes(m, wdtype, H, I):
    cfg = mi.get_config("C5").scaled(L=2, E=16, k=3, n_shared=1, N=60, prompt=16, H=H, I=I, wdtype=wdtype)
    _batch_case(m, cfg, 32, [3, 16])


def _ffn_only_case(m, cfg, B, idx, w, seed=3):
    """expert_ffn_grouped on given picks (all experts resident) against the oracle, token by token."""
    L, E = cfg.L, cfg.E
    rng = np.random.default_rng(seed)
    n_unique = min(E, 40)
    bank = mi.expert_bank(cfg, n_unique, threads=8)
    shared = mi.expert_bank(cfg.scaled(cid=cfg.cid + 50), max(L * cfg.n_shared, 1), threads=2)
    desc = m.ModelDesc.from_config(cfg)
    S = L * E
    cache = m.Cache(desc, S)
    packed, sh_packed = pack_bank(m, cfg, bank), pack_bank(m, cfg, shared)
    d_bank = [dev(packed[u]) for u in range(n_unique)]
    for s in range(S):
        t = cache.slot_tensor(s)
        t.copy_(d_bank[s % n_unique].view(t.dtype))
    for s in range(L * cfg.n_shared):
        t = cache.slot_tensor(S + s)
        t.copy_(dev(sh_packed[s]).view(t.dtype))
    cache.reset(S)
    x = (rng.standard_normal((B, cfg.H)) * 0.5).astype(np.float32)
    xr = mi.f32_to_bf16_bits(x) if cfg.wdtype == "bf16" else x  # stored form: the oracle decodes it exactly
    xq = dev(xr)
    layer = L - 1
    y = m.expert_ffn_grouped(cache, layer, dev(idx.astype(np.int32)), dev(w.astype(np.float32)), xq).cpu().numpy()
    for b in range(B):
        ex, ws = [], []
        for j, wj in zip(idx[b], w[b]):
            if j >= 0:
                ex.append(split_expert(cfg, bank[(layer * E + int(j)) % n_unique]))
                ws.append(float(wj))
        ex += [split_expert(cfg, shared[layer * cfg.n_shared + s]) for s in range(cfg.n_shared)]
        ref = O.expert_ffn(xr[b], ex, ws + [1.0] * cfg.n_shared)
        assert rel_max_err(y[b], ref) <= FFN_TOL_FP32ACC, b
    assert cache.error_flags() == 0
    cache.close()


def test_batched_ffn_token_without_picks_and_one_expert_for_all(m):
    # token 2 has no picks (what the routing kernels hand over when no softmax exists for its logits):
    # only the shared expert contributes; all other tokens route to the same experts, so these
    # experts' items are full and a fourth item of one token remains (13 = 3 x 4 + 1 tokens)
    cfg = mi.get_config("C5").scaled(L=2, E=16, k=3, n_shared=1, N=8, prompt=4, H=1024, I=50, wdtype="bf16")
    B = 14
    idx = np.tile(np.array([5, 0, 11]), (B, 1))
    idx[2] = -1
    w = np.random.default_rng(1).random((B, 3)) + 0.1
    w[2] = 0.0
    _ffn_only_case(m, cfg, B, idx, w)


def test_batched_ffn_at_the_item_builders_limits(m):
    # 256 experts, 16 tokens x 32 picks = 512 picks: every thread of the item builder holds two picks
    cfg = mi.get_config("C5").scaled(L=1, E=256, k=32, n_shared=0, N=4, prompt=4, H=512, I=6, wdtype="fp32")
    rng = np.random.default_rng(7)
    B = 16
    idx = np.stack([rng.permutation(256)[:32] for _ in range(B)])
    w = rng.random((B, 32)) + 0.05
    _ffn_only_case(m, cfg, B, idx, w)


def test_batched_ffn_rejects_more_experts_than_the_item_builder_takes(m):
    cfg = mi.get_config("C5").scaled(L=1, E=260, k=2, n_shared=0, N=4, prompt=4, H=256, I=4, wdtype="fp32")
    desc = m.ModelDesc.from_config(cfg)
    cache = m.Cache(desc, 260)
    cache.reset(260)
    idx, w = dev(np.zeros((2, 2), np.int32)), dev(np.ones((2, 2), np.float32))
    with pytest.raises(m.MoeiError):
        m.expert_ffn_grouped(cache, 0, idx, w, dev(np.zeros((2, 256), np.float32)))
    cache.close()
