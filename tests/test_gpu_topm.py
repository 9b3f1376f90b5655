"""Top-m EAMC match (Sec. 4.5: several matched EAMs, aggregated by the prediction) against
the oracle: the list of indices must agree exactly, order included; similarities to 1e-5.
"""
import numpy as np
import pytest
import torch

import moei_inputs as mi
from oracle import moei_oracle as O
from tests.helpers import EPS, dev

pytestmark = pytest.mark.gpu
SIM_RTOL = 1e-5


@pytest.fixture(scope="module")
def m():
    import paper_2401_14361_amd as mod
    mod.lib()
    return mod


def _check_topm(m, T, q, cell_bytes, ms, layer_hi=None):
    N, L, E = T.shape
    desc = m.ModelDesc(L, E, 1, 0, 8, 8, m.WDTYPE_BF16, 0, EPS)
    eamc = m.Eamc(desc, max(N, 1) + 5, cell_bytes)
    if N:
        eamc.load(T)
    d_q = dev(q.astype(np.int32))
    for mm in ms:
        top, sim, sims = m.eamc_match_topm(eamc, d_q, mm, layer_hi=layer_hi, want_sims=True)
        torch.cuda.synchronize()
        top, sim = top.cpu().numpy(), sim.cpu().numpy()
        ridx, rsim = O.eamc_match_topm(T, q, mm)
        n = len(ridx)
        assert top[:n].tolist() == ridx, (N, mm)
        assert (top[n:] == -1).all() and (sim[n:] == 0).all()
        np.testing.assert_allclose(sim[:n], rsim, rtol=SIM_RTOL, atol=1e-30)
        if N:
            np.testing.assert_allclose(sims.cpu().numpy(), O.eamc_match(T, q)[2], rtol=SIM_RTOL, atol=1e-30)
    eamc.close()


@pytest.mark.parametrize("N,L,E", [(64, 4, 8), (1000, 5, 16), (3, 2, 6), (1, 1, 1), (1024, 2, 8), (1025, 2, 8),
                                   (2500, 3, 12), (5000, 2, 4)])
@pytest.mark.parametrize("cell_bytes", [4, 2])
def test_topm_shapes_ties_and_short_collections(m, N, L, E, cell_bytes):
    rng = np.random.default_rng(N * 13 + E)
    T = (rng.integers(0, 600, size=(N, L, E)) * (rng.random((N, L, E)) < 0.5)).astype(np.int32)
    q = (rng.integers(1, 100, size=(L, E))).astype(np.int32)
    if N > 40:
        q = T[N // 2].copy() + (rng.random((L, E)) < 0.1)
        for t in (3, N - 2, N // 3):                       # exact ties at similarity 1, across workgroups
            T[t] = 2 * T[N // 2]
        T[7] = 0                                           # an empty trace
    _check_topm(m, T, q, cell_bytes, (1, 2, 5, 16))


def test_topm_many_equal_similarities(m):
    # few distinct cell values: most similarities coincide exactly, the order is the index order
    rng = np.random.default_rng(5)
    T = rng.integers(0, 2, size=(3000, 2, 3)).astype(np.int32)
    q = np.array([[1, 1, 0], [0, 1, 1]], dtype=np.int32)
    _check_topm(m, T, q, 4, (1, 7, 16))
    _check_topm(m, T, np.zeros((2, 3), dtype=np.int32), 2, (4,))    # empty query: indices 0..3


def test_topm_empty_collection_and_argument_checks(m):
    desc = m.ModelDesc(3, 16, 1, 0, 8, 8, m.WDTYPE_BF16, 0, EPS)
    eamc = m.Eamc(desc, 8, 4)
    q = dev(np.ones((3, 16), dtype=np.int32))
    top, sim, _ = m.eamc_match_topm(eamc, q, 4)
    assert top.cpu().numpy().tolist() == [-1] * 4 and sim.cpu().numpy().tolist() == [0.0] * 4
    for bad in (0, 17, -1):
        with pytest.raises(m.MoeiError):
            m.eamc_match_topm(eamc, q, bad)
    with pytest.raises(m.MoeiError):
        m.eamc_match_topm(eamc, q, 2, layer_hi=3)
    eamc.close()


def test_topm_workload_traces_full_size_and_aggregated_priorities(m):
    # 10,000 traces of the DeepSeek-V2-Lite shape; the top 16 feed the aggregated priorities
    cfg = mi.get_config("C2").scaled(N=10000)
    T, cl, _ = mi.eamc_traces(cfg, threads=16)
    req = mi.make_request(cfg, 4, decode=1)
    desc = m.ModelDesc.from_config(cfg)
    for cb in (4, 2):
        eamc = m.Eamc(desc, cfg.N, cb)
        eamc.load(T)
        for mm in (1, 4, 16):
            top, sim, _ = m.eamc_match_topm(eamc, dev(req.prefill_eam.astype(np.int32)), mm)
            torch.cuda.synchronize()
            ridx, rsim = O.eamc_match_topm(T, req.prefill_eam, mm)
            assert top.cpu().numpy().tolist() == ridx
            np.testing.assert_allclose(sim.cpu().numpy(), rsim, rtol=SIM_RTOL)
        rng = np.random.default_rng(cb)
        res = rng.random((cfg.L, cfg.E)) < 0.25
        slot_of = np.where(res.reshape(-1), np.arange(cfg.L * cfg.E), -1).astype(np.int32)
        cur = 9
        cur_idx = rng.choice(cfg.E, size=(1, cfg.k), replace=False).astype(np.int32)
        out = m.expert_priority(eamc, top, cur, dev(slot_of), EPS, dev(cur_idx))
        torch.cuda.synchronize()
        P, V, pf, n_pf, ev, n_ev = [o.cpu().numpy() for o in out]
        rP, rV, rpf, rev = O.expert_priority(O.aggregate_matches(T, ridx), cur, res, EPS,
                                             [cur * cfg.E + int(j) for j in cur_idx[0]])
        assert pf[:int(n_pf[0])].tolist() == rpf and ev[:int(n_ev[0])].tolist() == rev
        np.testing.assert_allclose(P, rP, rtol=1e-6)
        np.testing.assert_allclose(V, rV, rtol=1e-6)
        eamc.close()
