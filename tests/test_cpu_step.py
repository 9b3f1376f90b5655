"""The C/OpenMP CPU baseline (oracle/cpu_step.c, timed by the benchmark beside the GPU path) against
the Python oracle: two independent CPU implementations of the layer step must agree - discrete
results exactly, reals to fp64 rounding - with one thread and with several (CPU only)."""
import numpy as np
import pytest

import moei_inputs as mi
from oracle import cpu_step as CS
from oracle import moei_oracle as O


def _split(cfg, w):
    H, I = cfg.H, cfg.I
    return (np.ascontiguousarray(w[:I * H].reshape(I, H)), np.ascontiguousarray(w[I * H:2 * I * H].reshape(I, H)),
            np.ascontiguousarray(w[2 * I * H:].reshape(H, I)))


@pytest.mark.parametrize("cname,scale,threads", [("C1", {}, 1), ("C1", {}, 3),
                                                 ("C2", dict(L=5, H=128, I=96, N=60, prompt=48), 4),
                                                 ("C3", dict(L=4, H=256, I=160, N=30, prompt=32), 2)])
def test_cpu_step_agrees_with_the_oracle(cname, scale, threads):
    cfg = mi.get_config(cname).scaled(**scale)
    L, E, k = cfg.L, cfg.E, cfg.k
    T, _, _ = mi.eamc_traces(cfg, threads=1)
    req = mi.make_request(cfg, 1, decode=3)
    bank = mi.expert_bank(cfg, L * E, threads=2)
    shared = mi.expert_bank(cfg.scaled(cid=cfg.cid + 50), max(L * cfg.n_shared, 1), threads=1)
    triples = [_split(cfg, bank[f]) for f in range(L * E)]
    sh_triples = [_split(cfg, shared[s]) for s in range(L * cfg.n_shared)]
    S = max(k, (L * E) // 3)
    ref_cache = O.ExpertCache(L, E, S)
    eam_c = req.prefill_eam.astype(np.int64).copy()
    eam_o = eam_c.copy()
    for t in range(3):
        for l in range(L):
            W = mi.router_weights(cfg, l)
            resident = ref_cache.resident().copy()        # Alg. 1's bookkeeping stays with the oracle's cache
            ref = O.decode_layer(T, eam_o, ref_cache, l, W, req.bias[l], req.x[t, l], lambda f: triples[f],
                                 lambda layer: sh_triples[layer * cfg.n_shared:(layer + 1) * cfg.n_shared], k,
                                 bool(cfg.renorm), 2.0 ** -20)
            tab = CS.pointer_table(triples[l * E:(l + 1) * E])
            sh_tab = CS.pointer_table(sh_triples[l * cfg.n_shared:(l + 1) * cfg.n_shared]) if cfg.n_shared else None
            got = CS.decode_step(T, eam_c, l, W, req.bias[l], req.x[t, l], tab, sh_tab, cfg.H, cfg.I, k, cfg.renorm,
                                 2.0 ** -20, resident, threads=threads)
            where = (t, l)
            assert got["idx"].tolist() == ref["idx"].tolist(), where
            np.testing.assert_allclose(got["w"], ref["w"], rtol=1e-12, err_msg=str(where))
            assert (eam_c == eam_o).all(), where
            assert got["best"] == ref["best"], where
            np.testing.assert_allclose(got["sim"], ref["sim"], rtol=1e-14)
            np.testing.assert_array_equal(got["P"], ref["P"])       # one correctly rounded division on both sides
            np.testing.assert_array_equal(got["V"], ref["V"])
            assert got["pf_order"] == ref["pf_order"] and got["ev_order"] == ref["ev_order"], where
            np.testing.assert_allclose(got["y"], ref["y"], rtol=1e-9, atol=1e-12 * np.abs(ref["y"]).max())


def test_cpu_step_empty_collection_and_bad_arguments():
    cfg = mi.get_config("C1").scaled(H=32, I=16)
    L, E, k = cfg.L, cfg.E, cfg.k
    bank = mi.expert_bank(cfg, E, threads=1)
    triples = [_split(cfg, bank[f]) for f in range(E)]
    req = mi.make_request(cfg, 0, decode=1)
    eam = req.prefill_eam.astype(np.int64).copy()
    got = CS.decode_step(np.zeros((0, L, E), np.int32), eam, 0, mi.router_weights(cfg, 0), req.bias[0], req.x[0, 0],
                         CS.pointer_table(triples), None, cfg.H, cfg.I, k, cfg.renorm, 2.0 ** -20, np.ones(L * E))
    assert got["best"] == -1 and got["sim"] == 0.0 and got["pf_order"] == []
    assert len(got["ev_order"]) == L * E - k
    with pytest.raises(RuntimeError):
        CS.decode_step(np.zeros((0, L, E), np.int32), eam, L, mi.router_weights(cfg, 0), req.bias[0], req.x[0, 0],
                       CS.pointer_table(triples), None, cfg.H, cfg.I, k, cfg.renorm, 2.0 ** -20, np.ones(L * E))
    assert CS.threads_available() >= 1
