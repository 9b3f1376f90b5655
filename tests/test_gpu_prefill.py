"""The prefill iteration of one MoE layer (Sec. 4.3: n tokens routed together) against the
oracle: picks and the EAM bit-exact, gate weights to 1e-4, outputs within the stated FFN bar
(max |dy| / max |y| <= 2e-2; the grouped path rounds activations to bf16 between the
projections).  Tokens whose routing an fp32 summation order could flip are left out.
"""
import numpy as np
import pytest
import torch

import moei_inputs as mi
from oracle import moei_oracle as O
from tests.helpers import dev, pack_bank, rel_max_err, split_expert

pytestmark = pytest.mark.gpu
FFN_TOL = 2e-2
FFN_TOL_BF16_ACT = 8e-3      # what this path needs: one bf16 rounding of each activation


@pytest.fixture(scope="module")
def m():
    import paper_2401_14361_amd as mod
    mod.lib()
    return mod


def _clear_rows(cfg, W, bias, X, min_gap=1e-3):
    keep = []
    for t in range(X.shape[0]):
        z = np.sort(O.router_logits(W, X[t], bias))[::-1]
        gap = min(z[cfg.k - 1] - z[cfg.k] if cfg.k < cfg.E else np.inf,
                  np.min(-np.diff(z[:cfg.k])) if cfg.k > 1 else np.inf)
        if gap >= min_gap:
            keep.append(t)
    return keep


def _prefill_case(m, cfg, n, layer, n_unique=None, resident=None):
    L, E, k, H = cfg.L, cfg.E, cfg.k, cfg.H
    n_unique = n_unique or L * E
    bank = mi.expert_bank(cfg, n_unique, threads=4)
    shared = mi.expert_bank(cfg.scaled(cid=cfg.cid + 50), max(L * cfg.n_shared, 1), threads=2)
    W = mi.router_weights(cfg, layer)
    req = mi.make_request(cfg, 5, decode=1)
    rng = np.random.default_rng(1000 + n)
    Xall = mi.to_store(cfg, rng.standard_normal((n + n // 2 + 8, H)).astype(np.float32))
    rows = _clear_rows(cfg, W, req.bias[layer], Xall)[:n]
    assert len(rows) == n
    X = np.ascontiguousarray(Xall[rows])
    desc = m.ModelDesc.from_config(cfg)
    S = L * E
    cache = m.Cache(desc, S)
    packed, packed_sh = pack_bank(m, cfg, bank), pack_bank(m, cfg, shared)
    for s in range(S):
        t = cache.slot_tensor(s)
        t.copy_(dev(packed[s % n_unique]).view(t.dtype))
    for s in range(L * cfg.n_shared):
        t = cache.slot_tensor(S + s)
        t.copy_(dev(packed_sh[s]).view(t.dtype))
    cache.reset(S if resident is None else resident)
    eam0 = req.prefill_eam.astype(np.int32)
    d_eam = dev(eam0)
    Y, idx, w = m.moe_prefill_layer(cache, d_eam, layer, dev(W), dev(req.bias[layer]), dev(X), want_picks=True)
    torch.cuda.synchronize()
    ref_eam = eam0.astype(np.int64).copy()
    ridx, rw, rY = O.prefill_layer(ref_eam, layer, W, req.bias[layer], X,
                                   lambda f: split_expert(cfg, bank[f % n_unique]),
                                   lambda l: [split_expert(cfg, shared[l * cfg.n_shared + s]) for s in range(cfg.n_shared)],
                                   k, bool(cfg.renorm))
    flags = cache.error_flags()
    out = dict(idx=idx.cpu().numpy(), w=w.cpu().numpy(), Y=Y.cpu().numpy(), eam=d_eam.cpu().numpy(),
               ridx=ridx, rw=rw, rY=rY, ream=ref_eam, flags=flags)
    cache.close()
    return out


def _check(o):
    assert o["flags"] == 0
    assert (o["idx"] == o["ridx"]).all()
    np.testing.assert_allclose(o["w"], o["rw"], rtol=1e-4)
    assert (o["eam"] == o["ream"]).all()
    err = rel_max_err(o["Y"], o["rY"])
    assert err <= FFN_TOL_BF16_ACT <= FFN_TOL, err
    # row by row as well: no token may be off by more than the bar relative to its own largest entry
    for t in range(o["Y"].shape[0]):
        assert rel_max_err(o["Y"][t], o["rY"][t]) <= FFN_TOL, t


@pytest.mark.parametrize("n", [1, 7, 64, 65, 130, 200, 700])
def test_prefill_reduced_deepseek_shape(m, n):
    # DeepSeek-V2-Lite structure (top-6 of 64 + 2 shared, bf16), narrow matrices; token counts around the 64-token
    # tile, and one prompt long enough (n k > 64 E) that the items hold up to 128 tokens
    cfg = mi.get_config("C2").scaled(L=3, H=256, I=192, N=8, prompt=16)
    _check(_prefill_case(m, cfg, n, layer=1))


def test_prefill_ragged_rows_and_small_expert_counts(m):
    # I not a multiple of the 128-unit block nor of 32; few experts, so several items per expert
    cfg = mi.get_config("C2").scaled(L=2, E=8, k=2, H=384, I=200, N=8, prompt=16)
    _check(_prefill_case(m, cfg, 90, layer=0))
    cfg = mi.get_config("C3").scaled(L=2, H=512, I=72, N=8, prompt=16)      # Mixtral structure: renormalised top-2 of 8, no shared experts
    _check(_prefill_case(m, cfg, 50, layer=1))
    # the same structure with a prompt that takes 128-token items, the last item of most experts ragged
    _check(_prefill_case(m, cfg, 300, layer=0))


def test_prefill_wide_rows(m):
    cfg = mi.get_config("C3").scaled(L=1, H=4096, I=160, N=8, prompt=16)
    _check(_prefill_case(m, cfg, 40, layer=0, n_unique=4))


def test_prefill_full_width_deepseek_v2_lite_layer(m):
    # configuration 2 at full width (2048 x 1408 bf16 experts), one layer, a 512-token prompt
    cfg = mi.get_config("C2").scaled(L=1, N=8, prompt=16)
    o = _prefill_case(m, cfg, 512, layer=0, n_unique=16)
    _check(o)


def test_prefill_edge_cases(m):
    cfg = mi.get_config("C2").scaled(L=2, H=256, I=64, N=8, prompt=16)
    desc = m.ModelDesc.from_config(cfg)
    cache = m.Cache(desc, cfg.L * cfg.E)
    cache.reset(cfg.L * cfg.E)
    d_eam = dev(np.zeros((cfg.L, cfg.E), dtype=np.int32))
    W = dev(mi.router_weights(cfg, 0))
    # n = 0: nothing happens
    Y = m.moe_prefill_layer(cache, d_eam, 0, W, None, dev(np.zeros((0, cfg.H), dtype=np.uint16)))
    assert Y.shape == (0, cfg.H) and int(d_eam.sum()) == 0
    with pytest.raises(m.MoeiError):
        m.moe_prefill_layer(cache, d_eam, cfg.L, W, None, dev(np.zeros((4, cfg.H), dtype=np.uint16)))
    cache.close()
    # a pick that is not resident raises the flag and contributes nothing (no fault, no garbage)
    o = _prefill_case(m, cfg, 20, layer=1, resident=cfg.E)        # only layer 0's experts are resident
    assert o["flags"] & 2
    assert (o["idx"] == o["ridx"]).all() and np.isfinite(o["Y"]).all()
    # fp32 weights are refused, not mis-read
    cfg32 = mi.get_config("C1")
    c32 = m.Cache(m.ModelDesc.from_config(cfg32), cfg32.L * cfg32.E)
    with pytest.raises(m.MoeiError):
        m.moe_prefill_layer(c32, dev(np.zeros((cfg32.L, cfg32.E), dtype=np.int32)), 0,
                            dev(mi.router_weights(cfg32, 0)), None, dev(np.zeros((4, cfg32.H), dtype=np.float32)))
    c32.close()
