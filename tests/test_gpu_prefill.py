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


def _route_all(cfg, eam, layer, W, bias, X):
    """The oracle's routing decision and EAM update for every token of the prompt (no expert runs)."""
    n = X.shape[0]
    idx = np.zeros((n, cfg.k), dtype=np.int64)
    w = np.zeros((n, cfg.k), dtype=np.float64)
    for t in range(n):
        i_t, w_t = O.route_topk(O.router_logits(W, X[t], bias), cfg.k, bool(cfg.renorm))
        idx[t], w[t] = i_t[0], w_t[0]
        O.eam_update(eam, layer, idx[t])
    return idx, w


def _prefill_case(m, cfg, n, layer, n_unique=None, resident=None, sample=None, nan_token=None):
    """With ``sample`` (a token count) the oracle routes every token (picks, gate weights, EAM) but
    runs the expert FFNs only for that many tokens spread evenly over the prompt: at full width it
    needs a quarter of a second per token."""
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
    X_dev = X
    if nan_token is not None:   # the device sees a NaN in this token; the oracle is not asked about it
        X_dev = X.copy()
        X_dev[nan_token, 3] = 0x7FC0 if X.dtype == np.uint16 else np.nan
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
    Y, idx, w = m.moe_prefill_layer(cache, d_eam, layer, dev(W), dev(req.bias[layer]), dev(X_dev), want_picks=True)
    torch.cuda.synchronize()
    ref_eam = eam0.astype(np.int64).copy()
    expert_of = lambda f: split_expert(cfg, bank[f % n_unique])
    shared_of = lambda l: [split_expert(cfg, shared[l * cfg.n_shared + s]) for s in range(cfg.n_shared)]
    rows_y = None
    if sample is None:
        ridx, rw, rY = O.prefill_layer(ref_eam, layer, W, req.bias[layer], X, expert_of, shared_of, k, bool(cfg.renorm))
    else:
        # routing of all tokens without any expert (H -> picks only), outputs of the sampled tokens
        ridx, rw = _route_all(cfg, ref_eam, layer, W, req.bias[layer], X)
        rows_y = np.unique(np.linspace(0, n - 1, sample).astype(np.int64))
        scratch_eam = np.zeros_like(ref_eam)
        _, _, rY = O.prefill_layer(scratch_eam, layer, W, req.bias[layer], X[rows_y], expert_of, shared_of, k,
                                   bool(cfg.renorm))
    flags = cache.error_flags()
    Yh = Y.cpu().numpy()
    out = dict(idx=idx.cpu().numpy(), w=w.cpu().numpy(), Y=Yh if rows_y is None else Yh[rows_y], eam=d_eam.cpu().numpy(),
               ridx=ridx, rw=rw, rY=rY, ream=ref_eam, eam0=eam0, flags=flags, finite=bool(np.isfinite(Yh).all()))
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
    # tile, and prompts long enough (n k >= 48 E) that the items hold up to 256 tokens
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


def test_prefill_long_prompts_with_256_token_items(m):
    # n k > 128 E: the items hold up to 256 tokens and the gate/up products run in the kernel that
    # fills its LDS ring straight from global memory.  Mixtral structure, I = 72 (less than one
    # 128-unit block); then top-2 of 8 with two shared experts, I = 200 (a ragged second block),
    # H = 384 (twelve 32-wide stages), most experts with a full item and a ragged one
    cfg = mi.get_config("C3").scaled(L=2, H=512, I=72, N=8, prompt=16)
    _check(_prefill_case(m, cfg, 700, layer=1))
    cfg = mi.get_config("C2").scaled(L=2, E=8, k=2, H=384, I=200, N=8, prompt=16)
    _check(_prefill_case(m, cfg, 1100, layer=0))
    # an item of exactly 256 tokens and its neighbours (one expert, every token picks it)
    cfg = mi.get_config("C3").scaled(L=1, E=2, k=2, H=256, I=128, N=8, prompt=16)
    for n in (255, 256, 257):
        _check(_prefill_case(m, cfg, n, layer=0))


@pytest.mark.parametrize("tile", [64, 128, 256])
def test_prefill_every_item_size_on_one_prompt(m, tile, monkeypatch):
    # the item size is chosen from the prompt length; MOEI_PREFILL_TILE (read at every call) forces one, so
    # that each pair of matrix kernels serves the same prompt: 64- and 128-token items through the
    # kernels that stage through registers, 256-token items through the LDS-ring kernels (a prompt
    # shorter than their tile: most of the input rows of an item are absent and are not loaded)
    monkeypatch.setenv("MOEI_PREFILL_TILE", str(tile))
    cfg = mi.get_config("C2").scaled(L=2, E=8, k=2, H=256, I=128, N=8, prompt=16)
    _check(_prefill_case(m, cfg, 150, layer=1))
    _check(_prefill_case(m, cfg, 9, layer=0))


@pytest.mark.parametrize("E,k,n", [(40, 4, 1030), (100, 6, 1027), (160, 6, 1100), (256, 8, 1277)])
def test_prefill_long_prompt_routing_over_expert_counts(m, E, k, n):
    # prompts of 512 tokens and more form their logits in the routing kernel that runs on the matrix
    # cores, sixteen tokens per workgroup: fewer row groups than wavefronts (E = 40), a ragged last
    # 16-expert block (100), three and four blocks per wavefront (160, 256); n is no multiple of 16.
    # Every token's picks, gate weights and the EAM in full, the outputs of 12 sampled tokens.
    cfg = mi.get_config("C2").scaled(L=1, E=E, k=k, H=256, I=64, N=8, prompt=16)
    _check(_prefill_case(m, cfg, n, layer=0, sample=12))


def test_prefill_long_prompt_with_a_token_without_softmax(m):
    # the same kernel meets a NaN logit: that token alone gets no picks
    cfg = mi.get_config("C2").scaled(L=1, H=256, I=64, N=8, prompt=16)
    n, bad = 1040, 1033
    o = _prefill_case(m, cfg, n, layer=0, nan_token=bad, sample=12)
    assert o["flags"] & 4 and (o["idx"][bad] == -1).all() and (o["w"][bad] == 0).all()
    keep = [t for t in range(n) if t != bad]
    assert (o["idx"][keep] == o["ridx"][keep]).all()
    np.testing.assert_allclose(o["w"][keep], o["rw"][keep], rtol=1e-4)
    assert int(o["eam"][0].sum() - o["eam0"][0].sum()) == (n - 1) * cfg.k


def test_prefill_wide_rows(m):
    cfg = mi.get_config("C3").scaled(L=1, H=4096, I=160, N=8, prompt=16)
    _check(_prefill_case(m, cfg, 40, layer=0, n_unique=4))
    # the widest rows with 256-token items: 64 ring stages in the gate/up product, three in the down product
    cfg = mi.get_config("C3").scaled(L=1, H=4096, I=192, N=8, prompt=16)
    _check(_prefill_case(m, cfg, 600, layer=0, n_unique=4))


def test_prefill_full_width_deepseek_v2_lite_layer(m):
    # configuration 2 at full width (2048 x 1408 bf16 experts), one layer, a 512-token prompt (48 tokens per
    # expert on average: 256-token items, most of them a fifth full)
    cfg = mi.get_config("C2").scaled(L=1, N=8, prompt=16)
    o = _prefill_case(m, cfg, 512, layer=0, n_unique=16)
    _check(o)


def test_prefill_full_width_short_prompt_with_64_token_items(m):
    # the same layer with a 200-token prompt, which takes the 64-token items and the kernels that stage
    # through registers; every token's picks, gate weights and the EAM in full, the outputs of 24 sampled tokens
    cfg = mi.get_config("C2").scaled(L=1, N=8, prompt=16)
    o = _prefill_case(m, cfg, 200, layer=0, n_unique=16, sample=24)
    assert o["finite"]
    _check(o)


def test_prefill_full_width_1024_token_prompt(m):
    # configuration 2 at full width with a 1,024-token prompt: n k >= 48 E, so the items hold up to 256
    # tokens (96 on average: partly filled items); every token's picks, gate weights and the EAM in
    # full, the outputs of 40 sampled tokens
    cfg = mi.get_config("C2").scaled(L=1, N=8, prompt=16)
    o = _prefill_case(m, cfg, 1024, layer=0, n_unique=16, sample=40)
    assert o["finite"]
    _check(o)


def test_prefill_full_width_2048_token_prompt_with_256_token_items(m):
    # configuration 2 at full width with a 2,048-token prompt: n k > 128 E, items of up to 256 tokens;
    # every token's picks, gate weights and the EAM in full, the outputs of 40 sampled tokens
    cfg = mi.get_config("C2").scaled(L=1, N=8, prompt=16)
    o = _prefill_case(m, cfg, 2048, layer=0, n_unique=16, sample=40)
    assert o["finite"]
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
    # a token whose router logits have no softmax (NaN in its input): flag bit 2, no picks, its
    # output is the shared experts' alone (NaN here, as its input is); the other tokens are served as usual
    o = _prefill_case(m, cfg, 12, layer=0, nan_token=4)
    assert o["flags"] & 4 and (o["idx"][4] == -1).all() and (o["w"][4] == 0).all()
    keep = [t for t in range(12) if t != 4]
    assert (o["idx"][keep] == o["ridx"][keep]).all()
    assert rel_max_err(o["Y"][keep], o["rY"][keep]) <= FFN_TOL_BF16_ACT
    assert int(o["eam"][0].sum() - o["eam0"][0].sum()) == 11 * cfg.k
    # fp32 weights are refused, not mis-read
    cfg32 = mi.get_config("C1")
    c32 = m.Cache(m.ModelDesc.from_config(cfg32), cfg32.L * cfg32.E)
    with pytest.raises(m.MoeiError):
        m.moe_prefill_layer(c32, dev(np.zeros((cfg32.L, cfg32.E), dtype=np.int32)), 0,
                            dev(mi.router_weights(cfg32, 0)), None, dev(np.zeros((4, cfg32.H), dtype=np.float32)))
    c32.close()
