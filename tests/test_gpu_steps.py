"""Per-step parity of the HIP path against the CPU oracle, through the C ABI.

Bars: bit-exact for top-k indices, EAM counts, best-match index and the
prefetch / eviction orders; 1e-5 relative for similarities and gate weights;
max|y - y_ref| / max|y_ref| <= 2e-2 for FFN outputs (and a much tighter bound that
fp32 accumulation actually meets, asserted alongside).
"""
import numpy as np
import pytest
import torch

import moei_inputs as mi
from oracle import moei_oracle as O
from tests.helpers import EPS, dev, pack_bank, pinned, rel_max_err, split_expert

pytestmark = pytest.mark.gpu

SIM_RTOL = 1e-5
FFN_TOL = 2e-2          # stated bar
FFN_TOL_FP32ACC = 2e-4  # what fp32 accumulation of <= 16K terms of bf16/fp32 products meets


@pytest.fixture(scope="module")
def m():
    import paper_2401_14361_amd as mod
    mod.lib()
    return mod


# ----------------------------------------------------------------------- step 1
@pytest.mark.parametrize("B,E,k,renorm", [
    (1, 8, 2, True), (5, 64, 6, False), (3, 160, 6, False), (2, 1, 1, True), (4, 7, 7, True),
    (2, 4096, 8, False), (2, 130, 70, True), (16, 64, 6, True), (0, 8, 2, False),
])
def test_route_topk(m, B, E, k, renorm):
    rng = np.random.default_rng(100 + E + k)
    z = rng.standard_normal((B, E)).astype(np.float32) * 3
    if B and E >= 6:
        z[0, 1] = z[0, 4] = z[0, 5] = z[0].max() + 1          # exact ties in the top set
    idx, w = m.moe_route_topk(dev(z), k, renorm)
    torch.cuda.synchronize()
    if B == 0:
        return
    ridx, rw = O.route_topk(z, k, renorm)
    assert (idx.cpu().numpy() == ridx).all()
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=SIM_RTOL, atol=1e-30)


def test_route_topk_all_equal_and_neg_inf(m):
    z = np.zeros((1, 10), dtype=np.float32)
    idx, w = m.moe_route_topk(dev(z), 4, False)
    assert idx.cpu().numpy().tolist() == [[0, 1, 2, 3]]
    np.testing.assert_allclose(w.cpu().numpy(), 0.1, rtol=1e-6)
    z = np.array([[0.5, -np.inf, 2.0, -np.inf, 1.0]], dtype=np.float32)
    idx, w = m.moe_route_topk(dev(z), 4, True)
    ridx, rw = O.route_topk(z, 4, True)
    assert (idx.cpu().numpy() == ridx).all()
    np.testing.assert_allclose(w.cpu().numpy(), rw, rtol=SIM_RTOL)


@pytest.mark.parametrize("E,k", [(10, 4), (200, 70), (1500, 8)])
def test_route_topk_logits_without_a_softmax_give_no_picks(m, E, k):
    # error path (the paper's router always has a softmax): NaN, +inf or all -inf logits give the token
    # index -1 / weight 0 for every pick; its neighbours in the batch are routed as usual
    rng = np.random.default_rng(E)
    z = rng.standard_normal((5, E)).astype(np.float32)
    z[1, E // 2] = np.nan
    z[2, :] = -np.inf
    z[3, 3] = np.inf
    idx, w = m.moe_route_topk(dev(z), k, True)
    idx, w = idx.cpu().numpy(), w.cpu().numpy()
    for b in (1, 2, 3):
        assert (idx[b] == -1).all() and (w[b] == 0).all(), b
    ridx, rw = O.route_topk(z[[0, 4]], k, True)
    assert (idx[[0, 4]] == ridx).all()
    np.testing.assert_allclose(w[[0, 4]], rw, rtol=SIM_RTOL, atol=1e-30)
    # the EAM update passes over such picks
    d_eam = dev(np.zeros((5, 2, E), dtype=np.int32))
    m.eam_update(d_eam, 1, dev(idx.astype(np.int32)))
    got = d_eam.cpu().numpy()
    assert got[[1, 2, 3]].sum() == 0 and got[0, 1].sum() == k and got[4, 1].sum() == k


# ----------------------------------------------------------------------- step 2
def test_eam_update(m):
    rng = np.random.default_rng(7)
    B, L, E, k = 3, 5, 11, 4
    eam = rng.integers(0, 9, size=(B, L, E)).astype(np.int32)
    d_eam = dev(eam)
    ref = eam.astype(np.int64)
    for step in range(12):
        layer = step % L
        idx = np.stack([rng.choice(E, size=k, replace=False) for _ in range(B)]).astype(np.int32)
        m.eam_update(d_eam, layer, dev(idx))
        for b in range(B):
            O.eam_update(ref[b], layer, idx[b])
    assert (d_eam.cpu().numpy() == ref).all()
    with pytest.raises(m.MoeiError):
        m.eam_update(d_eam, L, dev(idx))


# ----------------------------------------------------------------------- step 3
def _check_match(m, T, Q, cell_bytes, layer_hi=None):
    N, L, E = T.shape
    desc = m.ModelDesc(L, E, 1, 0, 8, 8, m.WDTYPE_BF16, 0, EPS)
    eamc = m.Eamc(desc, max(N, 1) + 3, cell_bytes)       # capacity above N: the stride is not N
    eamc.load(T)
    best, sim, sims = m.eamc_match(eamc, dev(Q.astype(np.int32)), layer_hi=layer_hi, want_sims=True)
    torch.cuda.synchronize()
    best, sim, sims = best.cpu().numpy(), sim.cpu().numpy(), sims.cpu().numpy()
    for b in range(Q.shape[0]):
        rb, rs, rsims = O.eamc_match(T, Q[b])
        assert best[b] == rb, (b, best[b], rb)
        np.testing.assert_allclose(sims[b], rsims, rtol=SIM_RTOL, atol=1e-30)
        np.testing.assert_allclose(sim[b], rs, rtol=SIM_RTOL, atol=1e-30)
    eamc.close()


@pytest.mark.parametrize("N,L,E", [(64, 4, 8), (1000, 26, 64), (37, 3, 6), (1, 1, 1), (300, 5, 160),
                                   (513, 7, 12), (70, 2, 2048), (9, 33, 100)])
@pytest.mark.parametrize("cell_bytes", [4, 2])
def test_eamc_match_shapes(m, N, L, E, cell_bytes):
    rng = np.random.default_rng(N * 7 + E)
    T = (rng.integers(0, 600, size=(N, L, E)) * (rng.random((N, L, E)) < 0.4)).astype(np.int32)
    Q = (rng.integers(0, 100, size=(3, L, E)) * (rng.random((3, L, E)) < 0.5)).astype(np.int32)
    if N > 6:
        T[5] = 3 * T[2]                                   # exact tie between traces 2 and 5
        Q[1] = T[2] * 2
        T[4] = 0                                          # an empty trace
    Q[2] = 0                                              # an empty query
    _check_match(m, T, Q, cell_bytes)


def test_eamc_match_workload_traces_and_partial_rows(m):
    cfg = mi.get_config("C2").scaled(N=300)
    T, _, _ = mi.eamc_traces(cfg)
    req = mi.make_request(cfg, 1, decode=1)
    Q = np.stack([req.prefill_eam, T[17], req.prefill_eam // 3])
    _check_match(m, T, Q, 4)
    _check_match(m, T, Q, 2)
    # iteration-level reading (Sec. 4.3): rows above the current layer are zero and are not scanned
    Qp = Q.copy()
    Qp[:, 9:] = 0
    _check_match(m, T, Qp, 4, layer_hi=8)
    _check_match(m, T, Qp, 2, layer_hi=8)


@pytest.mark.parametrize("t_hi,q_hi", [(100, 90), (100, 3_000_000), (16_000, 16_000), (2_000_000, 120),
                                       (16_777_215, 16_777_215), (130, 16_383), (65_535, 70_000)])
def test_eamc_match_batches_over_cell_sizes(m, t_hi, q_hi):
    # two and more queries are matched by a matrix product over 7-bit digits of the cells: one to
    # four digits on either side, sixteen queries and five (a partly filled group), rows of 96 cells
    # (a full 64-cell unit and half of one), a layer range that splits unevenly, an exact tie
    rng = np.random.default_rng(t_hi % 1000 + q_hi % 77)
    N, L, E = 333, 7, 96
    T = (rng.integers(0, t_hi + 1, size=(N, L, E), dtype=np.int64) * (rng.random((N, L, E)) < 0.4)).astype(np.int32)
    T[7, 3, 95] = t_hi                                    # the largest value is present, in a row's last cell
    T[9] = 0
    for B in (16, 5, 3):
        Q = (rng.integers(0, q_hi + 1, size=(B, L, E), dtype=np.int64) * (rng.random((B, L, E)) < 0.5)).astype(np.int32)
        Q[B - 1, 6, 95] = q_hi
        Q[1] = T[20]
        Q[2] = 0
        if t_hi <= 5_000_000:
            T[21] = 3 * T[20]                             # ties with trace 20 for every query
        _check_match(m, T, Q, 4)
        if int(T.max()) <= 65535:
            _check_match(m, T, Q, 2)                      # the same traces stored in 2-byte cells
    Q[:, 5:] = 0                                          # rows above the current layer are zero and are not scanned
    _check_match(m, T, Q, 4, layer_hi=4)
    if int(T.max()) <= 65535:
        _check_match(m, T, Q, 2, layer_hi=4)


@pytest.mark.parametrize("N,L,E,B", [(300, 5, 160, 6), (130, 3, 448, 16), (65, 4, 452, 7), (100, 2, 512, 8)])
def test_eamc_match_batches_over_row_widths(m, N, L, E, B):
    # rows of several 64-cell units: 2.5 units (the DeepSeek-V2 width), 7 (the most a layer split holds), 7 with
    # a ragged last one, and 8 (too wide for the matrix-core scan: served by the other kernel)
    rng = np.random.default_rng(N + E)
    T = (rng.integers(0, 900, size=(N, L, E)) * (rng.random((N, L, E)) < 0.3)).astype(np.int32)
    Q = (rng.integers(0, 200, size=(B, L, E)) * (rng.random((B, L, E)) < 0.5)).astype(np.int32)
    T[3, L - 1, E - 1] = 899
    Q[0, L - 1, E - 1] = 199
    Q[B - 1] = T[N - 1]
    _check_match(m, T, Q, 4)
    if E % 8 == 0:
        _check_match(m, T, Q, 2)


def test_eamc_match_batch_of_two_byte_cells_up_to_their_limit(m):
    # 2-byte cells hold counts up to 65,535: three 7-bit digits; queries of one to four digits
    rng = np.random.default_rng(77)
    N, L, E = 150, 6, 64
    T = (rng.integers(0, 65536, size=(N, L, E)) * (rng.random((N, L, E)) < 0.4)).astype(np.int32)
    T[11, 5, 63] = 65535
    for q_hi in (100, 20_000, 16_777_215):
        Q = (rng.integers(0, q_hi + 1, size=(9, L, E), dtype=np.int64) * (rng.random((9, L, E)) < 0.5)).astype(np.int32)
        Q[8] = T[140]
        _check_match(m, T, Q, 2)


def test_eamc_match_batch_after_an_insert_with_larger_cells(m):
    # the number of digit planes of the traces follows the largest cell ever stored: a trace inserted
    # later may raise it
    rng = np.random.default_rng(11)
    N, L, E = 80, 4, 64
    T = rng.integers(0, 100, size=(N, L, E)).astype(np.int32)
    Q = rng.integers(0, 50, size=(4, L, E)).astype(np.int32)
    desc = m.ModelDesc(L, E, 1, 0, 8, 8, m.WDTYPE_BF16, 0, EPS)
    eamc = m.Eamc(desc, N + 2, 4)
    eamc.load(T)
    big = (Q[3].astype(np.int64) * 40_000).astype(np.int32)   # parallel to query 3, cells up to 2 million
    eamc.insert(big)
    best, sim, sims = m.eamc_match(eamc, dev(Q), want_sims=True)
    torch.cuda.synchronize()
    T2 = np.concatenate([T, big[None]])
    for b in range(4):
        rb, rs, rsims = O.eamc_match(T2, Q[b])
        assert int(best.cpu()[b]) == rb
        np.testing.assert_allclose(sims.cpu().numpy()[b], rsims, rtol=SIM_RTOL, atol=1e-30)
    assert int(best.cpu()[3]) == N
    eamc.close()


def test_eamc_match_large_counts_and_empty_collection(m):
    rng = np.random.default_rng(3)
    T = rng.integers(0, 16777215, size=(40, 3, 16), dtype=np.int64).astype(np.int32)
    Q = rng.integers(0, 16777215, size=(2, 3, 16), dtype=np.int64).astype(np.int32)
    _check_match(m, T, Q, 4)
    desc = m.ModelDesc(3, 16, 1, 0, 8, 8, m.WDTYPE_BF16, 0, EPS)
    eamc = m.Eamc(desc, 5, 4)
    best, sim, _ = m.eamc_match(eamc, dev(Q), want_sims=True)
    assert best.cpu().numpy().tolist() == [-1, -1] and sim.cpu().numpy().tolist() == [0.0, 0.0]
    bad = T.copy(); bad[3, 1, 2] = -1
    with pytest.raises(m.MoeiError):
        eamc.load(bad[:5])
    assert eamc.size == 0


def test_eamc_checkpoint_file_round_trip(m, tmp_path):
    # failure recovery (App. B.2): the collection is written to a file and read back into a fresh one
    rng = np.random.default_rng(9)
    L, E, N = 5, 12, 37
    T = (rng.integers(0, 500, size=(N, L, E)) * (rng.random((N, L, E)) < 0.5)).astype(np.int32)
    desc = m.ModelDesc(L, E, 1, 0, 8, 8, m.WDTYPE_BF16, 0, EPS)
    q = dev(T[11] + 1)
    for cb in (4, 2):
        a = m.Eamc(desc, 50, cb)
        a.load(T)
        path = str(tmp_path / f"eamc{cb}.bin")
        a.save(path)
        want = [t.cpu().numpy() for t in m.eamc_match(a, q, want_sims=True)]
        a.close()
        b = m.Eamc(desc, 40, 6 - cb)                       # another capacity and cell width
        b.restore(path)
        assert b.size == N and (b.export() == T).all()
        got = [t.cpu().numpy() for t in m.eamc_match(b, q, want_sims=True)]
        assert (got[0] == want[0]).all() and (got[1] == want[1]).all() and (got[2] == want[2]).all()
        # refused files leave the collection untouched
        raw = open(path, "rb").read()
        for bad in (raw[:100], b"XXXX" + raw[4:], raw[:12] + (99).to_bytes(4, "little") + raw[16:]):
            open(path, "wb").write(bad)
            with pytest.raises(m.MoeiError):
                b.restore(path)
            assert b.size == N and (b.export() == T).all()
        small = m.Eamc(desc, N - 1, 4)
        open(path, "wb").write(raw)
        with pytest.raises(m.MoeiError):
            small.restore(path)
        with pytest.raises(m.MoeiError):
            small.restore(str(tmp_path / "missing.bin"))
        small.close()
        b.close()
    # an empty collection round-trips too
    e = m.Eamc(desc, 4, 4)
    p0 = str(tmp_path / "empty.bin")
    e.save(p0)
    e.load(T[:3])
    e.restore(p0)
    assert e.size == 0
    e.close()


def test_eamc_insert_replace_and_export(m):
    # App. B.1: at capacity the incoming EAM replaces the stored one it is most similar to
    rng = np.random.default_rng(5)
    L, E, cap = 4, 8, 6
    desc = m.ModelDesc(L, E, 1, 0, 8, 8, m.WDTYPE_BF16, 0, EPS)
    for cb in (4, 2):
        eamc = m.Eamc(desc, cap, cb)
        ref = []
        for t in range(10):
            eam = rng.integers(0, 50, size=(L, E)).astype(np.int32)
            if len(ref) < cap:
                eamc.insert(eam)
                ref.append(eam)
            else:
                best, _, _ = m.eamc_match(eamc, dev(eam))
                victim = int(best.cpu()[0])
                assert victim == O.eamc_match(np.stack(ref), eam)[0]
                eamc.insert(eam, victim)
                ref[victim] = eam
            assert (eamc.export() == np.stack(ref)).all()
        q = rng.integers(0, 50, size=(L, E)).astype(np.int32)
        best, _, _ = m.eamc_match(eamc, dev(q))
        assert int(best.cpu()[0]) == O.eamc_match(np.stack(ref), q)[0]
        # failure recovery: a reloaded dump matches identically
        e2 = m.Eamc(desc, cap, cb)
        e2.load(eamc.export())
        b2, s2, _ = m.eamc_match(e2, dev(q))
        assert int(b2.cpu()[0]) == int(best.cpu()[0])


# ----------------------------------------------------------------------- step 4
@pytest.mark.parametrize("N,L,E,B,cb", [(20, 4, 8, 1, 4), (50, 26, 64, 1, 2), (30, 7, 13, 3, 4), (5, 1, 5, 1, 4),
                                        (12, 59, 160, 2, 2)])
def test_expert_priority(m, N, L, E, B, cb):
    rng = np.random.default_rng(N + L + E)
    T = (rng.integers(0, 400, size=(N, L, E)) * (rng.random((N, L, E)) < 0.5)).astype(np.int32)
    T[:, L // 2] = 0 if L > 2 else T[:, L // 2]           # an empty row in every trace
    if N > 3:
        T[2] = T[1]                                       # identical traces: exact score ties across...
    k = min(3, E)
    desc = m.ModelDesc(L, E, k, 0, 8, 8, m.WDTYPE_BF16, 0, EPS)
    eamc = m.Eamc(desc, N, cb)
    eamc.load(T)
    for trial in range(4):
        best = rng.integers(-1 if trial == 3 else 0, N, size=B).astype(np.int32)
        cur = int(rng.integers(-1, L))
        res = rng.random((L, E)) < 0.4
        slot_of = np.where(res.reshape(-1), np.arange(L * E), -1).astype(np.int32)
        cur_idx = None
        excl = []
        if cur >= 0:
            cur_idx = np.stack([rng.choice(E, size=k, replace=False) for _ in range(B)]).astype(np.int32)
            excl = [cur * E + int(j) for j in cur_idx.reshape(-1)]
        out = m.expert_priority(eamc, dev(best), cur, dev(slot_of), EPS,
                                dev(cur_idx) if cur_idx is not None else None)
        torch.cuda.synchronize()
        P, V, pf, n_pf, ev, n_ev = [o.cpu().numpy() for o in out]
        tstar = O.aggregate_matches(T, best)
        rP, rV, rpf, rev = O.expert_priority(tstar, cur, res, EPS, excl)
        assert int(n_pf[0]) == len(rpf) and int(n_ev[0]) == len(rev)
        assert pf[:len(rpf)].tolist() == rpf
        assert ev[:len(rev)].tolist() == rev
        np.testing.assert_allclose(P, rP, rtol=1e-6, atol=0)
        np.testing.assert_allclose(V, rV, rtol=1e-6, atol=0)


def test_expert_priority_worked_example(m):
    # Sec. 4.7 example: EAM [[1,2],[0,3],[0,3]]; E[2,2] (0-based (1,1)) is kept, (1,0) and (2,0) go first
    T = np.array([[[1, 2], [0, 3], [0, 3]]], dtype=np.int32)
    desc = m.ModelDesc(3, 2, 1, 0, 8, 8, m.WDTYPE_BF16, 0, EPS)
    eamc = m.Eamc(desc, 1, 4)
    eamc.load(T)
    slot_of = np.arange(6, dtype=np.int32)
    out = m.expert_priority(eamc, dev(np.zeros(1, np.int32)), 0, dev(slot_of), EPS)
    ev = out[4].cpu().numpy()[:int(out[5].cpu()[0])].tolist()
    assert ev == [4, 2, 5, 0, 3, 1]
    out = m.expert_priority(eamc, dev(np.zeros(1, np.int32)), 0, dev(np.full(6, -1, np.int32)), EPS)
    assert out[2].cpu().numpy()[:int(out[3].cpu()[0])].tolist() == [3, 5]


# ----------------------------------------------------------------------- step 5
def _ffn_case(m, cfg, n_unique, slot_pick, gates, seed, n_slots=None):
    bank = mi.expert_bank(cfg, n_unique, threads=4)
    S = n_slots or n_unique
    desc = m.ModelDesc.from_config(cfg)
    cache = m.Cache(desc, S)
    packed = pack_bank(m, cfg, bank)
    for s in range(min(S, n_unique)):
        cache.slot_tensor(s).copy_(dev(packed[s]).view(cache.slot_tensor(s).dtype))
    n_sh = cfg.L * cfg.n_shared
    sh = mi.expert_bank(cfg.scaled(cid=cfg.cid + 50), max(n_sh, 1), threads=2)
    sh_packed = pack_bank(m, cfg, sh)
    for s in range(n_sh):
        cache.slot_tensor(S + s).copy_(dev(sh_packed[s]).view(cache.slot_tensor(S + s).dtype))
    rng = np.random.default_rng(seed)
    x = mi.to_store(cfg, rng.standard_normal(cfg.H).astype(np.float32))
    y = m.expert_ffn_gemv(cache, dev(np.asarray(slot_pick, np.int32)), dev(np.asarray(gates, np.float32)), dev(x))
    torch.cuda.synchronize()

    def weights(s):
        return split_expert(cfg, bank[s] if s < S else sh[s - S])

    ref = O.expert_ffn(x, [weights(s) for s in slot_pick], gates)
    err = rel_max_err(y.cpu().numpy(), ref)
    assert cache.error_flags() == 0
    return err, cache


@pytest.mark.parametrize("wdtype", ["bf16", "fp32"])
@pytest.mark.parametrize("H,I", [(256, 512), (2048, 1408), (200, 136), (100, 52), (520, 4104), (64, 9000),
                                 (1536, 40), (4096, 96), (5120, 48), (8192, 16), (3584, 24)])
def test_expert_ffn_shapes(m, wdtype, H, I):
    cfg = mi.get_config("C1").scaled(H=H, I=I, wdtype=wdtype, L=2, n_shared=1, k=3, E=8)
    err, cache = _ffn_case(m, cfg, 5, [3, 0, 4, 5 + 1], [0.5, 0.3, 0.2, 1.0], seed=H + I)
    assert err <= FFN_TOL_FP32ACC <= FFN_TOL, err
    cache.close()


def test_expert_ffn_edge_cases(m):
    cfg = mi.get_config("C1").scaled(H=128, I=256, wdtype="bf16", L=1, n_shared=0, k=2, E=4)
    err, cache = _ffn_case(m, cfg, 3, [1], [1.0], seed=1)
    assert err <= FFN_TOL_FP32ACC
    x = dev(mi.to_store(cfg, np.ones(cfg.H, np.float32)))
    # no active expert: y = 0
    y = m.expert_ffn_gemv(cache, dev(np.zeros(0, np.int32)), dev(np.zeros(0, np.float32)), x)
    assert (y.cpu().numpy() == 0).all()
    # a slot id outside the pool contributes nothing and raises the flag
    y_ok = m.expert_ffn_gemv(cache, dev(np.array([2], np.int32)), dev(np.array([0.7], np.float32)), x).cpu().numpy()
    y_bad = m.expert_ffn_gemv(cache, dev(np.array([2, 99], np.int32)), dev(np.array([0.7, 1.0], np.float32)), x).cpu().numpy()
    assert (y_ok == y_bad).all()
    assert cache.error_flags() & 1
    assert cache.error_flags() == 0
    with pytest.raises(m.MoeiError):
        m.expert_ffn_gemv(cache, dev(np.zeros(3, np.int32)), dev(np.zeros(3, np.float32)), x)
    # deterministic: repeated runs give identical bits
    ids, g = dev(np.array([0, 1], np.int32)), dev(np.array([0.4, 0.6], np.float32))
    y0 = m.expert_ffn_gemv(cache, ids, g, x).cpu().numpy()
    for _ in range(20):
        assert (m.expert_ffn_gemv(cache, ids, g, x).cpu().numpy() == y0).all()
    cache.close()


def test_expert_ffn_full_deepseek_v2_lite_layer(m):
    # the benchmark shape: 6 routed + 2 shared experts of 2048 x 1408, bf16
    cfg = mi.get_config("C2").scaled(L=1)
    err, cache = _ffn_case(m, cfg, 7, [5, 0, 3, 6, 1, 2, 7, 8], [0.21, 0.18, 0.12, 0.09, 0.07, 0.05, 1.0, 1.0],
                           seed=2, n_slots=7)
    assert err <= FFN_TOL_FP32ACC, err
    cache.close()


# ------------------------------------------------------------------ full benchmark sizes
def test_eamc_match_and_priority_at_deepseek_v2_size(m):
    # configuration 4 / 5 sizes: 10,000 traces of 59 x 160 (378 MB of int32 cells), batched queries
    cfg = mi.get_config("C4")
    T, _, _ = mi.eamc_traces(cfg, threads=16)
    reqs = [mi.make_request(cfg.scaled(prompt=256), r, decode=1) for r in range(4)]
    Q = np.stack([r.prefill_eam for r in reqs] + [T[4321], 3 * T[77]]).astype(np.int32)
    desc = m.ModelDesc.from_config(cfg)
    for cb in (4, 2):
        eamc = m.Eamc(desc, cfg.N, cb)
        eamc.load(T)
        best, sim, sims = m.eamc_match(eamc, dev(Q), want_sims=True)
        torch.cuda.synchronize()
        best, sim, sims = best.cpu().numpy(), sim.cpu().numpy(), sims.cpu().numpy()
        for b in range(Q.shape[0]):
            rb, rs, rsims = O.eamc_match(T, Q[b])
            assert best[b] == rb
            np.testing.assert_allclose(sims[b], rsims, rtol=SIM_RTOL, atol=1e-30)
            np.testing.assert_allclose(sim[b], rs, rtol=SIM_RTOL)
        assert best[4] == 4321 and best[5] == 77
        # priorities from the first request's match, a third of the experts resident
        rng = np.random.default_rng(cb)
        res = rng.random((cfg.L, cfg.E)) < 0.33
        slot_of = np.where(res.reshape(-1), np.arange(cfg.L * cfg.E), -1).astype(np.int32)
        cur = 20
        cur_idx = rng.choice(cfg.E, size=(1, cfg.k), replace=False).astype(np.int32)
        out = m.expert_priority(eamc, dev(best[:1].astype(np.int32)), cur, dev(slot_of), EPS, dev(cur_idx))
        torch.cuda.synchronize()
        P, V, pf, n_pf, ev, n_ev = [o.cpu().numpy() for o in out]
        rP, rV, rpf, rev = O.expert_priority(O.aggregate_matches(T, best[:1]), cur, res, EPS,
                                             [cur * cfg.E + int(j) for j in cur_idx[0]])
        assert pf[:int(n_pf[0])].tolist() == rpf and ev[:int(n_ev[0])].tolist() == rev
        np.testing.assert_allclose(P, rP, rtol=1e-6)
        np.testing.assert_allclose(V, rV, rtol=1e-6)
        eamc.close()
