"""The seeded input generators: shapes, invariants and reproducibility (CPU only)."""
import numpy as np
import torch

import moei_inputs as mi


def test_bf16_rounding_matches_torch_round_to_nearest_even():
    rng = np.random.default_rng(0)
    a = (rng.standard_normal(10000) * 10.0 ** rng.integers(-6, 6, size=10000)).astype(np.float32)
    a[:4] = [1.00390625, 1.01171875, -1.00390625, 0.0]      # exact ties: go to the even mantissa
    bits = mi.f32_to_bf16_bits(a)
    ref = torch.from_numpy(a).to(torch.bfloat16)
    assert (bits == ref.view(torch.int16).numpy().view(np.uint16)).all()
    assert (mi.bf16_bits_to_f32(bits) == ref.float().numpy()).all()


def test_trace_counts_have_the_eam_row_properties():
    cfg = mi.get_config("C2").scaled(N=40)
    T, cl, rt = mi.eamc_traces(cfg, threads=2)
    assert T.shape == (40, cfg.L, cfg.E) and T.dtype == np.int32
    assert (T.sum(axis=2) == (rt * cfg.k)[:, None]).all()     # every layer row sums to r*k
    assert (T.max(axis=(1, 2)) <= rt).all() and T.min() >= 0   # a token picks k distinct experts
    assert ((32 <= rt) & (rt <= 512)).all() and set(cl) <= set(range(cfg.n_clusters))
    T2, _, _ = mi.eamc_traces(cfg, threads=1)
    assert (T == T2).all()                                     # seeded, thread-count independent


def test_counts_cap_redistribution():
    rng = np.random.default_rng(1)
    p = np.array([[0.9, 0.05, 0.03, 0.02]] * 5)
    c = mi.counts_from_preferences(rng, p, [10, 1, 100, 7, 0], 2)
    assert (c.sum(axis=1) == np.array([20, 2, 200, 14, 0])).all()
    assert (c <= np.array([10, 1, 100, 7, 0])[:, None]).all()
    assert (c[:3, 0] == [10, 1, 100]).all()                    # the dominant expert saturates


def test_request_and_weights_are_reproducible_and_shaped():
    cfg = mi.get_config("C1")
    r1, r2 = mi.make_request(cfg, 5), mi.make_request(cfg, 5)
    assert (r1.x == r2.x).all() and (r1.bias == r2.bias).all() and (r1.prefill_eam == r2.prefill_eam).all()
    assert r1.x.shape == (cfg.decode, cfg.L, cfg.H) and r1.x.dtype == np.float32
    assert (r1.prefill_eam.sum(axis=1) == cfg.prompt * cfg.k).all()
    np.testing.assert_allclose(np.exp(r1.bias.astype(np.float64)).sum(axis=1), 1.0, rtol=1e-5)
    w = mi.expert_weights(cfg, 3)
    assert w.shape == (cfg.expert_elems,) and abs(float(w.std()) - cfg.w_std) < 1e-3
    bank = mi.expert_bank(cfg, 4, threads=2)
    assert (bank[3] == w).all()
    c3 = mi.get_config("C3").scaled(N=8, H=64, I=32)
    rq = mi.make_request(c3, 0, decode=2)
    assert rq.x.dtype == np.uint16 and 0 <= rq.source < 8
    assert mi.router_weights(c3, 1).shape == (c3.E, 64)
