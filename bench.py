#!/usr/bin/env python3
"""Benchmark of the MoE decode layer step on one MI355X.

A "step" is one pass of the whole hot path for one MoE layer of one decode token:
router top-k, EAM update, EAMC match, priorities, slot lookup and the expert FFNs.
The default workload is the DeepSeek-V2-Lite-shaped configuration (C2): 26 layers,
64 routed experts top-6 + 2 shared, hidden 2048, intermediate 1408, bf16 weights,
EAMC of 1,000 traces, one request of 128 decode tokens.

Legs (all in this one process, so one rocprofv3 run covers them):
  1. resident replay (value): every expert in HBM, asynchronous layer steps, wall time
     over exactly --steps steps after --warmup steps;
  2. the same steps again with a start/stop HIP event pair on every kernel launch:
     average launch duration per kernel -> the roofline object (dominant kernel);
  3. eamc_match and expert_ffn_gemv on their own (traces/s, GB/s);
  4. offload replay: cache capped at 25 % of the routed experts, misses filled from
     pinned host memory (PCIe-inclusive, reported beside, never as `value`);
  5. the CPU oracle timed on a bounded sample of the same steps.
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0   # MI355X published HBM3E bandwidth


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="layer steps timed (default: one request's decode, tokens*L)")
    ap.add_argument("--warmup", type=int, default=None)
    ap.add_argument("--config", default="C2", choices=["C1", "C2", "C3", "C4"])
    ap.add_argument("--unique", type=int, default=16, help="distinct experts drawn on the host; slots repeat them")
    ap.add_argument("--offload-tokens", type=int, default=12)
    ap.add_argument("--cpu-steps", type=int, default=None, help="oracle layer steps timed (default: sized to ~15 s)")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-offload", action="store_true")
    ap.add_argument("--prefill", action="store_true", help="time the prefill iteration of one layer (extra.prefill)")
    ap.add_argument("--prefill-max", type=int, default=2048)
    ap.add_argument("--policy-sweep", action="store_true",
                    help="offload replay under each eviction rule and with prefetching (extra.policy_sweep)")
    ap.add_argument("--policy-tokens", type=int, default=16, help="decode tokens per request in the policy sweep")
    ap.add_argument("--policy-requests", type=int, default=6)
    ap.add_argument("--no-graph", action="store_true")
    ap.add_argument("--no-shapes", action="store_true",
                    help="skip the FFN kernel at the C3/C4 widths, the full C4 match (extra.other_shapes) and the short "
                         "decode-batch and prefill legs of the default run")
    ap.add_argument("--batch-sweep", action="store_true",
                    help="also time the batched match and grouped FFN for B = 1..16 (EAMC of 10,000 traces)")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also run a plain 512 MiB device copy (scale for rocprofv3 FETCH_SIZE / WRITE_SIZE)")
    return ap.parse_args()


def read_traffic(kernel: str, workload: str):
    """HBM bytes per launch from the committed rocprofv3 --pmc summary, if there is one."""
    p = os.path.join(ROOT, "profiles", f"{kernel}_{workload}_hbm_traffic.txt")
    if not os.path.exists(p):
        return None
    for line in open(p):
        if line.startswith("traffic_bytes_per_launch="):
            return float(line.split("=", 1)[1])
    return None


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import moei_inputs as mi
    import paper_2401_14361_amd as m
    from moei_inputs.plumbing import EPS, dev, pack_bank, pinned, split_expert

    if not os.path.exists(m.lib_path()):
        from paper_2401_14361_amd.build import build
        build()
    m.lib()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)

    cfg = mi.get_config(args.config)
    slice_note = ""
    if cfg.L * cfg.E * cfg.expert_bytes > 200e9:
        # the whole expert set does not fit in HBM next to everything else (DeepSeek-V2-shaped: 445 GB):
        # the replay runs on the first layers whose experts fill the configuration's slot pool
        L_fit = max(1, min(cfg.L, cfg.S // cfg.E))
        slice_note = f" (the first {L_fit} of {cfg.L} layers: {L_fit * cfg.E} experts fill the pool)"
        cfg = cfg.scaled(L=L_fit)
    L, E, k, H, I = cfg.L, cfg.E, cfg.k, cfg.H, cfg.I
    n_act = k + cfg.n_shared
    T_dec = cfg.decode
    # The timed unit is a whole decode token (L layer steps, one HIP graph): --steps and --warmup are
    # rounded up to whole tokens, at least 10 tokens are timed, and the JSON line reports the steps
    # that were actually timed.
    K_req = args.steps if args.steps is not None else T_dec * L
    W_req = args.warmup if args.warmup is not None else 4 * L
    tok_timed = max(10, -(-K_req // L))
    tok_warm = max(1, -(-W_req // L))
    K, W = tok_timed * L, tok_warm * L
    t_setup = time.time()

    # ------------------------------------------------------------------ inputs
    log(f"[bench] {cfg.name}: L={L} E={E} k={k}+{cfg.n_shared} H={H} I={I} {cfg.wdtype} N={cfg.N}")
    traces, _, _ = mi.eamc_traces(cfg, threads=8)
    req = mi.make_request(cfg, 0)
    n_unique = min(args.unique, L * E)
    bank = mi.expert_bank(cfg, n_unique, threads=8)
    shared = mi.expert_bank(cfg.scaled(cid=cfg.cid + 50), max(min(L * cfg.n_shared, 4), 1), threads=4)
    routers = [dev(mi.router_weights(cfg, l)) for l in range(L)]
    d_bias = dev(req.bias)
    d_x = dev(req.x)
    desc = m.ModelDesc.from_config(cfg)
    eamc = m.Eamc(desc, cfg.N, 4)
    eamc.load(traces)
    log(f"[bench] inputs drawn in {time.time() - t_setup:.1f}s")

    # resident pool: every routed expert has a slot (MI355X holds the whole model's experts)
    S_res = L * E
    cache = m.Cache(desc, S_res)
    bank_slots, shared_slots = pack_bank(m, cfg, bank), pack_bank(m, cfg, shared)     # slot layout
    d_bank = [dev(bank_slots[u]) for u in range(n_unique)]
    d_shared = [dev(shared_slots[u]) for u in range(shared.shape[0])]
    for s in range(S_res):
        t = cache.slot_tensor(s)
        t.copy_(d_bank[s % n_unique].view(t.dtype))
    for s in range(L * cfg.n_shared):
        t = cache.slot_tensor(S_res + s)
        t.copy_(d_shared[s % len(d_shared)].view(t.dtype))
    cache.reset(min(S_res, L * E))          # marks flat ids 0..S-1 resident (no host copy: nothing is moved)
    torch.cuda.synchronize()
    d_eam = dev(req.prefill_eam.astype(np.int32))
    prefill = d_eam.clone()
    y = torch.empty(H, dtype=torch.float32, device="cuda")
    stream = torch.cuda.current_stream()

    def layer_step(i, sync=False, c=cache):
        t, l = (i // L) % T_dec, i % L
        return m.moe_decode_layer(c, eamc, d_eam, l, routers[l], d_bias[l], d_x[t, l], y, sync=sync, stream=stream)

    # ------------------------------------------------ leg 1: resident replay, wall clock
    for i in range(W):
        layer_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        layer_step(W + i)
    torch.cuda.synchronize()
    us_step_eager = (time.perf_counter() - t0) / K * 1e6
    log(f"[bench] resident replay, one launch sequence per layer step: {us_step_eager:.1f} us per layer step")
    us_step, mode = us_step_eager, "asynchronous layer steps, launched one by one"

    # the same steps with one token's L layer steps captured in a HIP graph: the layer inputs
    # sit in a fixed staging buffer that is refreshed per token (in a model the previous
    # layer writes them there)
    if not args.no_graph:
        d_eam.copy_(prefill)
        x_stage = torch.empty_like(d_x[0])
        y_all = torch.empty((L, H), dtype=torch.float32, device="cuda")
        cache.sync()
        cap = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=cap):
            for l in range(L):
                m.moe_decode_layer(cache, eamc, d_eam, l, routers[l], d_bias[l], x_stage[l], y_all[l], sync=False)
            cache.join()
        cache.sync()

        def token(t):
            x_stage.copy_(d_x[t % T_dec])
            graph.replay()

        for t in range(W // L):
            token(t)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for t in range(K // L):
            token(W // L + t)
        torch.cuda.synchronize()
        us_step_graph = (time.perf_counter() - t0) / K * 1e6
        log(f"[bench] resident replay, one HIP graph per token: {us_step_graph:.1f} us per layer step")
        if us_step_graph < us_step:
            us_step, mode = us_step_graph, f"asynchronous layer steps, one HIP graph per token ({L} layer steps)"
    flags = cache.error_flags()
    assert flags == 0, f"device error flags {flags}"

    # ------------------------------------------------ leg 2: per-kernel durations (HIP events)
    d_eam.copy_(prefill)
    n_prof = min(K, 40 * L)
    m.profile_enable(n_prof * 12)
    for i in range(n_prof):
        layer_step(W + i)
    torch.cuda.synchronize()
    prof = m.profile_read()
    kern = {name: dict(launches=n, avg_us=(ms / n * 1e3 if n else None)) for name, (n, ms) in prof.items()}
    for name in kern:
        if kern[name]["launches"]:
            smp = m.profile_samples(name)
            kern[name]["median_us"] = float(np.median(smp))
            kern[name]["p95_us"] = float(np.percentile(smp, 95))
    m.profile_disable()
    wb = cfg.wbytes
    alg_bytes = {
        "ffn_fused_kernel": n_act * 3 * H * I * wb,
        "eamc_dot_kernel": cfg.N * L * E * 4,
        "route_topk_kernel": E * H * wb,
    }
    for name, b in alg_bytes.items():
        if kern.get(name, {}).get("avg_us"):
            kern[name]["alg_bytes"] = b
            kern[name]["GBps"] = b / kern[name]["avg_us"] / 1e3
    dom = max((n for n in kern if kern[n]["avg_us"]), key=lambda n: kern[n]["avg_us"] * kern[n]["launches"])
    achieved = kern[dom].get("GBps")
    roofline = {
        "bound": "hbm", "kernel": dom, "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
        "frac": (achieved / HBM_PEAK_GBPS) if achieved else None,
        "alg_bytes_per_launch": kern[dom].get("alg_bytes"), "avg_launch_us": kern[dom]["avg_us"],
        "median_launch_us": kern[dom].get("median_us"), "p95_launch_us": kern[dom].get("p95_us"),
        "traffic": read_traffic(dom, cfg.name),
    }
    ffn_us = sum(kern[n]["avg_us"] or 0 for n in ("ffn_fused_kernel", "ffn_reduce_kernel"))
    ffn_bytes = n_act * 3 * H * I * wb
    log(f"[bench] kernels: " + ", ".join(f"{n}={v['avg_us']:.2f}us" for n, v in kern.items() if v["avg_us"]))

    if args.calib_copy:
        src = torch.empty(512 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ------------------------------------------------ leg 3: steps on their own
    extra = {}
    # eamc_match alone (launch-inclusive: both of its kernels, back to back)
    reps = 200
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(10):
        m.eamc_match(eamc, d_eam, stream=stream)
    ev0.record(stream)
    for _ in range(reps):
        m.eamc_match(eamc, d_eam, stream=stream)
    ev1.record(stream)
    torch.cuda.synchronize()
    match_us = ev0.elapsed_time(ev1) / reps * 1e3
    extra["eamc_match"] = {
        "N": cfg.N, "us_per_match": match_us, "traces_per_s": cfg.N / match_us * 1e6,
        "alg_bytes": cfg.N * L * E * 4 + cfg.N * 8, "GBps": (cfg.N * L * E * 4 + cfg.N * 8) / match_us / 1e3,
        "note": "scan smaller than launch latency and the 256 MB last-level cache: not an HBM measurement",
    }
    # the same shape with the collection grown until the scan cannot stay in cache (> 512 MB)
    big_n = int(np.ceil(640e6 / (L * E * 4) / cfg.N)) * cfg.N
    big = np.tile(traces, (big_n // cfg.N, 1, 1))
    eamc_big = m.Eamc(desc, big_n, 4)
    eamc_big.load(big)
    del big
    for _ in range(3):
        m.eamc_match(eamc_big, d_eam, stream=stream)
    m.profile_enable(64)
    for _ in range(20):
        m.eamc_match(eamc_big, d_eam, stream=stream)
    torch.cuda.synchronize()
    pb = m.profile_read()
    m.profile_disable()
    dot_us = pb["eamc_dot_kernel"][1] / pb["eamc_dot_kernel"][0] * 1e3
    arg_us = pb["eamc_pick_kernel"][1] / pb["eamc_pick_kernel"][0] * 1e3
    big_bytes = big_n * L * E * 4
    extra["eamc_match_hbm_bound"] = {
        "N": big_n, "dot_kernel_us": dot_us, "pick_kernel_us": arg_us, "alg_bytes": big_bytes,
        "GBps": big_bytes / dot_us / 1e3, "frac_of_peak": big_bytes / dot_us / 1e3 / HBM_PEAK_GBPS,
        "traces_per_s": big_n / (dot_us + arg_us) * 1e6,
        "note": f"the {cfg.N} traces tiled {big_n // cfg.N}x so that the scan ({big_bytes / 1e6:.0f} MB) exceeds the cache",
    }
    eamc_big.close()
    # the dominant kernel against what a read-only streaming kernel reaches on this machine
    if roofline["achieved"]:
        roofline["measured_stream_GBps"] = big_bytes / dot_us / 1e3
        roofline["frac_of_measured_stream"] = roofline["achieved"] / roofline["measured_stream_GBps"]
    # expert_ffn_gemv alone over rotating slots (launch-inclusive)
    rng = np.random.default_rng(0)
    n_sets = 64
    slot_sets = [dev(np.concatenate([rng.choice(S_res, size=k, replace=False),
                                     S_res + (s % L) * cfg.n_shared + np.arange(cfg.n_shared)]).astype(np.int32))
                 for s in range(n_sets)]
    gates = dev(np.full(n_act, 0.125, np.float32))
    for s in range(8):
        m.expert_ffn_gemv(cache, slot_sets[s], gates, d_x[0, 0], stream=stream, out=y)
    ev0.record(stream)
    for r in range(reps):
        m.expert_ffn_gemv(cache, slot_sets[r % n_sets], gates, d_x[0, 0], stream=stream, out=y)
    ev1.record(stream)
    torch.cuda.synchronize()
    gemv_us = ev0.elapsed_time(ev1) / reps * 1e3
    # the same calls with per-launch stamps: the FFN kernel on its own, nothing overlapped; the
    # call with no active expert launches only an (almost) empty kernel -> the launch floor
    m.profile_enable(512)
    for r in range(100):
        m.expert_ffn_gemv(cache, slot_sets[r % n_sets], gates, d_x[0, 0], stream=stream, out=y)
    torch.cuda.synchronize()
    ps = m.profile_read()
    m.profile_disable()
    ffn_alone_us = ps["ffn_fused_kernel"][1] / ps["ffn_fused_kernel"][0] * 1e3
    none_i = torch.zeros(0, dtype=torch.int32, device="cuda")
    none_f = torch.zeros(0, dtype=torch.float32, device="cuda")
    m.profile_enable(64)
    for r in range(50):
        m.expert_ffn_gemv(cache, none_i, none_f, d_x[0, 0], stream=stream, out=y)
    torch.cuda.synchronize()
    pf = m.profile_read()
    m.profile_disable()
    floor_us = pf["ffn_reduce_kernel"][1] / pf["ffn_reduce_kernel"][0] * 1e3
    extra["expert_ffn_gemv"] = {
        "us_per_call": gemv_us, "alg_bytes": ffn_bytes, "GBps_launch_inclusive": ffn_bytes / gemv_us / 1e3,
        "GBps_kernels_only": ffn_bytes / ffn_us / 1e3, "frac_of_peak_kernels_only": ffn_bytes / ffn_us / 1e3 / HBM_PEAK_GBPS,
        "frac_of_peak_launch_inclusive": ffn_bytes / gemv_us / 1e3 / HBM_PEAK_GBPS,
        "ffn_fused_kernel_alone_us": ffn_alone_us, "ffn_fused_kernel_alone_GBps": ffn_bytes / ffn_alone_us / 1e3,
        "ffn_fused_kernel_alone_frac_of_peak": ffn_bytes / ffn_alone_us / 1e3 / HBM_PEAK_GBPS,
        "near_empty_kernel_us": floor_us,
    }
    log(f"[bench] match {match_us:.1f} us; big-N dot {dot_us:.1f} us = {big_bytes / dot_us / 1e3:.0f} GB/s; "
        f"gemv {gemv_us:.1f} us = {ffn_bytes / gemv_us / 1e3:.0f} GB/s")

    # ------------------------------------------------ leg 3b: the two streaming kernels at the other shapes
    # expert_ffn_gemv at the Mixtral (C3) and DeepSeek-V2 (C4) widths over rotating slots, and the
    # EAMC match over the full DeepSeek-V2 collection (10,000 x 59 x 160 cells, 377.6 MB): per-launch
    # kernel durations from the start/stop stamps, algorithmic bytes / duration against the HBM peak
    if not args.no_shapes and cfg.name == "C2":
        shapes = {}
        for cname, n_rot in (("C3", 8), ("C4", 64)):
            scfg = mi.get_config(cname).scaled(L=1)
            sdesc = m.ModelDesc.from_config(scfg)
            na = scfg.k + scfg.n_shared
            sc = m.Cache(sdesc, n_rot)
            gen = torch.Generator(device="cuda").manual_seed(mi.BASE_SEED + scfg.cid)
            for sl in range(n_rot):          # N(0, 0.02) weights in storage precision, drawn on the device
                t = sc.slot_tensor(sl)
                t.copy_((torch.randn(t.numel(), device="cuda", generator=gen) * scfg.w_std).to(t.dtype))
            sc.reset(0)
            sx = dev(mi.to_store(scfg, np.random.default_rng(scfg.cid).standard_normal(scfg.H).astype(np.float32)))
            sy = torch.empty(scfg.H, dtype=torch.float32, device="cuda")
            sets = [dev(((np.arange(na) + r * na) % n_rot).astype(np.int32)) for r in range(n_rot // na)]
            sg = dev(np.full(na, 1.0 / na, np.float32))
            n_call = 40
            for r in range(4):
                m.expert_ffn_gemv(sc, sets[r % len(sets)], sg, sx, stream=stream, out=sy)
            m.profile_enable(4 * n_call)
            for r in range(n_call):
                m.expert_ffn_gemv(sc, sets[r % len(sets)], sg, sx, stream=stream, out=sy)
            torch.cuda.synchronize()
            smp = m.profile_samples("ffn_fused_kernel")
            m.profile_disable()
            assert sc.error_flags() == 0 and bool(torch.isfinite(sy).all())
            b = na * scfg.expert_bytes
            us = float(np.mean(smp))
            shapes[f"ffn_fused_kernel_{cname}"] = {
                "workload": f"{cname} width: {na} experts of H={scfg.H}, I={scfg.I} bf16 per launch, rotating over "
                            f"{n_rot} slots ({n_rot * scfg.expert_bytes / 1e9:.1f} GB)",
                "launches": len(smp), "avg_us": us, "median_us": float(np.median(smp)),
                "alg_bytes": b, "GBps": b / us / 1e3, "frac": b / us / 1e3 / HBM_PEAK_GBPS}
            log(f"[bench] {cname}-width FFN kernel: {us:.1f} us = {b / us / 1e3:.0f} GB/s = {b / us / 1e3 / HBM_PEAK_GBPS:.3f} of peak")
            sc.close()
            del sc
            torch.cuda.empty_cache()
        c4 = mi.get_config("C4")
        t0 = time.time()
        tr4, _, _ = mi.eamc_traces(c4, threads=16)
        d4 = m.ModelDesc.from_config(c4)
        e4 = m.Eamc(d4, c4.N, 4)
        e4.load(tr4)
        q4 = dev(mi.make_request(c4, 0, decode=1).prefill_eam.astype(np.int32))
        q4[0, :c4.k] += 1                       # the configuration has no prompt: one routed token
        for _ in range(3):
            m.eamc_match(e4, q4, stream=stream)
        m.profile_enable(256)
        for _ in range(30):
            m.eamc_match(e4, q4, stream=stream)
        torch.cuda.synchronize()
        dsm, psm = m.profile_samples("eamc_dot_kernel"), m.profile_samples("eamc_pick_kernel")
        m.profile_disable()
        b4 = c4.N * c4.L * c4.E * 4
        us4 = float(np.mean(dsm))
        shapes["eamc_match_C4"] = {
            "workload": f"C4 collection: {c4.N} traces x {c4.L} x {c4.E} int32 cells ({b4 / 1e6:.1f} MB), one query",
            "launches": len(dsm), "dot_kernel_avg_us": us4, "dot_kernel_median_us": float(np.median(dsm)),
            "pick_kernel_avg_us": float(np.mean(psm)), "alg_bytes": b4, "GBps": b4 / us4 / 1e3,
            "frac": b4 / us4 / 1e3 / HBM_PEAK_GBPS, "traces_per_s": c4.N / (us4 + float(np.mean(psm))) * 1e6}
        log(f"[bench] C4 match ({time.time() - t0:.0f}s to draw and load): dot kernel {us4:.1f} us = {b4 / us4 / 1e3:.0f} GB/s = "
            f"{b4 / us4 / 1e3 / HBM_PEAK_GBPS:.3f} of peak, pick {float(np.mean(psm)):.1f} us")
        e4.close()
        del tr4
        extra["other_shapes"] = shapes

    # ------------------------------------------------ optional: decode batches on this shape
    # (the default run on C2 carries a short form of it: B = 1, 4, 16)
    short_legs = args.config == "C2" and not args.no_shapes
    if args.batch_sweep or short_legs:
        big_cfg = cfg.scaled(cid=5, N=10000)
        tr10k, _, _ = mi.eamc_traces(big_cfg, threads=16)
        e10k = m.Eamc(desc, big_cfg.N, 4)
        e10k.load(tr10k)
        sweep = []
        for Bq in ((1, 2, 4, 8, 16) if args.batch_sweep else (1, 4, 16)):
            rq = [mi.make_request(cfg, 200 + b, decode=1) for b in range(Bq)]
            q = dev(np.stack([r.prefill_eam for r in rq]).astype(np.int32))
            xb = dev(np.stack([r.x[0, 0] for r in rq]))
            lg = dev(np.stack([r.bias[0] for r in rq]).astype(np.float32) + rng.standard_normal((Bq, E)).astype(np.float32))
            idx_b, w_b = m.moe_route_topk(lg, k, bool(cfg.renorm))
            distinct = len(set(idx_b.cpu().numpy().reshape(-1).tolist())) + cfg.n_shared
            for _ in range(5):
                m.eamc_match(e10k, q, stream=stream)
                m.expert_ffn_grouped(cache, 0, idx_b, w_b, xb, stream=stream)
            ev0.record(stream)
            for _ in range(50):
                m.eamc_match(e10k, q, stream=stream)
            ev1.record(stream)
            torch.cuda.synchronize()
            t_match = ev0.elapsed_time(ev1) / 50 * 1e3
            ev0.record(stream)
            for i in range(50):  # another layer's slots every call: the weights come from HBM, not from a cache
                m.expert_ffn_grouped(cache, i % L, idx_b, w_b, xb, stream=stream)
            ev1.record(stream)
            torch.cuda.synchronize()
            t_ffn = ev0.elapsed_time(ev1) / 50 * 1e3
            sweep.append({"B": Bq, "match_us": t_match, "match_alg_bytes": big_cfg.N * L * E * 4,
                          "distinct_experts": distinct, "ffn_us": t_ffn, "ffn_alg_bytes": distinct * cfg.expert_bytes,
                          "ffn_GBps": distinct * cfg.expert_bytes / t_ffn / 1e3})
            log(f"[bench] batch {Bq}: match {t_match:.1f} us, grouped FFN {t_ffn:.1f} us over {distinct} experts "
                f"= {distinct * cfg.expert_bytes / t_ffn / 1e3:.0f} GB/s")
        extra["batch_sweep"] = sweep
        e10k.close()

    # ------------------------------------------------ optional: the prefill iteration on this shape
    # (the default run on C2 carries a short form of it: 512 and 2,048 tokens)
    if (args.prefill or short_legs) and cfg.wdtype == "bf16" and H <= 4096:
        rows = []
        for n_tok in ((64, 128, 256, 512, 1024, 2048) if args.prefill else (512, 2048)):
            if n_tok > args.prefill_max:
                break
            rng = np.random.default_rng(n_tok)
            Xp = dev(mi.to_store(cfg, rng.standard_normal((n_tok, H)).astype(np.float32)))
            Yp = torch.empty((n_tok, H), dtype=torch.float32, device="cuda")
            eam_p = prefill.clone()
            for _ in range(2):
                _, pidx, _ = m.moe_prefill_layer(cache, eam_p, 0, routers[0], d_bias[0], Xp, Y=Yp, want_picks=True)
            torch.cuda.synchronize()
            reps = 10
            ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            ev0.record()
            for i in range(reps):
                m.moe_prefill_layer(cache, eam_p, i % L, routers[i % L], d_bias[i % L], Xp, Y=Yp)
            ev1.record()
            torch.cuda.synchronize()
            us = ev0.elapsed_time(ev1) / reps * 1e3
            distinct = len(np.unique(pidx.cpu().numpy())) + cfg.n_shared
            flops = 6.0 * H * cfg.I * n_tok * (k + cfg.n_shared)
            rows.append({"tokens": n_tok, "us_per_layer": us, "distinct_experts": distinct,
                         "weight_GBps": distinct * cfg.expert_bytes / us / 1e3, "TFLOPs": flops / us / 1e6,
                         "tokens_per_s": n_tok / us * 1e6})
            log(f"[bench] prefill {n_tok} tokens: {us:.0f} us per layer, {distinct} experts -> "
                f"{rows[-1]['weight_GBps']:.0f} GB/s of distinct weights, {rows[-1]['TFLOPs']:.1f} TFLOP/s")
        extra["prefill"] = rows

    # ------------------------------------------------ leg 4: offload replay (capped cache, PCIe misses)
    if not args.no_offload and cfg.S < L * E:
        host_bank = pinned(bank_slots)
        oc = m.Cache(desc, cfg.S, host_bank, None)
        for s in range(L * cfg.n_shared):
            t = oc.slot_tensor(cfg.S + s)
            t.copy_(d_shared[s % len(d_shared)].view(t.dtype))

        def offload_run(policy, depth, tokens, n_req=1):
            # n_req > 1: requests of different activation groups served back to back; the cache and
            # the policy's own history carry over, the request's EAM starts from its own prefill
            oc.reset(cfg.S)
            oc.set_policy(policy)
            oc.set_prefetch(depth)
            per, n_pf = [], 0
            for r in range(n_req):
                if r == 0:
                    rq_eam, rq_bias, rq_x = prefill, d_bias, d_x
                else:
                    rq = mi.make_request(cfg, r, decode=tokens)
                    rq_eam, rq_bias, rq_x = dev(rq.prefill_eam.astype(np.int32)), dev(rq.bias), dev(rq.x)
                d_eam.copy_(rq_eam)
                for i in range(tokens * L):
                    t, l = i // L, i % L
                    torch.cuda.synchronize()
                    a = time.perf_counter()
                    idx, best, n_miss = m.moe_decode_layer(oc, eamc, d_eam, l, routers[l], rq_bias[l], rq_x[t, l], y,
                                                           sync=True, stream=stream)
                    torch.cuda.synchronize()
                    per.append((time.perf_counter() - a, n_miss))
                    if depth:
                        n_pf += len(oc.last_prefetch())
            oc.sync()
            n_off = len(per)
            hit_steps = [t for t, nm in per if nm == 0]
            miss_steps = [(t, nm) for t, nm in per if nm > 0]
            tot_miss = sum(nm for _, nm in per)
            return {
                "policy": policy, "prefetch_depth": depth, "requests": n_req,
                "slots": cfg.S, "layer_steps": n_off, "hit_rate": 1.0 - tot_miss / (n_off * k),
                "prefetched_experts": n_pf,
                "us_per_step_blended": sum(t for t, _ in per) / n_off * 1e6,
                "us_per_step_all_hit": (sum(hit_steps) / len(hit_steps) * 1e6) if hit_steps else None,
                "all_hit_steps": len(hit_steps),
                "us_per_step_with_miss": (sum(t for t, _ in miss_steps) / len(miss_steps) * 1e6) if miss_steps else None,
                "host_link_GBps": (tot_miss * cfg.expert_bytes / sum(t for t, _ in miss_steps) / 1e9) if miss_steps else None,
            }

        extra["offload"] = offload_run("eam", 0, args.offload_tokens)
        extra["offload"]["note"] = "synchronous steps, each timed from the host; misses copied from pinned host memory"
        log(f"[bench] offload: hit rate {extra['offload']['hit_rate']:.3f}, "
            f"{extra['offload']['us_per_step_blended']:.0f} us/step blended")
        if args.policy_sweep:
            # the same request under the comparison eviction rules and with prefetching switched on
            rows = []
            for policy, depth in (("eam", 0), ("eam", 2), ("lru", 0), ("count", 0)):
                r = offload_run(policy, depth, args.policy_tokens, args.policy_requests)
                rows.append(r)
                log(f"[bench] policy {policy} prefetch {depth}: hit rate {r['hit_rate']:.3f}, "
                    f"{r['us_per_step_blended']:.0f} us/step, {r['prefetched_experts']} prefetched")
            extra["policy_sweep"] = rows
        oc.close()

    # ------------------------------------------------ leg 5: CPU oracle on a bounded sample
    cpu = None
    if not args.no_cpu:
        from oracle import moei_oracle as O
        try:
            from threadpoolctl import threadpool_info
            threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            threads = 1
        ref_eam = req.prefill_eam.astype(np.int64).copy()
        ref_cache = O.ExpertCache(L, E, L * E)
        h_routers = [mi.router_weights(cfg, l) for l in range(L)]

        def expert_of(fid):
            return split_expert(cfg, bank[fid % n_unique])

        def shared_of(layer):
            return [split_expert(cfg, shared[(layer * cfg.n_shared + s) % shared.shape[0]]) for s in range(cfg.n_shared)]

        n_cpu, spent = 0, 0.0
        budget = 15.0
        limit = args.cpu_steps if args.cpu_steps is not None else 10 ** 9
        while n_cpu < limit and (spent < budget or n_cpu < 2):
            l = n_cpu % L
            a = time.perf_counter()
            O.decode_layer(traces, ref_eam, ref_cache, l, h_routers[l], req.bias[l], req.x[n_cpu // L, l], expert_of,
                           shared_of, k, bool(cfg.renorm), EPS)
            spent += time.perf_counter() - a
            n_cpu += 1
        model = ""
        try:
            for line in open("/proc/cpuinfo"):
                if line.startswith("model name"):
                    model = line.split(":", 1)[1].strip()
                    break
        except OSError:
            pass
        cpu = {"value": spent / n_cpu * 1e6, "unit": "us per MoE-layer decode step", "cores": threads, "kind": "oracle",
               "sample": f"first {n_cpu} layer steps of the same request (all experts resident), {spent:.1f} s of CPU time",
               "host_cpus": os.cpu_count(), "cpu_model": model}
        log(f"[bench] oracle: {cpu['value'] / 1e3:.0f} ms per layer step on {threads} thread(s)")

        # the same steps as plain C loops (oracle/cpu_step.c: scalar, fp64 accumulation, OpenMP over traces
        # and over weight rows), on one core and on all of the cores this process may use
        from oracle import cpu_step as CS
        try:
            usable = len(os.sched_getaffinity(0))
        except AttributeError:
            usable = os.cpu_count() or 1
        n_all = max(1, min(usable, CS.threads_available()))
        triples = [tuple(np.ascontiguousarray(a) for a in split_expert(cfg, bank[u])) for u in range(n_unique)]
        sh_triples = [tuple(np.ascontiguousarray(a) for a in split_expert(cfg, shared[u])) for u in range(shared.shape[0])]
        tabs = [CS.pointer_table([triples[(l * E + e) % n_unique] for e in range(E)]) for l in range(L)]
        sh_tabs = [CS.pointer_table([sh_triples[(l * cfg.n_shared + s_) % len(sh_triples)] for s_ in range(cfg.n_shared)])
                   if cfg.n_shared else None for l in range(L)]
        all_resident = np.ones(L * E, dtype=np.uint8)
        c_rows = {}
        for nthr, budget_s in ((1, 8.0), (n_all, 5.0)):
            c_eam = req.prefill_eam.astype(np.int64).copy()
            n_c, spent_c = 0, 0.0
            while spent_c < budget_s or n_c < 2:
                l = n_c % L
                a = time.perf_counter()
                CS.decode_step(traces, c_eam, l, h_routers[l], req.bias[l], req.x[(n_c // L) % T_dec, l], tabs[l], sh_tabs[l],
                               H, I, k, cfg.renorm, EPS, all_resident, threads=nthr)
                spent_c += time.perf_counter() - a
                n_c += 1
            c_rows[nthr] = {"threads": nthr, "us_per_step": spent_c / n_c * 1e6, "layer_steps": n_c, "cpu_s": spent_c}
            log(f"[bench] C loops, {nthr} thread(s): {spent_c / n_c * 1e3:.1f} ms per layer step ({n_c} steps)")
        cpu["c_loops"] = {"kind": "plain C loops, fp64 accumulation, OpenMP over traces and weight rows (oracle/cpu_step.c)",
                          "one_core": c_rows[1], "all_cores": c_rows[n_all], "usable_cpus": usable,
                          "sample": "layer steps of the same request from its start, all experts resident"}

    out = {
        "metric": "us per MoE-layer decode step (EAMC traces scanned/s and expert GEMV HBM GB/s in `extra`)",
        "value": us_step, "unit": "us", "n_gpus": 1, "steps": K, "warmup": W,
        "steps_requested": K_req, "warmup_requested": W_req,
        "ms_per_step": us_step / 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16 weights, fp32 accumulate" if cfg.wdtype == "bf16" else "fp32", "data": "synthetic",
        "config": {"workload": f"{cfg.name}{slice_note}: {L} MoE layers x {E} experts top-{k} + {cfg.n_shared} shared, H={H}, I={I}, "
                               f"{cfg.wdtype}; EAMC {cfg.N} traces; batch 1, {T_dec} decode tokens; all experts resident "
                               f"in HBM ({S_res} slots, {n_unique} distinct weight sets repeated)",
                   "mode": mode, "us_per_step_without_graph": us_step_eager,
                   "timed": f"{tok_timed} decode tokens x {L} layer steps after {tok_warm} warm-up token(s)"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "kernels": kern,
        "extra": extra,
        "context": {"paper_tpot_ms_deepseek_v2_lite_a5000": 155, "paper_match_us_1k_cpu": 21, "paper_match_us_10k_cpu": 226},
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
