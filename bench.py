#!/usr/bin/env python3
"""Benchmark of the speculative-round hot path on one MI355X.

One step = one whole round (K draft steps with the entropy early stop, the target's verify forward, the head on every
verified row, the accept test, cache commit) over one batch of synthetic, seeded input.  The headline workload is
BASELINE configs[3], the largest configuration that fits one GPU (11 B parameters, 72 verify rows); configs[1] and
configs[2] are measured in the same run and carried as sub-objects.  Prints ONE JSON line.

  python bench.py --gpus 1 --steps 20 --warmup 5 [--config 3] [--also 1,2] [--no-cpu]
  python bench.py --config 4          # adds the pre-filter sweep (0 / 25 / 50 / 75 / 100 % of the drafts filtered)
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0      # MI355X dense bf16 MFMA
PEAK_FP32_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0
CLASSES = ("gemm", "attention", "entropy", "other", "gemm_narrow")     # spec_profile_read's kernel classes


def hbm_traffic_per_launch(config, kernel_class):
    """HBM bytes per launch of a GEMM kernel class ("gemm": the streaming kernels, "gemm_narrow") from the committed
    rocprofv3 --pmc summary of this benchmark (FETCH_SIZE and WRITE_SIZE, scaled by a plain copy kernel).  The summary
    names the kernel sources it was measured on (`sources_sha16`); None when no summary covers the configuration or the
    sources have changed since."""
    from paper_2512_08537_amd.build import sources_hash
    path = os.path.join(ROOT, "profiles", f"gemm_cfg{config}_hbm_traffic.txt")
    val, sha = None, None
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(f"traffic_bytes_per_launch[{kernel_class}]:"):
                    val = int(line.split(":")[1])
                if line.startswith("sources_sha16:"):
                    sha = line.split(":")[1].strip()
    except OSError:
        return None
    return val if sha == sources_hash() else None


def measure(cfg_idx, args, headline):
    """Builds configs[cfg_idx], times the round, and (headline) everything else the line carries."""
    import torch
    from paper_2512_08537_amd import binding
    from synth.cases import build_case
    from paper_2512_08537_amd.workload import make_ctx, gpu_inputs

    t0 = time.time()
    shared = cfg_idx == 4                              # 44 GB of distinct synthetic cache would not fit the host
    # deep_gain: output projections of the target layers the draft lacks are drawn 50x smaller, so the truncated
    # draft predicts the target's feature about as well as a trained draft (acceptance ~0.7/token).  configs[3]'s
    # draft is a model of its own (2048 wide): nothing to damp, its drafts are not accepted (see config.value_counts).
    deep_gain = args.deep_gain if args.deep_gain is not None else (1.0 if cfg_idx == 3 else 0.02)
    # (configs[3]: 11 B parameters are drawn tensor by tensor while they are uploaded, not held on the host)
    case = build_case(cfg_idx, seed=args.seed, affine=False, cache_layers_shared=shared, deep_gain=deep_gain,
                      lazy=cfg_idx == 3)
    rc, B, K = case.rc, case.B, case.rc.K
    # a stream of its own, so that rounds can be captured into a HIP graph (--no-graph: the default stream)
    ctx = make_ctx(case, stream=None if args.no_graph else torch.cuda.Stream())
    gi = gpu_inputs(ctx, case)
    out = ctx._round_bufs(B)
    lens_dev = ctx.dev_i32(np.full(B, case.n_ctx, dtype=np.int32))
    print(f"[bench] case {rc.name} built in {time.time() - t0:.1f}s", file=sys.stderr, flush=True)

    # threshold from a calibration round's entropies, the paper's rule tau = 0.3 mean - 0.1 std
    cal = ctx.spec_round(gi["pending"], gi["eps"], gi["r"], -1.0, out=out)
    ctx.sync()
    Hc = cal["H"].cpu().numpy().copy()
    tau = binding.entropy_threshold(float(Hc.mean()), float(Hc.std()))

    def reset():                                        # cache lengths back to n_ctx, from device memory: no host sync
        ctx.spec_kv_restore(binding.TARGET, lens_dev, case.n_ctx)
        ctx.spec_kv_restore(binding.DRAFT, lens_dev, case.n_ctx)

    def step(t=None):
        reset()
        ctx.spec_round(gi["pending"], gi["eps"], gi["r"], tau if t is None else t, out=out)

    def timed(t=None, steps=None, warmup=None):
        steps, warmup = steps or args.steps, args.warmup if warmup is None else warmup
        for _ in range(warmup):
            step(t)
        ctx.sync()
        t1 = time.perf_counter()
        for _ in range(steps):
            step(t)
        ctx.sync()
        return (time.perf_counter() - t1) / steps * 1e3

    def graphs(on):
        if not args.no_graph:
            ctx.spec_graph_enable(on)

    # kernel-by-kernel launches first (reported beside the headline), then the library's graph replay of the same
    # round: identical kernels and arguments, recorded on the second call and replayed afterwards.  The headline is the
    # replay (what a serving loop would run); both are in the line.
    ms_eager = timed()
    ms, ms_graph = ms_eager, None
    if not args.no_graph:
        graphs(True)
        step(); step()                                   # first sighting of the arguments, then the recording call
        ms_graph = timed()
        ms = ms_graph

    n_keep = out["n_keep"].cpu().numpy().copy()
    n_acc = out["n_accept"].cpu().numpy().copy()
    accepted = float(n_acc.sum())
    verified = float(n_keep.sum())
    t, d = rc.target, rc.draft
    res = {
        "workload": f"BASELINE configs[{cfg_idx}] ({rc.name}): B={B}, K={K}, n_ctx={case.n_ctx}, target L={t.n_layers} "
                    f"d={t.d_model}, draft L={d.n_layers} d={d.d_model}, head {rc.head.n_blocks}x{rc.head.width} "
                    f"S={rc.head.n_steps}; weights N(0, 0.02) (models wider than 2048: N(0, 0.64/sqrt(d))), "
                    + ("draft = first layers of the target, " if case.shared_layers else "draft = a model of its own, ")
                    + f"deep-layer output projections x{deep_gain}",
        "ms_per_step": round(ms, 4),
        "launch": "kernel by kernel" if ms_graph is None else "HIP graph replay of the round (spec_graph_enable)",
        "ms_per_step_kernel_by_kernel": round(ms_eager, 4),
        "ms_per_step_graph_replay": None if ms_graph is None else round(ms_graph, 4),
        "tau_ent": round(tau, 4), "accepted_per_round": accepted, "verified_per_round": verified,
        "acceptance_rate": round(accepted / max(verified, 1.0), 4),
        "prefilter_rate": round(1.0 - verified / (B * K), 4),
        "value_counts": "accepted drafts plus the one token every round always yields (Alg. 1 Step 5 / the closing "
                        "token): tokens committed to the sequence per second",
        "committed_tokens_per_s": round((accepted + B) / (ms * 1e-3), 1),
        "accepted_drafts_per_s": round(accepted / (ms * 1e-3), 1),
        "verified_tokens_per_s": round(verified / (ms * 1e-3), 1),
    }

    # per-kernel-class time with HIP events on the library's stream, over `steps` more rounds
    graphs(False)
    ctx.spec_profile_enable(True)
    for _ in range(args.steps):
        step()
    prof = {name: ctx.spec_profile_read(i) for i, name in enumerate(CLASSES)}
    ctx.spec_profile_enable(False)
    # the dominant kernel class: the streaming GEMM kernels (every GEMM above a few hundred rows; at configs[3] the
    # weight stream of the 72-row verify stage) or the narrow-tile GEMM kernel (draft steps, head decodes, and at
    # configs[1] nearly every GEMM), whichever the round spends more time in; the other one is in `kernels`
    # An event pair around every launch adds the dispatch gap to each bracket: the brackets of a round sum to more
    # than the round takes without them.  That excess, spread evenly over the launches, is taken off every bracket,
    # which brings the figure to the kernel durations a rocprofv3 trace shows (profiles/).
    all_ms = sum(v["ms"] for v in prof.values())
    all_launches = sum(v["launches"] for v in prof.values())
    overhead_us = max(0.0, all_ms / args.steps - ms_eager) / max(all_launches / args.steps, 1) * 1e3
    net_ms = {k: max(v["ms"] - overhead_us * 1e-3 * v["launches"], 0.25 * v["ms"]) for k, v in prof.items()}
    dom = "gemm" if net_ms["gemm"] >= net_ms["gemm_narrow"] else "gemm_narrow"
    g = prof[dom]
    g_raw_us = g["ms"] / max(g["launches"], 1) * 1e3
    g_avg_us = max(g_raw_us - overhead_us, 0.25 * g_raw_us)
    g_ms = g_avg_us * g["launches"] * 1e-3
    g_tflops = g["flops"] / (g_ms * 1e-3) / 1e12 if g_ms > 0 else 0.0
    peak = PEAK_BF16_TFLOPS if rc.dtype == 1 else PEAK_FP32_TFLOPS
    g_gbs = g["bytes"] / (g_ms * 1e-3) / 1e9 if g_ms > 0 else 0.0
    # which roof the GEMMs of this workload sit under: flops per algorithmic byte against the ridge peak_flops / peak_bytes
    # (a few tens to a few hundred rows per weight matrix: the weights are streamed once, the roof is HBM)
    intensity = g["flops"] / max(g["bytes"], 1.0)
    hbm_bound = intensity < peak * 1e12 / (PEAK_HBM_GBS * 1e9)
    roofline = {"bound": "hbm" if hbm_bound else ("mfma" if rc.dtype == 1 else "alu"),
                "kernel": ("streaming GEMM kernels (gemm_bf16_kernel, gemm_bf16_res_kernel: all instances)" if dom == "gemm"
                           else "narrow-tile GEMM kernel (gemm_narrow_kernel: all instances)"),
                "share_of_round_kernel_time": round(net_ms[dom] / max(sum(net_ms.values()), 1e-9), 4),
                "achieved": round(g_gbs, 1) if hbm_bound else round(g_tflops, 3),
                "peak": PEAK_HBM_GBS if hbm_bound else peak, "unit": "GB/s" if hbm_bound else "TFLOP/s",
                "frac": round(g_gbs / PEAK_HBM_GBS, 5) if hbm_bound else round(g_tflops / peak, 5),
                "traffic": hbm_traffic_per_launch(cfg_idx, dom), "launches_per_step": g["launches"] / args.steps,
                "avg_launch_us": round(g_avg_us, 3), "avg_launch_us_with_event_pair": round(g_raw_us, 3),
                "event_pair_overhead_us": round(overhead_us, 3),
                "flops_per_launch": g["flops"] / max(g["launches"], 1),
                "algorithmic_bytes_per_launch": g["bytes"] / max(g["launches"], 1),
                "flops_per_byte": round(intensity, 1), "achieved_TFLOPs": round(g_tflops, 3),
                "frac_mfma": round(g_tflops / peak, 5), "achieved_GBs": round(g_gbs, 1)}
    # attention: algorithmic K/V bytes of the verify forward + the K draft steps
    esz = 2 if rc.dtype == 1 else 4
    att_bytes = 0.0
    for (m, L, rows_list) in ((t, t.n_layers, [K + 1]), (d, d.n_layers, [1] * K)):
        for i, nq in enumerate(rows_list):
            ctx_len = case.n_ctx + (i if len(rows_list) > 1 else 0)
            att_bytes += L * B * (2 * (ctx_len + nq) * m.n_kv_heads * m.d_head * esz + 2 * nq * m.n_heads * m.d_head * esz)
    a = prof["attention"]
    a_ms = max(a["ms"] - overhead_us * 1e-3 * a["launches"], 0.25 * a["ms"])      # event-pair excess taken off, as above
    att_gbs = att_bytes * args.steps / (a_ms * 1e-3) / 1e9 if a_ms > 0 else 0.0
    kernels = {k: {"ms_per_step": round(max(v["ms"] - overhead_us * 1e-3 * v["launches"], 0.25 * v["ms"]) / args.steps, 4),
                   "ms_per_step_with_event_pairs": round(v["ms"] / args.steps, 4),
                   "launches_per_step": v["launches"] / args.steps}
               for k, v in prof.items()}
    kernels["attention"]["achieved_GBs"] = round(att_gbs, 1)
    kernels["attention"]["frac_hbm"] = round(att_gbs / PEAK_HBM_GBS, 5)
    for name in ("gemm", "gemm_narrow"):
        v = prof[name]
        ms_c = max(v["ms"] - overhead_us * 1e-3 * v["launches"], 0.25 * v["ms"])
        if ms_c > 0:
            kernels[name]["achieved_GBs"] = round(v["bytes"] / (ms_c * 1e-3) / 1e9, 1)
            kernels[name]["achieved_TFLOPs"] = round(v["flops"] / (ms_c * 1e-3) / 1e12, 2)
            kernels[name]["avg_launch_us"] = round(ms_c / max(v["launches"], 1) * 1e3, 3)
    if net_ms["attention"] > net_ms[dom]:
        # the cached attention is the round's largest kernel class (long contexts, large batches): the roofline object
        # is its K/V stream, and the GEMM classes' figures stay in `kernels`
        roofline = {"bound": "hbm", "kernel": "cached attention (attn_bf16_kernel incl. the merge launch of split keys)",
                    "share_of_round_kernel_time": round(net_ms["attention"] / max(sum(net_ms.values()), 1e-9), 4),
                    "achieved": round(att_gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s", "frac": round(att_gbs / PEAK_HBM_GBS, 5),
                    "traffic": None, "launches_per_step": a["launches"] / args.steps,
                    "avg_launch_us": round(a_ms / max(a["launches"], 1) * 1e3, 3),
                    "avg_launch_us_with_event_pair": round(a["ms"] / max(a["launches"], 1) * 1e3, 3),
                    "event_pair_overhead_us": round(overhead_us, 3),
                    "algorithmic_bytes_per_launch": att_bytes * args.steps / max(a["launches"], 1), "achieved_GBs": round(att_gbs, 1)}
        hbm_bound, g_gbs = True, att_gbs
    res["roofline"], res["kernels"] = roofline, kernels
    if not headline:
        ctx.close()
        return res

    # what this machine sustains on the two roofs (a 1 GiB streaming read, a register-only bf16 MFMA loop): `frac` stays
    # against the published peaks, the probed ones are reported beside it
    probe_buf = torch.empty(1 << 28, device="cuda", dtype=torch.float32)
    probe_buf.zero_()
    torch.cuda.synchronize()
    rd_ms, rd_bytes = ctx.spec_peak_probe(0, probe_buf, reps=10)
    mf_ms, mf_flop = ctx.spec_peak_probe(1, iters=4096, reps=5)
    del probe_buf
    probed_gbs = rd_bytes / (rd_ms * 1e-3) / 1e9
    probed_tflops = mf_flop / (mf_ms * 1e-3) / 1e12
    roofline["probed_peak"] = {"hbm_read_GBs": round(probed_gbs, 1), "mfma_bf16_TFLOPs": round(probed_tflops, 1)}
    if hbm_bound:
        roofline["frac_of_probed"] = round(g_gbs / probed_gbs, 5)
    elif rc.dtype == 1:
        roofline["frac_of_probed"] = round(g_tflops / probed_tflops, 5)
    kernels["attention"]["frac_hbm_probed"] = round(att_gbs / probed_gbs, 5)

    # configs[4]: the pre-filter stress as a round measurement.  tau is chosen per target fraction on the calibration
    # round's entropies (a sample's drafts are cut at its first step with H < tau, so the survivor count of a tau is
    # known before the round is run); per fraction: round time, time per kernel class, rows the verify stage and the
    # head see.  What the round saves is the work on filtered rows, so its time should fall linearly in the survivors.
    if cfg_idx == 4 or args.sweep:
        cands = np.unique(np.concatenate([[-1.0], np.sort(Hc.reshape(-1)) + 1e-7, [1e9]]))

        def keeps(tv):
            below = Hc < tv
            first = np.where(below.any(axis=1), below.argmax(axis=1), K)
            return int(first.sum())

        sweep = []
        for frac in (0.0, 0.25, 0.5, 0.75, 1.0):
            want = (1.0 - frac) * B * K
            lo, hi = 0, len(cands) - 1                      # keeps() falls as tau rises: bisect for the first tau at or below
            while lo < hi:
                mid = (lo + hi) // 2
                if keeps(cands[mid]) <= want:
                    hi = mid
                else:
                    lo = mid + 1
            tv = float(cands[lo])
            ms_f = timed(tv, steps=max(3, args.steps // 4), warmup=1)
            nk = out["n_keep"].cpu().numpy()
            ctx.spec_profile_enable(True)
            step(tv)
            pf = {name: ctx.spec_profile_read(i) for i, name in enumerate(CLASSES)}
            ctx.spec_profile_enable(False)
            sweep.append({"target_filtered": frac, "tau": round(tv, 5), "filtered": round(1.0 - float(nk.sum()) / (B * K), 4),
                          "surviving_drafts": int(nk.sum()), "verify_rows": int(nk.sum()) + B,
                          "samples_with_no_survivor": int((nk == 0).sum()), "ragged": bool(nk.min() != nk.max()),
                          "ms_per_round": round(ms_f, 4),
                          "ms_by_class_with_event_pairs": {k: round(v["ms"], 3) for k, v in pf.items()}})
        t0_, t1_ = sweep[0]["ms_per_round"], sweep[-1]["ms_per_round"]
        r0_, r1_ = sweep[0]["verify_rows"], sweep[-1]["verify_rows"]
        for srow in sweep:                                  # the straight line through the two ends, in rows
            lin = t1_ + (t0_ - t1_) * (srow["verify_rows"] - r1_) / max(r0_ - r1_, 1)
            srow["ms_linear_in_rows"] = round(lin, 4)
        res["prefilter_sweep"] = {"rows": sweep, "launch": "kernel by kernel",
                                  "max_dev_from_linear": round(max(abs(x["ms_per_round"] - x["ms_linear_in_rows"]) / t0_
                                                                   for x in sweep), 4)}

    # Steps 1-5 over several rounds without a host synchronisation (spec_generate): tokens per second including the
    # closing token of every round; as many rounds as the cache capacity bound allows from n_ctx, at most 16
    gen_stats = None
    R = min(16, (rc.max_ctx - case.n_ctx) // (K + 1))
    if rc.target.pos == 0 and rc.target.max_pos:
        R = min(R, (rc.target.max_pos - case.n_ctx) // (K + 1))
    if R >= 1 and not args.no_generate:
        J, D, S = 16, rc.target.d_latent, rc.head.n_steps
        gt = torch.Generator(device=ctx.dev).manual_seed(args.seed)
        g_eps = torch.randn((R, S + 1, B, K + 1, D), generator=gt, device=ctx.dev)
        g_r = torch.rand((R, B, K), generator=gt, device=ctx.dev)
        g_er = torch.randn((R, B, J, D), generator=gt, device=ctx.dev)
        g_ur = torch.rand((R, B, J), generator=gt, device=ctx.dev)
        torch.cuda.synchronize()                         # (torch filled these on its own stream)
        reps = max(1, min(5, args.steps))

        def gen_timed():
            go = None
            for i in range(reps + 2):                        # two untimed calls (with replay on: the recording ones)
                if i == 2:
                    ctx.sync()
                    tg0 = time.perf_counter()
                reset()
                go = ctx.spec_generate(gi["pending"], g_eps, g_r, g_er, g_ur, tau, out=go)
            ctx.sync()
            return (time.perf_counter() - tg0) / reps, go

        graphs(False)
        tg_eager, go = gen_timed()
        tg, tg_graph = tg_eager, None
        if not args.no_graph:
            graphs(True)
            tg_graph, go = gen_timed()
            tg = tg_graph
        n_tok = float(go["n_tokens"].sum().item())
        gen_stats = {"rounds": R, "ms_per_round": round(tg / R * 1e3, 4), "tokens": n_tok,
                     "tokens_per_s": round(n_tok / tg, 1), "resample_tries_mean":
                     round(float(go["tries"].float().sum().item()) / max(1.0, float((go["tries"] > 0).sum().item())), 2),
                     "ms_per_round_kernel_by_kernel": round(tg_eager / R * 1e3, 4),
                     "ms_per_round_graph_replay": None if tg_graph is None else round(tg_graph / R * 1e3, 4)}

    # Prefill (the next row after the round itself): both caches rebuilt from a prefix of n_ctx known tokens per sample
    # (a class token and latents), timed on the stream; GEMM and attention time of the target's prefill from HIP events
    pf_stats = None
    if not args.no_generate:
        npf = np.full(B, case.n_ctx, dtype=np.int32)
        gp = torch.Generator(device=ctx.dev).manual_seed(args.seed + 1)
        xpf = torch.randn((B, case.n_ctx, rc.target.d_latent), generator=gp, device=ctx.dev)
        ids = None
        if rc.target.n_cond_ids > 0:
            ids = torch.randint(0, rc.target.n_cond_ids, (B,), generator=gp, device=ctx.dev, dtype=torch.int32)
        torch.cuda.synchronize()
        pf_ms = {}
        for which, name in ((binding.TARGET, "target"), (binding.DRAFT, "draft")):
            reps = 3
            for i in range(reps + 1):
                if i == 1:
                    ctx.sync()
                    tp0 = time.perf_counter()
                ctx.spec_kv_reset(which, None)
                ctx.spec_prefill(which, xpf, npf, first_id=ids, want_z=False)
            ctx.sync()
            pf_ms[name] = (time.perf_counter() - tp0) / reps * 1e3
        ctx.spec_profile_enable(True)
        ctx.spec_kv_reset(binding.TARGET, None)
        ctx.spec_prefill(binding.TARGET, xpf, npf, first_id=ids, want_z=False)
        pg, pa = ctx.spec_profile_read(0), ctx.spec_profile_read(1)
        ctx.spec_profile_enable(False)
        ntok = float(B * case.n_ctx)
        pf_tflops = pg["flops"] / (pg["ms"] * 1e-3) / 1e12 if pg["ms"] > 0 else 0.0
        pf_stats = {"tokens": ntok, "ms_target": round(pf_ms["target"], 3), "ms_draft": round(pf_ms["draft"], 3),
                    "tokens_per_s_target": round(ntok / (pf_ms["target"] * 1e-3), 1),
                    "gemm": {"ms": round(pg["ms"], 3), "launches": pg["launches"], "achieved_TFLOPs": round(pf_tflops, 1),
                             "frac_mfma": round(pf_tflops / peak, 5)},
                    "attention_ms": round(pa["ms"], 3)}
    res["generate"], res["prefill"] = gen_stats, pf_stats

    cpu = None
    if not args.no_cpu:
        cores = len(os.sched_getaffinity(0))
        n_cpu = min(args.cpu_samples if args.cpu_samples else (1 if cfg_idx == 3 else 8), B)
        idx = sorted(set(np.linspace(0, B - 1, n_cpu).astype(int).tolist()))
        from oracle.run_case import run_oracle_round      # the oracle: this leg only
        import copy
        ocase = case
        if cfg_idx == 3:                                   # the oracle walks the 11 B parameters through a 16 GB window
            ocase = copy.copy(case)
            ocase.W = case.W.view(as_f64=True, budget_bytes=16 << 30, readahead=6)
        tc0 = time.perf_counter()
        o = run_oracle_round(ocase, tau, samples=idx)
        tcpu = time.perf_counter() - tc0
        o_tok = float(o["n_accept"].sum()) + len(idx)
        cpu = {"value": round(o_tok / tcpu, 4), "unit": "tokens/s", "cores": cores,
               "kind": "oracle", "sample": f"samples {idx} of {B} (one full round each: {K} draft steps + verify of "
               f"n_keep+1 rows), numpy fp64, {tcpu:.1f}s; value counts accepted drafts plus one token per sample, as the headline",
               "verified_tokens_per_s": round(float(o["n_keep"].sum()) / tcpu, 4),
               "n_accept_gpu": n_acc[idx].tolist(), "n_accept_oracle": np.asarray(o["n_accept"]).tolist(),
               "n_keep_gpu": n_keep[idx].tolist(), "n_keep_oracle": np.asarray(o["n_keep"]).tolist(),
               "n_accept_agree": int((n_acc[idx] == np.asarray(o["n_accept"])).sum()), "n_compared": len(idx)}
    res["cpu_baseline"] = cpu
    ctx.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=3, help="BASELINE config index (0..4) of the headline workload")
    ap.add_argument("--also", type=str, default=None, help="further configs measured in the same run and carried as "
                    "sub-objects (default: 1,2 beside configs[3], none otherwise)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle baseline")
    ap.add_argument("--no-generate", action="store_true", help="skip the multi-round generation and prefill figures "
                    "(counter runs: fewer dispatches to collect)")
    ap.add_argument("--no-graph", action="store_true", help="time kernel-by-kernel launches instead of graph replays")
    ap.add_argument("--sweep", action="store_true", help="the pre-filter sweep of configs[4] on the chosen config")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--deep-gain", type=float, default=None)
    ap.add_argument("--cpu-samples", type=int, default=0)
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives are part of it); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    also = args.also if args.also is not None else ("1,2" if args.config == 3 else "")
    also = [int(x) for x in also.split(",") if x.strip() != ""]

    head = measure(args.config, args, headline=True)
    others = {}
    for c in also:
        if c != args.config:
            others[f"configs[{c}]"] = measure(c, args, headline=False)

    line = {
        "metric": "accepted latent tokens/sec per GPU", "value": head["committed_tokens_per_s"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": head["ms_per_step"],
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if args.config != 0 else "f32", "data": "synthetic",
        "config": {k: head[k] for k in ("workload", "launch", "ms_per_step_kernel_by_kernel", "ms_per_step_graph_replay",
                                        "tau_ent", "accepted_per_round", "verified_per_round", "acceptance_rate",
                                        "prefilter_rate", "value_counts", "committed_tokens_per_s", "accepted_drafts_per_s",
                                        "verified_tokens_per_s")},
        "roofline": head["roofline"], "cpu_baseline": head["cpu_baseline"], "kernels": head["kernels"],
        "generate": head["generate"], "prefill": head["prefill"],
    }
    if "prefilter_sweep" in head:
        line["prefilter_sweep"] = head["prefilter_sweep"]
    if others:
        line["other_configs"] = others
    print(json.dumps(line))


if __name__ == "__main__":
    main()
