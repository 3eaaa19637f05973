#!/usr/bin/env python3
"""Per-kernel roofline measurements that the round benchmark cannot isolate.

  python -m paper_2512_08537_amd.kernel_bench entropy     # entropy pre-filter: config shapes + 2^20-row shape
  python -m paper_2512_08537_amd.kernel_bench narrow      # narrow-tile GEMM launches (time them with rocprofv3 --kernel-trace)
  python -m paper_2512_08537_amd.kernel_bench losses      # attention-entropy loss + gradients at training shapes
  python -m paper_2512_08537_amd.kernel_bench peaks       # probed peaks: streaming read GB/s, bf16 MFMA TFLOP/s
  python -m paper_2512_08537_amd.kernel_bench copy        # 256 MiB copy: calibration of the HBM traffic counters

Prints one JSON line per measurement: algorithmic bytes / HIP-event time on the library's stream.
"""
from __future__ import annotations

import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_HBM_GBS = 8000.0


def entropy():
    import torch
    from synth.cases import build_case
    from .workload import make_ctx
    case = build_case("ln-gelu-bf16", seed=0)
    ctx = make_ctx(case)
    # (B, K, L): configs[0..4] feature shapes, then the scaled shape that shows the asymptotic bandwidth
    shapes = [(1, 4, 256), (32, 8, 1024), (64, 8, 1280), (8, 8, 2048), (256, 8, 1280), (1 << 17, 8, 1280)]
    for (B, K, L) in shapes:
        g = torch.Generator(device="cuda").manual_seed(0)
        feat = (torch.randn((B, K, L), generator=g, device="cuda", dtype=torch.float32) * 0.25).to(torch.bfloat16)
        for _ in range(3):
            out = ctx.entropy_prefilter(feat, 2.14)
        ctx.sync()
        iters = 20 if B * K * L < (1 << 28) else 5
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(iters):
            out = ctx.entropy_prefilter(feat, 2.14)
        e1.record()
        ctx.sync()
        us = e0.elapsed_time(e1) * 1e3 / iters
        nbytes = B * K * L * 2 + B * K * 9
        gbs = nbytes / us / 1e3
        print(json.dumps({"kernel": "entropy_prefilter entry point, bf16 (small shapes: host-loop bound, see the kernel trace)", "rows": B * K, "len": L, "us_per_launch": round(us, 2),
                          "algorithmic_bytes": nbytes, "achieved_GBs": round(gbs, 1), "frac_hbm": round(gbs / PEAK_HBM_GBS, 4),
                          "n_surv": int(out[4].cpu()[0])}), flush=True)
    ctx.close()


def narrow():
    """Launches the narrow-tile GEMM at the shapes of a configs[1] round; kernel durations are read from a
    rocprofv3 kernel trace of this run (the host loop here is slower than the kernels)."""
    import torch
    from synth.cases import build_case
    from .workload import make_ctx
    case = build_case("ln-gelu-bf16", seed=0)
    ctx = make_ctx(case)
    dev = ctx.dev
    for M in (16, 32, 64, 288):
        for (K, N, epi) in [(1024, 1024, 0), (1024, 1024, 2), (1024, 1024, 3), (4096, 1024, 2), (1024, 4096, 0),
                            (1024, 3072, 0), (1280, 1280, 3), (2048, 2048, 0)]:
            W = (torch.randn((K, N), device=dev) * 0.02).to(torch.bfloat16)
            A = torch.randn((M, K), device=dev).to(torch.bfloat16)
            out = torch.zeros((M, N), device=dev, dtype=torch.bfloat16 if epi == 0 else torch.float32)
            gate = torch.ones((M, N), device=dev) if epi == 3 else None
            bias = torch.zeros(N, device=dev)
            for _ in range(12):
                ctx.spec_gemm_narrow(A, W, out, bias=bias, gate=gate, epi=epi)
            ctx.sync()
            print(json.dumps({"case": [M, K, N, epi]}), flush=True)
    ctx.close()


def copy():
    """A plain device copy of known size (256 MiB read + 256 MiB written per launch): the yardstick that the
    FETCH_SIZE / WRITE_SIZE counters of a rocprofv3 --pmc run are scaled by."""
    import torch
    n = 64 << 20
    a = torch.zeros(n, device="cuda", dtype=torch.float32)
    b = torch.ones(n, device="cuda", dtype=torch.float32)
    for _ in range(5):
        a.copy_(b)
    torch.cuda.synchronize()
    print(json.dumps({"kernel": "torch copy_", "bytes_read": n * 4, "bytes_written": n * 4, "launches": 5}), flush=True)


def peaks():
    """What the box sustains on the two roofs: a streaming read over several sizes, a register-only bf16 MFMA loop."""
    import torch
    from synth.cases import build_case
    from .workload import make_ctx
    ctx = make_ctx(build_case("ln-gelu-bf16", seed=0))
    for mib in (64, 256, 1024, 4096):
        buf = torch.zeros(mib << 18, device="cuda", dtype=torch.float32)
        torch.cuda.synchronize()
        ms, nbytes = ctx.spec_peak_probe(0, buf, reps=10)
        gbs = nbytes / (ms * 1e-3) / 1e9
        print(json.dumps({"probe": "streaming read", "MiB": mib, "us": round(ms * 1e3, 2), "GBs": round(gbs, 1),
                          "frac_of_published_hbm": round(gbs / PEAK_HBM_GBS, 4)}), flush=True)
        del buf
    for iters in (1024, 4096, 16384):
        ms, flop = ctx.spec_peak_probe(1, iters=iters, reps=5)
        tf = flop / (ms * 1e-3) / 1e12
        print(json.dumps({"probe": "bf16 mfma 32x32x16", "iters": iters, "us": round(ms * 1e3, 2), "TFLOPs": round(tf, 1),
                          "frac_of_published_bf16": round(tf / 2500.0, 4)}), flush=True)


def losses():
    """The attention-entropy loss with both gradients at the draft's training shapes (batch x heads x sequence x head
    dim); flops = score tiles (forward, and once more per gradient) + the two second products, causal half only."""
    import torch
    from synth.cases import build_case
    from .workload import make_ctx
    case = build_case("ln-gelu-bf16", seed=0)
    ctx = make_ctx(case)
    for (B, H, Hkv, R, dh) in [(32, 16, 16, 256, 64), (64, 20, 20, 256, 64), (8, 16, 16, 1024, 64), (8, 40, 8, 1024, 128)]:
        g = torch.Generator(device="cuda").manual_seed(0)
        q = torch.randn((B, H, R, dh), generator=g, device="cuda").to(torch.bfloat16)
        k = torch.randn((B, Hkv, R, dh), generator=g, device="cuda").to(torch.bfloat16)
        torch.cuda.synchronize()
        for _ in range(2):
            out = ctx.spec_entropy_loss(q, k)
        ctx.sync()
        ctx.spec_profile_enable(True)
        iters = 10
        for _ in range(iters):
            out = ctx.spec_entropy_loss(q, k)
        p = ctx.spec_profile_read(1)
        ctx.spec_profile_enable(False)
        us = p["ms"] / iters * 1e3
        tf = p["flops"] / (p["ms"] * 1e-3) / 1e12
        print(json.dumps({"kernel": "spec_entropy_loss (statistics, dq, dk passes + two transposes)", "B": B, "H": H, "H_kv": Hkv, "R": R,
                          "d_head": dh, "us_per_call": round(us, 1), "flops": p["flops"] / iters, "achieved_TFLOPs": round(tf, 1),
                          "frac_mfma": round(tf / 2500.0, 4), "loss": round(float(out[0].item()), 5)}), flush=True)
    ctx.close()


if __name__ == "__main__":
    what = sys.argv[1] if len(sys.argv) > 1 else "entropy"
    {"entropy": entropy, "narrow": narrow, "copy": copy, "losses": losses, "peaks": peaks}[what]()
