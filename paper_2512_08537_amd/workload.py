"""Runs a seeded case (synth.cases.Case) through the HIP library: context set-up, cache upload, one round.

Used by bench.py, the kernel benchmarks, smoke() and the GPU tests.  Nothing here computes a step of the method.
"""
from __future__ import annotations

import numpy as np

from synth.cases import Case


def make_ctx(case: Case, stream=None):
    from . import binding
    ctx = binding.Context(case.rc, case.W, stream=stream)
    load_caches(ctx, case)
    return ctx


def load_caches(ctx, case: Case):
    from . import binding
    for which, caches in ((binding.TARGET, case.cache_t), (binding.DRAFT, case.cache_d)):
        last, last_dev = None, None
        for l, (k, v) in enumerate(caches):
            if last is not None and k is last[0]:
                kd, vd = last_dev
            else:
                kd, vd = ctx.dev_store(k), ctx.dev_store(v)
            ctx.spec_kv_load(which, l, kd, vd)
            last, last_dev = (k, v), (kd, vd)
        ctx.spec_kv_reset(which, np.full(case.B, case.n_ctx, dtype=np.int32))
    ctx.sync()


def gpu_inputs(ctx, case: Case):
    return dict(pending=ctx.dev_f32(case.inp["pending"]), eps=ctx.dev_f32(case.inp["eps_draft"]),
                r=ctx.dev_f32(case.inp["r"]))


def to_np(o: dict) -> dict:
    out = {}
    for k, v in o.items():
        if v is None:
            continue
        out[k] = v.float().cpu().numpy() if v.dtype.is_floating_point else v.cpu().numpy()
    return out


def run_gpu_round(case: Case, tau: float, ctx=None):
    own = ctx is None
    ctx = ctx or make_ctx(case)
    g = gpu_inputs(ctx, case)
    o = ctx.spec_round(g["pending"], g["eps"], g["r"], tau)
    ctx.sync()
    out = to_np(o)
    from . import binding
    out["len_t"] = ctx.spec_kv_lengths(binding.TARGET, case.B)
    out["len_d"] = ctx.spec_kv_lengths(binding.DRAFT, case.B)
    if own:
        ctx.close()
    return out
