"""Runs a seeded case (synth.cases.Case) through the CPU oracle: the counterpart of the HIP library's round on the
same inputs.  Test infrastructure, like everything under oracle/: only tests, the smoke check and the benchmark's
cpu_baseline leg call it."""
from __future__ import annotations

import numpy as np

from synth.cases import Case


def oracle_caches(case: Case, samples=None):
    from oracle import transformer as tf
    idx = list(range(case.B)) if samples is None else list(samples)
    tc, dc = tf.KVCache(case.rc.target, len(idx)), tf.KVCache(case.rc.draft, len(idx))
    for l, (k, v) in enumerate(case.cache_t):
        tc.load(l, k[idx], v[idx])
    for l, (k, v) in enumerate(case.cache_d):
        dc.load(l, k[idx], v[idx])
    return tc, dc


def run_oracle_round(case: Case, tau: float, samples=None):
    from oracle import round as rnd
    idx = list(range(case.B)) if samples is None else list(samples)
    tc, dc = oracle_caches(case, idx)
    out = rnd.spec_round(case.rc, case.W, tc, dc, case.inp["pending"][idx], case.inp["eps_draft"][:, idx],
                         case.inp["r"][idx], tau, len(idx))
    out["len_t"] = np.array([tc.length(b) for b in range(len(idx))])
    out["len_d"] = np.array([dc.length(b) for b in range(len(idx))])
    return out
