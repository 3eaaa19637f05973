"""Shared imports of the parity tests: seeded cases (synth.cases), the HIP library's side
(paper_2512_08537_amd.workload) and the CPU oracle's side (oracle.run_case).  The two sides only share `synth`."""
from __future__ import annotations

import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from synth.cases import Case, build_case                                         # noqa: E402,F401
from oracle.run_case import oracle_caches, run_oracle_round                      # noqa: E402,F401


def make_ctx(case, stream=None):
    from paper_2512_08537_amd import workload
    return workload.make_ctx(case, stream=stream)


def load_caches(ctx, case):
    from paper_2512_08537_amd import workload
    return workload.load_caches(ctx, case)


def gpu_inputs(ctx, case):
    from paper_2512_08537_amd import workload
    return workload.gpu_inputs(ctx, case)


def to_np(o):
    from paper_2512_08537_amd import workload
    return workload.to_np(o)


def run_gpu_round(case, tau, ctx=None):
    from paper_2512_08537_amd import workload
    return workload.run_gpu_round(case, tau, ctx=ctx)


def rel_inf(g, o):
    """||g - o||_inf / ||o||_inf per tensor (the floating-point bar of the parity tests)."""
    o = np.asarray(o, dtype=np.float64)
    den = np.abs(o).max()
    return float(np.abs(np.asarray(g, dtype=np.float64) - o).max() / (den if den > 0 else 1.0))
