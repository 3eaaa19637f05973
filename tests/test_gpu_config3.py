"""BASELINE configs[3] at its own shape (text-to-image 14B class: 40 layers, d = 5120, 40 query / 8 KV heads of 128,
SwiGLU 13824, RMSNorm, RoPE; draft 4 layers d = 2048 with the 2048 -> 5120 up-projection; flow head 12 x 1536, 4 steps;
B = 8, K = 8, 768 cached tokens) against the CPU oracle on one sample.  The oracle streams the 11 B parameters layer by
layer (they are re-drawn from their sub-seeds when read, gen.LazyWeights), the HIP library holds them all."""
import copy

import numpy as np
import pytest

from synth import gen
from tests.harness import build_case, make_ctx, rel_inf, gpu_inputs, to_np
from tests.test_gpu_round import teacher_forced_round

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]

SAMPLE = 5


@pytest.fixture(scope="module")
def cfg3():
    import time
    t0 = time.time()
    case = build_case(3, seed=0, affine=False, lazy=True)
    ctx = make_ctx(case)
    print(f"[configs[3]] context built in {time.time() - t0:.0f} s", flush=True)
    # the oracle's view of the same tensors: float64, a 16 GB window that the forward walks through
    ocase = copy.copy(case)
    ocase.W = case.W.view(as_f64=True, budget_bytes=16 << 30, readahead=6)
    yield case, ocase, ctx
    ctx.close()


def test_config3_round_teacher_forced_on_one_sample(cfg3):
    """One whole round of sample 5 through the oracle (8 draft steps with the 4-step head, the 9-row verify forward
    through all 40 layers, the head on 9 rows, the ratio test), then the library at B = 8 (72 verify rows, the launch
    configuration bench.py times) with that sample teacher-forced: flat bars on every step and row."""
    import time
    from oracle.run_case import run_oracle_round
    case, ocase, ctx = cfg3
    t0 = time.time()
    o = run_oracle_round(ocase, tau=-1.0, samples=[SAMPLE])
    print(f"[configs[3]] oracle round of one sample: {time.time() - t0:.0f} s", flush=True)
    free = teacher_forced_round(case, ctx, o, [SAMPLE])
    assert abs(float(free["H"][SAMPLE, 0]) - float(o["H"][0, 0])) <= 1e-3
    assert rel_inf(free["mu_q"][SAMPLE, 0], o["mu_q"][0, 0]) < 2e-2
    assert rel_inf(free["mu_p"][SAMPLE, 0], o["mu_p"][0, 0]) < 2e-2
    assert np.isfinite(free["mu_p"]).all() and np.isfinite(free["log_ratio"]).all()
    # the draft's features reach the head through the 2048 -> 5120 up-projection: its decode on the oracle's own
    # features (12 blocks x 1536, 4 steps, d_cond 5120), row by row
    z = np.stack(o["z_q"][0])                              # [K, 5120]
    eps = case.inp["eps_draft"][:, SAMPLE, :z.shape[0]]    # [S+1, K, D]
    mu, x = ctx.diffhead_decode(ctx.dev_store(gen.bf16_round(z.astype(np.float32))), ctx.dev_f32(eps))
    ctx.sync()
    e = rel_inf(mu.cpu().numpy(), o["mu_q"][0, :z.shape[0]])
    print(f"[configs[3]] diffhead_decode on the oracle's draft features: {e:.2e}")
    assert e < 2e-2


def test_config3_forward_of_both_models_on_one_sample(cfg3):
    """spec_forward at the configuration's shapes: the target over ragged rows (9 for the sampled sample) and the
    draft including its up-projection, features and the shallow stream, sample 5 against the oracle."""
    from oracle import transformer as tf
    from oracle.run_case import oracle_caches
    from paper_2512_08537_amd import binding
    case, ocase, ctx = cfg3
    rc, B, D = case.rc, case.B, case.rc.target.d_latent
    lens = np.full(B, case.n_ctx, dtype=np.int32)
    rng = np.random.default_rng(11)
    n_q = rng.integers(1, rc.K + 2, size=B)
    n_q[SAMPLE] = rc.K + 1
    xs = [gen.bf16_round(rng.normal(size=(n, D)).astype(np.float32)) for n in n_q]
    tc, dc = oracle_caches(ocase, [SAMPLE])
    for which, cfg, prefix, cache in ((binding.TARGET, rc.target, "target", tc), (binding.DRAFT, rc.draft, "draft", dc)):
        ctx.spec_kv_reset(which, lens)
        z, sh, _ = ctx.spec_forward(which, ctx.dev_f32(np.concatenate(xs)), n_q, commit=False, want_shallow=True)
        ctx.sync()
        zo, sho, _ = tf.forward_sample(cfg, ocase.W, prefix, cache, 0, xs[SAMPLE], commit=False, shallow_layer=rc.entropy_layer)
        r0 = int(n_q[:SAMPLE].sum())
        ez = rel_inf(z.float().cpu().numpy()[r0:r0 + n_q[SAMPLE]], zo)
        es = rel_inf(sh.cpu().numpy()[r0:r0 + n_q[SAMPLE]], sho)
        print(f"[configs[3]] {prefix}: z {ez:.2e} shallow {es:.2e}")
        assert zo.shape[1] == 5120
        assert ez < 2e-2 and es < 2e-2
