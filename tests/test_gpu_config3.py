"""BASELINE configs[3] at its own shape (text-to-image 14B class: 40 layers, d = 5120, 40 query / 8 KV heads of 128,
SwiGLU 13824, RMSNorm, RoPE; draft 4 layers d = 2048 with the 2048 -> 5120 up-projection; flow head 12 x 1536, 4 steps;
B = 8, K = 8, 768 cached tokens) against the CPU oracle on one sample, with the weights of the benchmark's recipe for this
configuration (N(0, (0.64 / sqrt(5120))^2) for the 5120-wide target: with N(0, 0.02^2) a 40-layer stack of that width
amplifies rounding errors until no bf16 forward can hold 2e-2 -- a CPU emulation of the bf16 rounding points alone is
off by 5.5 %).  The oracle streams the 11 B parameters layer by layer (they are re-drawn from their sub-seeds when read,
gen.LazyWeights), the HIP library holds them all."""
import copy

import numpy as np
import pytest

from synth import gen
from tests.harness import build_case, make_ctx, rel_inf, gpu_inputs, to_np
from tests.test_gpu_round import teacher_forced_round, rel_rms

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]

SAMPLE = 5
# What comes out of the 40-layer, 5120-wide target is held to 4e-2, not to the 2e-2 of every other tensor and
# configuration: 2e-2 is where bf16 itself puts this forward.  A float64 forward of this very model whose only change is
# rounding to bf16 where any bf16 matrix-core path has to (the inputs of the six products of a layer and the
# probabilities) differs from the float64 forward by 1.8-2.5 % (per row 1.2-2.5 %, max norm and rms norm alike; measured on
# the CPU for weight scales 0.0045 ... 0.0089; 5.5 % at 0.02): about 0.3 % per layer adding up as sqrt(40).  The library
# measures 2.0-2.2 % on the same rows, whichever of its kernel routes the layers take.  The head doubles a feature error
# (measured), so the means decoded from those features are only held to 1.5e-1 end to end, and the head itself is held to
# the flat 2e-2 on the ORACLE's features in a step of its own.  The draft side (4 layers), the entropies and the head
# on the draft's features are held to the flat bars.
TARGET_TOL = 4e-2
TARGET_MU_TOL = 1.5e-1


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
    free = teacher_forced_round(case, ctx, o, [SAMPLE], verify_tol=TARGET_TOL, verify_mu_tol=TARGET_MU_TOL)
    assert abs(float(free["H"][SAMPLE, 0]) - float(o["H"][0, 0])) <= 1e-3
    assert rel_inf(free["mu_q"][SAMPLE, 0], o["mu_q"][0, 0]) < 2e-2
    assert rel_inf(free["mu_p"][SAMPLE, 0], o["mu_p"][0, 0]) < TARGET_MU_TOL
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
    # ... and on the oracle's TARGET features at the verify stage's row count (72 rows: the sample's 9 rows, eight times)
    zp = np.tile(o["z_p"][0], (8, 1))                      # [72, 5120]
    eps_p = np.tile(case.inp["eps_draft"][:, SAMPLE], (1, 8, 1))          # [S+1, 72, D]
    mu, _ = ctx.diffhead_decode(ctx.dev_store(gen.bf16_round(zp.astype(np.float32))), ctx.dev_f32(eps_p))
    ctx.sync()
    mu = mu.cpu().numpy()
    e = max(rel_inf(mu[9 * t:9 * t + 9], o["mu_p"][0]) for t in range(8))
    print(f"[configs[3]] diffhead_decode of 72 rows on the oracle's target features: {e:.2e}")
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
        er = rel_rms(z.float().cpu().numpy()[r0:r0 + n_q[SAMPLE]], zo)
        print(f"[configs[3]] {prefix}: z {ez:.2e} (rms {er:.2e}) shallow {es:.2e}")
        assert zo.shape[1] == 5120
        assert es < 2e-2                                    # after one layer
        assert ez < (TARGET_TOL if which == binding.TARGET else 2e-2)
