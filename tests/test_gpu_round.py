"""GPU parity of the whole speculative round (draft stage, verify stage, accept, commit) against the
CPU oracle, through the C-ABI."""
import numpy as np
import pytest

from synth import gen
from synth.configs import DT_BF16, DT_F32, ENT_ATTN, config
from tests.harness import (build_case, make_ctx, run_gpu_round, run_oracle_round, rel_inf, gpu_inputs, to_np,
                           oracle_caches)

pytestmark = pytest.mark.gpu

TOL = {DT_BF16: 2e-2, DT_F32: 2e-4}


def _compare_round(case, g, o, tau, samples=None):
    """Element-wise comparison; decisions are compared where they are not within the stated
    distance of their threshold (entropy 1e-3 of tau; ln r within 1e-3*max(1,|ln rho|) of ln rho)."""
    idx = list(range(case.B)) if samples is None else list(samples)
    tol = TOL[case.rc.dtype]
    K = case.rc.K
    Hg, Ho = g["H"][idx], o["H"]
    # entropies of executed steps
    executed = np.zeros_like(Ho, dtype=bool)
    for b in range(len(idx)):
        executed[b, :min(int(o["n_keep"][b]) + 1, K)] = True
    near_tau = (np.abs(Ho - tau) <= 1e-3) & executed
    clean = ~near_tau.any(axis=1)
    assert clean.sum() >= max(1, len(idx) // 2)
    eH = float(np.abs(Hg - Ho)[executed & clean[:, None]].max())
    assert eH <= 1e-3
    assert np.array_equal(g["keep"][idx][clean], o["keep"][clean])
    assert np.array_equal(g["n_keep"][idx][clean], o["n_keep"][clean])
    for bi, b in enumerate(idx):
        if not clean[bi]:
            continue
        nk = int(o["n_keep"][bi])
        if nk:
            ex, eq = rel_inf(g["x_draft"][b, :nk], o["x"][bi, :nk]), rel_inf(g["mu_q"][b, :nk], o["mu_q"][bi, :nk])
            assert ex < tol
            assert eq < tol
        ep = rel_inf(g["mu_p"][b, :nk + 1], o["mu_p"][bi, :nk + 1])
        assert ep < tol
        tail_zero = not g["mu_p"][b, nk + 1:].any()
        assert tail_zero
    return clean


@pytest.mark.parametrize("kind", ["ln-gelu-bf16", "gqa-rope-bf16", "ln-gelu-f32", "mid-bf16"])
def test_round_matches_oracle_no_filtering(kind):
    case = build_case(kind, seed=31)
    g = run_gpu_round(case, tau=-1.0)
    o = run_oracle_round(case, tau=-1.0)
    clean = _compare_round(case, g, o, -1.0)
    assert clean.all()
    assert np.array_equal(g["n_keep"], np.full(case.B, case.rc.K))
    # accept decisions on the library's own means, checked with the oracle's accept rule (unit level)
    from oracle import accept as oac
    s = case.rc.head.sigma_last * case.rc.head.temperature
    n_o, lr_o, _ = oac.accept(g["x_draft"], g["mu_p"], g["mu_q"], case.inp["r"], g["n_keep"], 0.0, s, s)
    assert np.allclose(g["log_ratio"], lr_o, rtol=1e-3, atol=2e-3)
    with np.errstate(divide="ignore"):
        margin = np.abs(lr_o - np.log(case.inp["r"].astype(np.float64)))
    safe = (margin > 1e-3 * np.maximum(1.0, np.abs(lr_o))).all(axis=1)
    assert np.array_equal(g["n_accept"][safe], n_o[safe])
    # cache bookkeeping follows the accepted length
    assert np.array_equal(g["len_t"], case.n_ctx + 1 + g["n_accept"])
    assert np.array_equal(g["len_d"], case.n_ctx + np.minimum(1 + g["n_accept"], case.rc.K))


@pytest.mark.parametrize("kind", ["ln-gelu-bf16", "gqa-rope-bf16", "ln-gelu-f32"])
def test_round_with_entropy_early_stop(kind):
    """tau placed inside the spread of the draft entropies: some samples stop early."""
    # a wide input projection makes the shallow features, hence their entropies, differ per token
    case = build_case(kind, seed=32, std_overrides={"in.w": 0.5})
    o_all = run_oracle_round(case, tau=-1.0)
    Hs = np.sort(o_all["H"].reshape(-1))
    gaps = np.diff(Hs)
    j = int(np.argmax(gaps))                              # widest gap: decisions stay off the threshold
    tau = float(0.5 * (Hs[j] + Hs[j + 1]))
    print(f"tau {tau:.4f} in a gap of {gaps[j]:.2e}")
    o = run_oracle_round(case, tau=tau)
    g = run_gpu_round(case, tau=tau)
    assert 0 < o["n_keep"].sum() < case.B * case.rc.K
    _compare_round(case, g, o, tau)


def test_draft_equal_to_target_accepts_everything():
    case = build_case("ln-gelu-bf16", seed=33, same_draft=True)
    g = run_gpu_round(case, tau=-1.0)
    assert np.array_equal(g["n_keep"], np.full(case.B, case.rc.K))
    # same weights, same caches, same noise: mu_p == mu_q up to the GEMM tile shapes (M differs)
    assert rel_inf(g["mu_p"][:, :case.rc.K], g["mu_q"]) < 2e-2
    o = run_oracle_round(case, tau=-1.0)
    assert np.array_equal(o["n_accept"], np.full(case.B, case.rc.K))
    # with rho ~ 1 every uniform below 1 - margin accepts
    lr = g["log_ratio"]
    ok = (np.log(case.inp["r"].astype(np.float64)) <= lr - 1e-3).all(axis=1)
    assert np.array_equal(g["n_accept"][ok], np.full(ok.sum(), case.rc.K))


def test_all_filtered_round_is_a_plain_ar_step():
    case = build_case("ln-gelu-bf16", seed=34)
    g = run_gpu_round(case, tau=1e9)
    o = run_oracle_round(case, tau=1e9)
    assert not g["keep"].any() and not g["n_accept"].any()
    assert rel_inf(g["mu_p"][:, 0], o["mu_p"][:, 0]) < 2e-2
    assert not g["mu_p"][:, 1:].any()
    assert np.array_equal(g["len_t"], np.full(case.B, case.n_ctx + 1))
    assert np.array_equal(g["len_d"], np.full(case.B, case.n_ctx + 1))


def test_attn_mode_entropy_round():
    case = build_case("ln-gelu-bf16", seed=35, peaky=True)
    case.rc.entropy_mode = ENT_ATTN
    o_all = run_oracle_round(case, tau=-1.0)
    tau = float(np.median(o_all["H"][:, 1]))
    o = run_oracle_round(case, tau=tau)
    g = run_gpu_round(case, tau=tau)
    # a stress variant outside the workload recipe (scores with a standard deviation near 2): the bf16 rounding of
    # q and k alone moves these entropies by up to 1e-2; the stated 1e-3 is held at the recipe, in
    # test_attn_mode_entropy_at_the_workload_recipe
    executed = np.zeros_like(o["H"], dtype=bool)
    for b in range(case.B):
        executed[b, :min(int(o["n_keep"][b]) + 1, case.rc.K)] = True
    eH = float(np.abs(g["H"] - o["H"])[executed].max())
    assert eH < 2e-2


def test_attn_mode_entropy_at_the_workload_recipe():
    """ATTN-mode entropy (Eq. 1 / S2.1 read on the attention rows of draft layer l_s) at configs[1]'s full shape and
    the workload recipe, held to the stated 1e-3 on every draft step (teacher-forced, so that a step is not charged
    with the drift of the steps before it) and on the free-running first step."""
    case = build_case(1, seed=0, affine=False)
    case.rc.entropy_mode = ENT_ATTN
    idx = [0, case.B - 1]
    o = run_oracle_round(case, tau=-1.0, samples=idx)
    assert o["H"].min() > 1.0                              # ln(130) = 4.9 for uniform rows: these are attention entropies
    ctx = make_ctx(case)
    free = teacher_forced_round(case, ctx, o, idx)
    for bi, b in enumerate(idx):
        assert abs(float(free["H"][b, 0]) - float(o["H"][bi, 0])) <= 1e-3
    ctx.close()


def test_two_rounds_in_a_row_reuse_the_context():
    """Second round starts from the committed caches; compare with an oracle that does the same."""
    from oracle import round as rnd
    case = build_case("ln-gelu-bf16", seed=36)
    ctx = make_ctx(case)
    gi = gpu_inputs(ctx, case)
    o1 = to_np(ctx.spec_round(gi["pending"], gi["eps"], gi["r"], -1.0))
    inp2 = gen.round_inputs(case.rc, 77, case.B)
    o2 = to_np(ctx.spec_round(ctx.dev_f32(inp2["pending"]), ctx.dev_f32(inp2["eps_draft"]), ctx.dev_f32(inp2["r"]), -1.0))
    ctx.sync()
    tc, dc = oracle_caches(case)
    r1 = rnd.spec_round(case.rc, case.W, tc, dc, case.inp["pending"], case.inp["eps_draft"], case.inp["r"], -1.0, case.B)
    if not np.array_equal(r1["n_accept"], o1["n_accept"]):
        pytest.skip("first-round accept decisions differ within tolerance; second round not comparable")
    # the draft cache is one token short for samples that accepted all K drafts: skip those
    full = r1["n_accept"] == case.rc.K
    r2 = rnd.spec_round(case.rc, case.W, tc, dc, inp2["pending"], inp2["eps_draft"], inp2["r"], -1.0, case.B)
    for b in range(case.B):
        if full[b]:
            continue
        assert rel_inf(o2["mu_p"][b], r2["mu_p"][b]) < 2e-2
        assert rel_inf(o2["mu_q"][b], r2["mu_q"][b]) < 2e-2
    ctx.close()


def test_config1_full_size_sampled_samples():
    """BASELINE configs[1] at full size in the launch configuration the benchmark times; the oracle
    recomputes two of the 32 samples (samples are independent)."""
    case = build_case(1, seed=0, affine=False)
    g = run_gpu_round(case, tau=-1.0)
    idx = [0, case.B - 1]
    o = run_oracle_round(case, tau=-1.0, samples=idx)
    _compare_round(case, g, o, -1.0, samples=idx)
    assert np.isfinite(g["mu_p"]).all() and np.isfinite(g["log_ratio"]).all()
    # no kernel on this path combines partial sums with atomics: a second run gives the same bits
    g2 = run_gpu_round(case, tau=-1.0)
    for k in ("H", "x_draft", "mu_q", "mu_p", "log_ratio", "n_accept"):
        assert np.array_equal(g[k], g2[k]), k


def rel_rms(g, o):
    """Root-mean-square error over the root-mean-square of the oracle's values."""
    o = np.asarray(o, dtype=np.float64)
    return float(np.sqrt(np.mean((np.asarray(g, dtype=np.float64) - o) ** 2) / max(np.mean(o ** 2), 1e-300)))


def teacher_forced_round(case, ctx, o, idx, tau=-1.0, verify_tol=None, verify_mu_tol=None):
    """The full-size check that bounds the kernels rather than the chain: the K draft steps depend on one another
    (the latent of step i is the input of step i + 1 and enters the draft cache), so a free-running comparison of
    step 7 measures seven steps of accumulated bf16 rounding.  Here every draft step of the sampled samples is fed the
    ORACLE's previous token (spec_draft_step), and spec_verify gets the oracle's drafts, draft means and survivor
    counts; every row is then held to the flat bars (latents and means 2e-2 over the sample's tensor, entropy 1e-3
    absolute).  The other samples of the batch run on the library's own tokens, so the launch shapes are those of the
    benchmark.  Returns the free-running round (whose drift against the oracle is printed, not gated).
    verify_tol / verify_mu_tol: other bars for the target's features and for the means decoded from them (see
    tests/test_gpu_config3.py; there the head is checked on the oracle's features in a step of its own)."""
    from paper_2512_08537_amd import binding
    rc, B, K = case.rc, case.B, case.rc.K
    tol = TOL[rc.dtype]
    gi = gpu_inputs(ctx, case)
    lens = np.full(B, case.n_ctx, dtype=np.int32)

    def rewind():
        ctx.spec_kv_reset(binding.TARGET, lens)
        ctx.spec_kv_reset(binding.DRAFT, lens)

    rewind()
    free = to_np(ctx.spec_round(gi["pending"], gi["eps"], gi["r"], tau))
    ctx.sync()
    # --- draft steps on the oracle's tokens
    rewind()
    out = ctx._round_bufs(B)
    for i in range(K):
        x_prev = case.inp["pending"].copy() if i == 0 else free["x_draft"][:, i - 1].copy()
        if i > 0:
            for bi, b in enumerate(idx):
                if i - 1 < int(o["n_keep"][bi]):
                    x_prev[b] = o["x"][bi, i - 1]
        ctx.spec_draft_step(i, ctx.dev_f32(x_prev), gi["eps"], tau, out)
    ctx.sync()
    g = to_np(out)
    for bi, b in enumerate(idx):
        nk = int(o["n_keep"][bi])
        n_ex = min(nk + 1, K)
        eh = np.abs(g["H"][b, :n_ex] - o["H"][bi, :n_ex])
        drift_h = np.abs(free["H"][b, :n_ex] - o["H"][bi, :n_ex])
        print(f"sample {b}: entropy per step (teacher-forced) {np.array2string(eh, precision=1)}  free-running {np.array2string(drift_h, precision=1)}")
        assert eh.max() <= 1e-3
        assert int(g["n_keep"][b]) == nk
        if nk:
            per = [rel_inf(g["mu_q"][b, i], o["mu_q"][bi, i]) for i in range(nk)]
            drift = [rel_inf(free["mu_q"][b, i], o["mu_q"][bi, i]) for i in range(nk)]
            print(f"sample {b}: mu_q per step (teacher-forced) {np.array2string(np.array(per), precision=4)}  free-running {np.array2string(np.array(drift), precision=4)}")
            assert rel_inf(g["mu_q"][b, :nk], o["mu_q"][bi, :nk]) < tol
            assert rel_inf(g["x_draft"][b, :nk], o["x"][bi, :nk]) < tol
            assert max(per) < 2 * tol                      # no single step hides behind a large row of the tensor
    # --- verify on the oracle's drafts
    x_d, mu_q, nk_all = free["x_draft"].copy(), free["mu_q"].copy(), free["n_keep"].copy()
    for bi, b in enumerate(idx):
        x_d[b], mu_q[b], nk_all[b] = o["x"][bi], o["mu_q"][bi], o["n_keep"][bi]
    rewind()
    v = ctx.spec_verify(gi["pending"], ctx.dev_f32(x_d), ctx.dev_f32(mu_q), ctx.dev_i32(nk_all), gi["r"], gi["eps"], want_z=True)
    ctx.sync()
    v = to_np(v)
    from oracle import accept as oac
    sg = rc.head.sigma_last * rc.head.temperature
    tol_z = tol if verify_tol is None else verify_tol
    tol_mu = tol_z if verify_mu_tol is None else verify_mu_tol
    for bi, b in enumerate(idx):
        nk = int(o["n_keep"][bi])
        rz, rp = rel_rms(v["z_p"][b, :nk + 1], o["z_p"][bi]), rel_rms(v["mu_p"][b, :nk + 1], o["mu_p"][bi, :nk + 1])
        print(f"sample {b}: verify rms-relative z_p {rz:.2e} mu_p {rp:.2e}")
        ep = rel_inf(v["mu_p"][b, :nk + 1], o["mu_p"][bi, :nk + 1])
        ez = rel_inf(v["z_p"][b, :nk + 1], o["z_p"][bi])
        per = [rel_inf(v["mu_p"][b, j], o["mu_p"][bi, j]) for j in range(nk + 1)]
        drift = [rel_inf(free["mu_p"][b, j], o["mu_p"][bi, j]) for j in range(min(nk, int(free["n_keep"][b])) + 1)]
        print(f"sample {b}: verify z_p {ez:.2e} mu_p {ep:.2e}; per row {np.array2string(np.array(per), precision=4)}  free-running {np.array2string(np.array(drift), precision=4)}")
        assert ez < tol_z and ep < tol_mu
        assert max(per) < 2 * tol_mu
        assert not v["mu_p"][b, nk + 1:].any()
        if nk:
            # ln rho: exact rule on the library's own means (unit level), and against the oracle's value
            _, lr_unit, _ = oac.accept(x_d[b:b + 1], v["mu_p"][b:b + 1], mu_q[b:b + 1], case.inp["r"][b:b + 1], nk_all[b:b + 1], 0.0, sg, sg)
            assert np.allclose(v["log_ratio"][b, :nk], lr_unit[0, :nk], rtol=1e-3, atol=2e-3)
            el = rel_inf(v["log_ratio"][b, :nk], o["log_ratio"][bi, :nk])
            print(f"sample {b}: ln rho against the oracle {el:.2e}")
            assert el < tol_mu
    return free


def test_config2_full_size_teacher_forced():
    """BASELINE configs[2] (L=32, d=1280, B=64: 576 verify rows, K = 1280 / 5120 GEMMs) at full size; the oracle
    recomputes one of the 64 samples; flat bars on every step and row (teacher_forced_round)."""
    case = build_case(2, seed=0, affine=False)
    idx = [case.B - 1]
    o = run_oracle_round(case, tau=-1.0, samples=idx)
    ctx = make_ctx(case)
    free = teacher_forced_round(case, ctx, o, idx)
    # the free-running round itself: its first step and first verify row have no chain behind them
    for bi, b in enumerate(idx):
        assert abs(float(free["H"][b, 0]) - float(o["H"][bi, 0])) <= 1e-3
        assert rel_inf(free["mu_q"][b, 0], o["mu_q"][bi, 0]) < 2e-2
        assert rel_inf(free["mu_p"][b, 0], o["mu_p"][bi, 0]) < 2e-2
    assert np.isfinite(free["mu_p"]).all() and np.isfinite(free["log_ratio"]).all()
    ctx.close()


def test_config4_full_size_teacher_forced():
    """BASELINE configs[4] shape (configs[2] model, B=256, n_ctx=1024: 2304 verify rows, 33 key blocks per head) at
    full size, one synthetic cache shared by all layers (44 GB of distinct cache would not fit the host); the
    oracle recomputes two samples; flat bars on every step and row."""
    case = build_case(4, seed=0, affine=False, cache_layers_shared=True)
    idx = [0, case.B // 2]
    o = run_oracle_round(case, tau=-1.0, samples=idx)
    ctx = make_ctx(case)
    free = teacher_forced_round(case, ctx, o, idx)
    for bi, b in enumerate(idx):
        assert abs(float(free["H"][b, 0]) - float(o["H"][bi, 0])) <= 1e-3
        assert rel_inf(free["mu_q"][b, 0], o["mu_q"][bi, 0]) < 2e-2
        assert rel_inf(free["mu_p"][b, 0], o["mu_p"][bi, 0]) < 2e-2
    assert np.isfinite(free["mu_p"]).all() and np.isfinite(free["log_ratio"]).all()
    ctx.close()


def test_config0_full_round_fp32():
    """BASELINE configs[0] at its own shape (4 layers, d = 256, 4 heads, MLP 1024, 1-layer draft, K = 4, batch 1,
    64 cached tokens, 3-block head, one step, fp32): the whole batch, every output, at the fp32 bar; the cache is
    built by the library's own prefill of 64 latents, as that configuration says."""
    from oracle import transformer as tf
    from oracle import round as rnd
    from paper_2512_08537_amd import binding
    case = build_case(0, seed=0, affine=False)
    rc = case.rc
    assert (rc.target.n_layers, rc.target.d_model, rc.K, case.B, case.n_ctx, rc.dtype) == (4, 256, 4, 1, 64, DT_F32)
    ctx = make_ctx(case)
    rng = np.random.default_rng(0)
    x = rng.normal(size=(1, 64, rc.target.d_latent)).astype(np.float32)
    n = np.array([64], np.int32)
    tc, dc = tf.KVCache(rc.target, 1), tf.KVCache(rc.draft, 1)
    for which, cfg, prefix, cache in ((binding.TARGET, rc.target, "target", tc), (binding.DRAFT, rc.draft, "draft", dc)):
        ctx.spec_kv_reset(which, None)
        ctx.spec_prefill(which, ctx.dev_f32(x), n)
        tf.forward_sample(cfg, case.W, prefix, cache, 0, x[0], commit=True)
    for tau in (-1.0, None):
        if tau is None:                                    # the paper's threshold rule on this round's entropies
            tau = float(binding.entropy_threshold(float(o["H"].mean()), float(o["H"].std())))
            tc.truncate(0, 64), dc.truncate(0, 64)
            ctx.spec_kv_reset(binding.TARGET, n), ctx.spec_kv_reset(binding.DRAFT, n)
        o = rnd.spec_round(rc, case.W, tc, dc, case.inp["pending"], case.inp["eps_draft"], case.inp["r"], tau, 1)
        gi = gpu_inputs(ctx, case)
        g = to_np(ctx.spec_round(gi["pending"], gi["eps"], gi["r"], tau))
        ctx.sync()
        nk = int(o["n_keep"][0])
        assert int(g["n_keep"][0]) == nk == rc.K
        assert np.abs(g["H"] - o["H"]).max() <= 1e-3
        for k_g, k_o in (("x_draft", "x"), ("mu_q", "mu_q"), ("mu_p", "mu_p")):
            e = rel_inf(g[k_g], o[k_o])
            print(f"configs[0] tau {tau:.3f}: {k_g} {e:.2e}")
            assert e < TOL[DT_F32]
        assert rel_inf(g["log_ratio"], o["log_ratio"]) < 2e-3
        with np.errstate(divide="ignore"):
            margin = np.abs(o["log_ratio"] - np.log(case.inp["r"].astype(np.float64)))
        if (margin > 1e-3 * np.maximum(1.0, np.abs(o["log_ratio"]))).all():
            assert np.array_equal(g["n_accept"], o["n_accept"])
        assert np.array_equal(ctx.spec_kv_lengths(binding.TARGET, 1), [64 + 1 + int(g["n_accept"][0])])
    ctx.close()


def test_draft_steps_one_by_one_equal_spec_draft_and_lengths_restore_from_device():
    """spec_draft_step K times (tokens taken from the library's own previous drafts) is spec_draft bit for bit, with
    other calls on the context in between; spec_kv_restore rewinds the lengths from device memory and clamps them to
    the bound the host is given; spec_kv_lengths resets the host's bound to the true maximum."""
    import torch
    from paper_2512_08537_amd import binding
    case = build_case("mid-bf16", seed=37, std_overrides={"in.w": 0.5})
    rc, B, K = case.rc, case.B, case.rc.K
    ctx = make_ctx(case)
    gi = gpu_inputs(ctx, case)
    o_all = to_np(ctx.spec_draft(gi["pending"], gi["eps"], -1.0))
    tau = float(np.median(o_all["H"]))                     # some samples stop early
    lens = ctx.dev_i32(np.full(B, case.n_ctx, dtype=np.int32))
    ctx.spec_kv_restore(binding.DRAFT, lens, case.n_ctx)
    ref = to_np(ctx.spec_draft(gi["pending"], gi["eps"], tau))
    assert 0 < ref["n_keep"].sum() < B * K
    assert np.array_equal(ctx.spec_kv_lengths(binding.DRAFT, B), np.full(B, case.n_ctx + K))
    ctx.spec_kv_restore(binding.DRAFT, lens, case.n_ctx)
    out = ctx._round_bufs(B)
    junk = ctx.dev_f32(np.zeros((B, 16), np.float32))
    for i in range(K):
        ctx.spec_draft_step(i, gi["pending"] if i == 0 else None, gi["eps"], tau, out)
        if i == 2:                                          # another call in between uses the row maps and the workspace
            ctx.spec_forward(binding.TARGET, junk, np.ones(B, np.int32), commit=False)
    ctx.sync()
    got = to_np(out)
    for k in ("H", "keep", "n_keep", "x_draft", "mu_q"):
        assert np.array_equal(got[k], ref[k]), k
    with pytest.raises(binding.FardError) as e:             # steps out of order
        ctx.spec_draft_step(3, None, gi["eps"], tau, out)
    assert e.value.code == -6
    # lengths from device memory: clamped to the host's bound, and the bound is what capacity is checked against
    big = ctx.dev_i32(np.array([5, 10 ** 6, -4] + [7] * (B - 3), dtype=np.int32))
    ctx.spec_kv_restore(binding.TARGET, big, 40)
    got_len = ctx.spec_kv_lengths(binding.TARGET, B)
    assert got_len[0] == 5 and got_len[1] == 40 and got_len[2] == 0 and (got_len[3:] == 7).all()
    with pytest.raises(binding.FardError) as e:
        ctx.spec_kv_restore(binding.TARGET, big, rc.max_ctx + 1)
    assert e.value.code == -3
    # a round raises the host's bound by K + 1 whatever was accepted; reading the lengths brings it back to the truth
    ctx.spec_kv_restore(binding.TARGET, lens, rc.max_ctx - K - 1)      # the bound says: nearly full
    ctx.spec_kv_restore(binding.DRAFT, lens, case.n_ctx)
    ctx.spec_round(gi["pending"], gi["eps"], gi["r"], -1.0)
    with pytest.raises(binding.FardError):                  # by the bound there is no room for another round
        ctx.spec_round(gi["pending"], gi["eps"], gi["r"], -1.0)
    ctx.spec_kv_lengths(binding.TARGET, B)                  # true lengths: n_ctx + 1 + n_accept
    ctx.spec_kv_restore(binding.DRAFT, lens, case.n_ctx)
    ctx.spec_round(gi["pending"], gi["eps"], gi["r"], -1.0)
    ctx.sync()
    ctx.close()
