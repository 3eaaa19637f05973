"""Pins for oracle/head.py, oracle/accept.py and oracle/round.py (Sec. 3.2, Sec. 4.2, S3, Alg. 1)."""
import math

import numpy as np
import pytest
from scipy.stats import norm as gauss

from oracle import head as hd
from oracle import accept as ac
from oracle import round as rnd
from oracle import transformer as tf
from oracle import entropy as ent
from oracle import loops
from synth import gen
from synth.configs import HeadCfg, RoundCfg, TfCfg, DT_F32, reduced, clone, ENT_ATTN

RNG = np.random.default_rng(99)


def small_head(S=1, renoise=1, N=2):
    return HeadCfg(n_blocks=N, width=24, d_cond=12, d_latent=4, n_steps=S, t_freq_dim=16, renoise=renoise)


def head_w(hc, seed=0, std=0.3):
    return gen.head_weights(hc, seed, DT_F32, w_std=std, affine=True)


# ----------------------------------------------------------------------------- head
def test_zero_weight_head_reduces_to_bias():
    hc = small_head(S=1)
    W = {k: np.zeros_like(v) for k, v in head_w(hc).items()}
    W["head.out.b"] = np.array([0.5, -1.0, 2.0, 0.25], np.float32)
    z = RNG.normal(size=(3, hc.d_cond))
    x_t = RNG.normal(size=(3, 4))
    for t in (1.0, 0.5):
        assert np.allclose(hd.velocity(hc, W, x_t, t, z), W["head.out.b"][None, :])
    eps = RNG.normal(size=(2, 3, 4))
    mu, x = hd.decode(hc, W, z, eps)
    assert np.allclose(mu, eps[0] - 1.0 * W["head.out.b"])          # x0_hat = x_t - t v at t = 1
    assert np.allclose(x, mu + hc.sigma_last * eps[1])


def test_zero_modulation_makes_blocks_identity():
    hc = small_head()
    W = head_w(hc)
    for j in range(hc.n_blocks):
        W[f"head.B{j}.mod.w"][:] = 0
        W[f"head.B{j}.mod.b"][:] = 0
    W["head.f.mod.w"][:] = 0
    W["head.f.mod.b"][:] = 0
    z = RNG.normal(size=(5, hc.d_cond))
    x_t = RNG.normal(size=(5, 4))
    h = x_t @ W["head.in.w"].astype(float) + W["head.in.b"]
    want = hd.ln_plain(h) @ W["head.out.w"].astype(float) + W["head.out.b"]
    assert np.allclose(hd.velocity(hc, W, x_t, 0.7, z), want, rtol=1e-12)


def test_gate_only_scales_the_branch():
    """One block, mod.w = 0: (shift, scale, gate) are constants b; doubling the gate bias
    doubles the block's contribution to h, seen through a linear read-out of h."""
    hc = small_head(N=1)
    W = head_w(hc)
    w = hc.width
    W["head.B0.mod.w"][:] = 0
    W["head.f.mod.w"][:] = 0
    W["head.f.mod.b"][:] = 0
    z = RNG.normal(size=(2, hc.d_cond))
    x_t = RNG.normal(size=(2, 4))

    def h_after(gscale):
        V = {k: v.copy() for k, v in W.items()}
        V["head.B0.mod.b"][2 * w:] *= gscale
        h = x_t @ V["head.in.w"].astype(float) + V["head.in.b"]
        b = V["head.B0.mod.b"].astype(float)
        a = hd.ln_plain(h) * (1 + b[w:2 * w]) + b[:w]
        a = hd.silu(a @ V["head.B0.w1"].astype(float) + V["head.B0.b1"])
        return V, h, b[2 * w:] * (a @ V["head.B0.w2"].astype(float) + V["head.B0.b2"])

    V1, h, br1 = h_after(1.0)
    want = hd.ln_plain(h + br1) @ V1["head.out.w"].astype(float) + V1["head.out.b"]
    assert np.allclose(hd.velocity(hc, V1, x_t, 0.3, z), want, rtol=1e-12)
    V2, _, br2 = h_after(2.0)
    assert np.allclose(br2, 2 * br1)


def test_time_embedding_at_zero_and_frequency_layout():
    hc = small_head()
    W = head_w(hc)
    half = hc.t_freq_dim // 2
    feat = np.concatenate([np.ones(half), np.zeros(half)])        # cos(0), sin(0)
    a = hd.silu(feat @ W["head.t1.w"].astype(float) + W["head.t1.b"])
    assert np.allclose(hd.time_embedding(hc, W, 0.0), a @ W["head.t2.w"].astype(float) + W["head.t2.b"])
    # the lowest frequency is omega_0 = 1: only row 0 (cos) and row `half` (sin) see t*t_scale directly
    V = {k: np.zeros_like(v) for k, v in W.items()}
    V["head.t1.w"][half, 0] = 1.0                                   # picks sin(t * t_scale * 1)
    V["head.t2.w"][0, 0] = 1.0
    t = 0.001
    got = hd.time_embedding(hc, V, t)[0]
    s = math.sin(t * hc.t_scale)
    assert got == pytest.approx(s / (1 + math.exp(-s)), rel=1e-12)


def test_euler_with_constant_velocity_and_multi_step_equals_one_step():
    W1 = {k: np.zeros_like(v) for k, v in head_w(small_head()).items()}
    v = np.array([0.3, -0.2, 1.0, 0.0], np.float32)
    W1["head.out.b"] = v
    z = RNG.normal(size=(2, 12))
    eps = RNG.normal(size=(5, 2, 4))
    outs = []
    for S in (1, 2, 4):
        hc = small_head(S=S, renoise=0)
        e = np.concatenate([eps[:1], eps[1:S], eps[4:5]]) if S > 1 else np.stack([eps[0], eps[4]])
        mu, _ = hd.decode(hc, W1, z, e)
        outs.append(mu)
        assert np.allclose(mu, eps[0] - v)                          # x0 = eps0 - v for a constant field
    assert np.allclose(outs[0], outs[1]) and np.allclose(outs[0], outs[2])


def test_renoise_step_uses_fresh_noise():
    hc = small_head(S=2, renoise=1)
    W = {k: np.zeros_like(v) for k, v in head_w(hc).items()}
    v = np.array([1.0, 2.0, 3.0, 4.0], np.float32)
    W["head.out.b"] = v
    z = np.zeros((1, 12))
    eps = RNG.normal(size=(3, 1, 4))
    mu, x = hd.decode(hc, W, z, eps)
    x0_a = eps[0] - v                       # t = 1
    x_half = 0.5 * x0_a + 0.5 * eps[1]      # re-noise to t = 1/2 with eps[1]
    assert np.allclose(mu, x_half - 0.5 * v)
    assert np.allclose(x, mu + 0.25 * eps[2])


def test_temperature_scales_start_and_final_noise():
    hc = small_head(S=1)
    hc.temperature = 0.5
    W = {k: np.zeros_like(v) for k, v in head_w(hc).items()}
    eps = RNG.normal(size=(2, 1, 4))
    mu, x = hd.decode(hc, W, np.zeros((1, 12)), eps)
    assert np.allclose(mu, 0.5 * eps[0]) and np.allclose(x, mu + 0.25 * 0.5 * eps[1])


# ----------------------------------------------------------------------------- accept
def test_equal_means_give_ratio_one_and_accept_everything():
    B, K, D = 4, 6, 16
    x = RNG.normal(size=(B, K, D))
    mu = RNG.normal(size=(B, K, D))
    mu_p = np.concatenate([mu, RNG.normal(size=(B, 1, D))], axis=1)
    r = np.concatenate([np.zeros((B, 1)), RNG.random((B, K - 1)) * (1 - 1e-12)], axis=1)
    n_keep = np.array([6, 3, 0, 5])
    n_acc, lr, acc = ac.accept(x, mu_p, mu, r, n_keep, 0.0, 0.25, 0.25)
    assert np.allclose(lr, 0.0, atol=1e-12)
    assert np.array_equal(n_acc, n_keep) and acc.all()


def test_log_ratio_closed_form_1d():
    x, mp, mq, sp, sq = 0.3, -0.2, 0.5, 0.7, 0.4
    want = math.log(gauss.pdf(x, mp, sp) / gauss.pdf(x, mq, sq))
    got = ac.log_ratio(np.array([x]), np.array([mp]), np.array([mq]), 0.0, sp, sq)
    assert got == pytest.approx(want, rel=1e-12)
    assert ac.log_ratio(np.array([x]), np.array([mp]), np.array([mq]), 0.75, sp, sq) == pytest.approx(want + 0.75)


def test_log_ratio_matches_multivariate_density():
    D = 16
    x, mp, mq = RNG.normal(size=D), RNG.normal(size=D), RNG.normal(size=D)
    sp, sq = 0.3, 0.45
    lp = gauss.logpdf(x, mp, sp).sum()
    lq = gauss.logpdf(x, mq, sq).sum()
    assert ac.log_ratio(x, mp, mq, 0.0, sp, sq) == pytest.approx(lp - lq, rel=1e-11)


def test_log_sigma_factor():
    assert ac.log_sigma_factor([], [], 16) == 0.0
    # T = 3: steps t = 2, 3; |Sigma| = sigma^(2D) -> ln Sigma = D sum ln(sigma_q / sigma_p)
    want = 0.5 * (math.log((0.5 ** 32) / (0.25 ** 32)) + math.log((0.2 ** 32) / (0.4 ** 32)))
    assert ac.log_sigma_factor([0.5, 0.2], [0.25, 0.4], 16) == pytest.approx(want, rel=1e-12)


def test_acceptance_probability_monte_carlo():
    """Equal-sigma Gaussians: E_q[min(1, p/q)] = 2 Phi(-|delta| / (2 sigma))."""
    n, D, s = 100_000, 3, 0.25
    delta = np.array([0.2, -0.1, 0.15])
    x = RNG.normal(size=(n, 1, D)) * s                     # x ~ q = N(0, s^2 I)
    mu_q = np.zeros((n, 1, D))
    mu_p = np.broadcast_to(delta, (n, 2, D))
    r = RNG.random((n, 1))
    n_acc, _, _ = ac.accept(x, mu_p, mu_q, r, np.ones(n, int), 0.0, s, s)
    p = 2 * gauss.cdf(-np.linalg.norm(delta) / (2 * s))
    se = math.sqrt(p * (1 - p) / n)
    assert abs(n_acc.mean() - p) < 3 * se


def test_accept_is_leading_run_and_strictness():
    B, K, D = 50, 8, 2
    x, mu_q = RNG.normal(size=(B, K, D)), RNG.normal(size=(B, K, D))
    mu_p = RNG.normal(size=(B, K + 1, D)) * 0.3 + np.concatenate([mu_q, mu_q[:, :1]], 1)
    r = RNG.random((B, K))
    n_keep = RNG.integers(0, K + 1, size=B)
    n_acc, lr, acc = ac.accept(x, mu_p, mu_q, r, n_keep, 0.1, 0.8, 0.9)
    for b in range(B):
        flags = [math.log(r[b, i]) <= lr[b, i] for i in range(K)]
        assert n_acc[b] == loops.leading_run(flags, n_keep[b])
    # r == rho accepts (reject only on r > rho); r = 0 always accepts
    lr1 = ac.log_ratio(x[:1, :1], mu_p[:1, :1], mu_q[:1, :1], 0.0, 1.0, 1.0)
    rr = np.exp(lr1)
    if rr[0, 0] < 1:
        n1, _, _ = ac.accept(x[:1, :1], mu_p[:1, :2], mu_q[:1, :1], rr, np.array([1]), 0.0, 1.0, 1.0)
        assert n1[0] == 1
    n0, _, _ = ac.accept(x[:1, :1], mu_p[:1, :2] + 50, mu_q[:1, :1], np.zeros((1, 1)), np.array([1]), 0.0, 1.0, 1.0)
    assert n0[0] == 1


# ----------------------------------------------------------------------------- round
def _round_setup(kind="ln-gelu-f32", same=False, seed=0, tau=0.0):
    rc = reduced(kind)
    if same:
        rc.draft = clone(rc).target
    W = gen.tf_weights(rc.target, seed, "target", rc.dtype, w_std=0.08, affine=True)
    if same:
        W.update(gen.truncated_draft(W, rc.target, rc.draft))
    elif rc.draft.d_model == rc.target.d_model:
        W.update(gen.truncated_draft(W, rc.target, rc.draft))
    else:
        W.update(gen.tf_weights(rc.draft, seed, "draft", rc.dtype, w_std=0.08, affine=True))
    W.update(gen.head_weights(rc.head, seed, rc.dtype, w_std=0.08, affine=True))
    B = rc.batch
    tc, dc = tf.KVCache(rc.target, B), tf.KVCache(rc.draft, B)
    n = 5
    for l in range(rc.target.n_layers):
        k, v = gen.kv_cache(rc.target, seed, "target", l, B, n, rc.dtype)
        tc.load(l, k, v)
        if l < rc.draft.n_layers and rc.draft.d_model == rc.target.d_model:
            dc.load(l, k, v)
    if rc.draft.d_model != rc.target.d_model:
        for l in range(rc.draft.n_layers):
            k, v = gen.kv_cache(rc.draft, seed, "draft", l, B, n, rc.dtype)
            dc.load(l, k, v)
    inp = gen.round_inputs(rc, seed)
    return rc, W, tc, dc, inp, B


def test_draft_equal_to_target_accepts_everything():
    rc, W, tc, dc, inp, B = _round_setup(same=True)
    out = rnd.spec_round(rc, W, tc, dc, inp["pending"], inp["eps_draft"], inp["r"], tau=-1.0, B=B)
    assert np.array_equal(out["n_keep"], np.full(B, rc.K))
    assert np.array_equal(out["n_accept"], out["n_keep"])
    assert np.allclose(out["log_ratio"], 0.0, atol=1e-7)
    assert np.allclose(out["mu_p"][:, :rc.K], out["mu_q"], rtol=1e-9, atol=1e-11)
    for b in range(B):
        assert tc.length(b) == 5 + 1 + rc.K
        assert dc.length(b) == 5 + rc.K          # the draft never read its last token


def test_all_filtered_round_is_a_plain_ar_step():
    rc, W, tc, dc, inp, B = _round_setup()
    out = rnd.spec_round(rc, W, tc, dc, inp["pending"], inp["eps_draft"], inp["r"], tau=1e9, B=B)
    assert not out["keep"].any() and not out["n_accept"].any()
    ref = tf.KVCache(rc.target, 1)
    for l in range(rc.target.n_layers):
        k, v = gen.kv_cache(rc.target, 0, "target", l, B, 5, rc.dtype)
        ref.load(l, k[1:2], v[1:2])
    z, _, _ = tf.forward_sample(rc.target, W, "target", ref, 0, inp["pending"][1][None, :])
    mu, _ = hd.decode(rc.head, W, z, inp["eps_draft"][:, 1, :1])
    assert np.allclose(out["mu_p"][1, 0], mu[0], rtol=1e-12)
    assert tc.length(1) == 6


def test_round_is_independent_of_batch_composition():
    rc, W, tc, dc, inp, B = _round_setup(kind="gqa-rope-bf16")
    H = rnd.draft_stage(rc, W, dc, inp["pending"], inp["eps_draft"], -1.0, B)["H"]
    tau = float(np.sort(H.reshape(-1))[H.size // 3])          # filters some drafts
    rc, W, tc, dc, inp, B = _round_setup(kind="gqa-rope-bf16")
    full = rnd.spec_round(rc, W, tc, dc, inp["pending"], inp["eps_draft"], inp["r"], tau=tau, B=B)
    assert 0 < full["n_keep"].sum() < B * rc.K
    b = B - 1
    rc1, W1, tc1, dc1, inp1, _ = _round_setup(kind="gqa-rope-bf16")
    t1, d1 = tf.KVCache(rc.target, 1), tf.KVCache(rc.draft, 1)
    for l in range(rc.target.n_layers):
        t1.load(l, tc1.k[l][b][None], tc1.v[l][b][None])
    for l in range(rc.draft.n_layers):
        d1.load(l, dc1.k[l][b][None], dc1.v[l][b][None])
    solo = rnd.spec_round(rc, W, t1, d1, inp["pending"][b:b + 1], inp["eps_draft"][:, b:b + 1], inp["r"][b:b + 1],
                          tau=tau, B=1)
    for key in ("H", "keep", "x", "mu_q", "mu_p", "log_ratio", "n_accept"):
        assert np.array_equal(np.asarray(full[key])[b], np.asarray(solo[key])[0]), key


def test_attn_mode_round_runs_and_orders_entropy():
    rc, W, tc, dc, inp, B = _round_setup()
    rc.entropy_mode = ENT_ATTN
    out = rnd.spec_round(rc, W, tc, dc, inp["pending"], inp["eps_draft"], inp["r"], tau=-1.0, B=B)
    # attention rows have 5 + i + 1 visible keys at draft step i: 0 < H <= ln(count)
    for i in range(rc.K):
        assert np.all(out["H"][:, i] > 0) and np.all(out["H"][:, i] <= math.log(6 + i) + 1e-12)


def test_head_conditioning_path_written_out_by_hand():
    """One block, non-zero modulation weights and a non-zero z: c = W_c z + b_c + temb(t), every modulation is a
    projection of SiLU(c), split as shift | scale | gate (Sec. 3.2's conditioning on the AR feature).  Everything is
    evaluated here with explicit loops and the math module; dropping SiLU(c), dropping temb from c, or permuting the
    split changes the result by far more than the tolerance (checked below on the hand computation itself)."""
    hc = HeadCfg(n_blocks=1, width=6, d_cond=5, d_latent=3, n_steps=1, t_freq_dim=4, t_scale=10.0)
    W = head_w(hc, seed=3, std=0.5)
    w, D = hc.width, hc.d_latent
    Wf = {k: np.asarray(v, dtype=np.float64) for k, v in W.items()}
    z = RNG.normal(size=hc.d_cond)
    x_t = RNG.normal(size=D)
    t = 0.6

    def mv(vec, M, b):                                               # vec @ M + b by loops
        return [sum(float(vec[k]) * float(M[k][j]) for k in range(len(vec))) + float(b[j]) for j in range(len(b))]

    def silu(v):
        return [a / (1.0 + math.exp(-a)) for a in v]

    def ln(v):
        m = sum(v) / len(v)
        var = sum((a - m) ** 2 for a in v) / len(v)
        return [(a - m) / math.sqrt(var + 1e-6) for a in v]

    def by_hand(use_silu=True, use_temb=True, order=(0, 1, 2)):
        half = hc.t_freq_dim // 2
        om = [10000.0 ** (-k / half) for k in range(half)]
        feat = [math.cos(t * hc.t_scale * o) for o in om] + [math.sin(t * hc.t_scale * o) for o in om]
        temb = mv(silu(mv(feat, Wf["head.t1.w"], Wf["head.t1.b"])), Wf["head.t2.w"], Wf["head.t2.b"])
        c = mv(z, Wf["head.c.w"], Wf["head.c.b"])
        if use_temb:
            c = [a + b for a, b in zip(c, temb)]
        sc = silu(c) if use_silu else c
        h = mv(x_t, Wf["head.in.w"], Wf["head.in.b"])
        mod = mv(sc, Wf["head.B0.mod.w"], Wf["head.B0.mod.b"])
        parts = [mod[0:w], mod[w:2 * w], mod[2 * w:3 * w]]
        shift, scale, gate = parts[order[0]], parts[order[1]], parts[order[2]]
        a = [n_ * (1.0 + s) + sh for n_, s, sh in zip(ln(h), scale, shift)]
        a = silu(mv(a, Wf["head.B0.w1"], Wf["head.B0.b1"]))
        br = mv(a, Wf["head.B0.w2"], Wf["head.B0.b2"])
        h = [hv + g * b for hv, g, b in zip(h, gate, br)]
        fm = mv(sc, Wf["head.f.mod.w"], Wf["head.f.mod.b"])
        a = [n_ * (1.0 + s) + sh for n_, s, sh in zip(ln(h), fm[w:2 * w], fm[0:w])]
        return np.array(mv(a, Wf["head.out.w"], Wf["head.out.b"]))

    want = by_hand()
    got = hd.velocity(hc, W, x_t[None, :], t, z[None, :])[0]
    assert np.allclose(got, want, rtol=1e-11, atol=1e-13)
    # the planted mistakes are visible at this size
    for kw in (dict(use_silu=False), dict(use_temb=False), dict(order=(1, 0, 2)), dict(order=(0, 2, 1))):
        assert np.abs(by_hand(**kw) - want).max() > 1e-3, kw
    # and z really drives the modulation: another z, another velocity
    got2 = hd.velocity(hc, W, x_t[None, :], t, (z + 1.0)[None, :])[0]
    assert np.abs(got2 - got).max() > 1e-3
