"""Pins for oracle/resample.py (Alg. 1 Step 5, S3 item 3; multi-round generation)."""
import math

import numpy as np
import pytest
from scipy.stats import norm as gauss, kstest

from oracle import accept as ac
from oracle import resample as rs
from oracle import round as rnd
from oracle import transformer as tf
from synth import gen
from tests.test_oracle_head_accept_round import _round_setup

RNG = np.random.default_rng(2024)


def test_alpha_closed_forms():
    """alpha = max(0, 1 - q/(Sigma p)): 0 where the draft density dominates, -> 1 far on the target's side, and
    the hand-computed value at a 1-D point."""
    s = 0.5
    mu_p, mu_q = np.array([0.3]), np.array([-0.2])
    assert rs.residual_accept_prob(np.array([-0.5]), mu_p, mu_q, 0.0, s, s) == 0.0        # q > p left of the midpoint
    assert rs.residual_accept_prob(np.array([0.05]), mu_p, mu_q, 0.0, s, s) == pytest.approx(0.0, abs=1e-12)  # midpoint
    assert rs.residual_accept_prob(np.array([9.0]), mu_p, mu_q, 0.0, s, s) > 1 - 1e-6
    x = 0.7
    want = 1.0 - gauss.pdf(x, -0.2, s) / gauss.pdf(x, 0.3, s)
    assert rs.residual_accept_prob(np.array([x]), mu_p, mu_q, 0.0, s, s) == pytest.approx(want, rel=1e-12)
    # Sigma scales the target density
    want2 = 1.0 - gauss.pdf(x, -0.2, s) / (math.exp(0.4) * gauss.pdf(x, 0.3, s))
    assert rs.residual_accept_prob(np.array([x]), mu_p, mu_q, 0.4, s, s) == pytest.approx(want2, rel=1e-12)


def test_tries_follow_the_geometric_law_of_the_residual_mass():
    """Equal-sigma Gaussians: a proposal x ~ p is accepted with probability Z = int max(0, p - q) = 2 Phi(|d|/2s) - 1,
    so the number of proposals is geometric with mean 1/Z."""
    n, D, s, J = 20_000, 3, 0.25, 400
    delta = np.array([0.2, -0.1, 0.15])
    Z = 2 * gauss.cdf(np.linalg.norm(delta) / (2 * s)) - 1
    tries = np.empty(n)
    for i in range(n):
        _, tries[i] = rs.resample_one(delta, np.zeros(D), RNG.normal(size=(J, D)), RNG.random(J), 0.0, s, s)
    assert tries.max() < J
    se = math.sqrt((1 - Z) / Z ** 2 / n)
    assert abs(tries.mean() - 1 / Z) < 4 * se
    assert abs((tries == 1).mean() - Z) < 4 * math.sqrt(Z * (1 - Z) / n)


def test_accept_or_resample_reproduces_the_target_distribution():
    """The point of S3 item 3: a draft x ~ q kept when r <= p/q, otherwise replaced by a residual sample, is
    distributed as p.  1-D, unequal means and variances, Sigma from the variance ratio convention."""
    n, J = 60_000, 64
    mu_p, mu_q, sp, sq = 0.4, -0.1, 0.30, 0.45
    x = mu_q + sq * RNG.normal(size=(n, 1, 1))
    r = RNG.random((n, 1))
    mp = np.full((n, 2, 1), mu_p)
    mq = np.full((n, 1, 1), mu_q)
    n_acc, _, _ = ac.accept(x, mp, mq, r, np.ones(n, int), 0.0, sp, sq)
    out = np.empty(n)
    exhausted = 0
    for i in range(n):
        if n_acc[i] == 1:
            out[i] = x[i, 0, 0]
        else:
            xi, t = rs.resample_one(np.array([mu_p]), np.array([mu_q]), RNG.normal(size=(J, 1)), RNG.random(J), 0.0, sp, sq)
            out[i] = xi[0]
            exhausted += t == J
    assert exhausted < 5
    assert 0.2 < n_acc.mean() < 0.95                         # both branches are exercised
    assert kstest(out, "norm", args=(mu_p, sp)).pvalue > 1e-3
    assert abs(out.mean() - mu_p) < 4 * sp / math.sqrt(n)
    assert abs(out.std() - sp) < 0.01
    # a swapped ratio (keeping the draft when r <= q/p and sampling max(0, q - p)) would centre the output elsewhere
    assert abs(out.mean() - mu_q) > 0.3


def test_exhausted_loop_returns_the_last_proposal():
    mu = np.zeros(2)
    eps = RNG.normal(size=(5, 2))
    x, t = rs.resample_one(mu, mu, eps, np.full(5, 0.5), 0.0, 0.3, 0.3)      # p == q: alpha = 0 everywhere
    assert t == 5 and np.allclose(x, 0.3 * eps[-1])
    x, t = rs.resample_one(mu, mu + 50.0, eps, np.full(5, 0.5), 0.0, 0.3, 0.3)   # q far away: alpha ~ 1 at once
    assert t == 1 and np.allclose(x, 0.3 * eps[0])


def test_next_token_branches():
    B, K, D, J = 4, 3, 2, 6
    mu_p, mu_q = RNG.normal(size=(B, K + 1, D)), RNG.normal(size=(B, K, D)) + 30.0
    eps_last, eps_res, u = RNG.normal(size=(B, K + 1, D)), RNG.normal(size=(B, J, D)), RNG.random((B, J))
    n_keep = np.array([3, 3, 2, 0])
    n_acc = np.array([3, 1, 2, 0])
    x, tries = rs.next_token(n_acc, n_keep, mu_p, mu_q, eps_last, eps_res, u, 0.0, 0.5, 0.5)
    assert np.allclose(x[0], mu_p[0, 3] + 0.5 * eps_last[0, 3]) and tries[0] == 0      # all accepted: bonus row K
    assert np.allclose(x[1], mu_p[1, 1] + 0.5 * eps_res[1, 0]) and tries[1] == 1      # rejected at draft 2: row 1
    assert np.allclose(x[2], mu_p[2, 2] + 0.5 * eps_last[2, 2]) and tries[2] == 0      # early stop, both kept accepted
    assert np.allclose(x[3], mu_p[3, 0] + 0.5 * eps_last[3, 0]) and tries[3] == 0      # nothing drafted: plain AR step


def _gen_inputs(rc, B, R, J, seed):
    D, K, S = rc.target.d_latent, rc.K, rc.head.n_steps
    return dict(eps=[gen.noise(seed, f"g.eps{t}", (S + 1, B, K + 1, D)) for t in range(R)],
                r=[gen.uniforms(seed, f"g.r{t}", (B, K)) for t in range(R)],
                eps_res=[gen.noise(seed, f"g.er{t}", (B, J, D)) for t in range(R)],
                u_res=[gen.uniforms(seed, f"g.ur{t}", (B, J)) for t in range(R)])


def test_generate_bookkeeping_and_cache_lengths():
    rc, W, tc, dc, inp, B = _round_setup()
    R, J = 3, 8
    g = _gen_inputs(rc, B, R, J, 5)
    toks, rounds = rs.generate(rc, W, tc, dc, inp["pending"], g["eps"], g["r"], g["eps_res"], g["u_res"], -1.0, B)
    for b in range(B):
        n = sum(int(rr["n_accept"][b]) + 1 for rr in rounds)
        assert toks[b].shape == (n, rc.target.d_latent)
        assert tc.length(b) == 5 + n                          # every generated token but the newest is cached, plus the first pending
        assert dc.length(b) == 5 + n
        # the closing token of round t is the pending token of round t+1, which the next verify reads first
        pos = 0
        for rr in rounds:
            k = int(rr["n_accept"][b])
            assert np.array_equal(toks[b][pos:pos + k], rr["x"][b, :k])
            assert np.array_equal(toks[b][pos + k], rr["x_next"][b])
            pos += k + 1


def test_generate_with_draft_equal_to_target_accepts_every_round():
    """Shared noise + identical models: every round accepts all K drafts and ends with the bonus token; this holds
    in later rounds only if the draft cache was caught up with the K-th draft."""
    rc, W, tc, dc, inp, B = _round_setup(same=True)
    R, J = 3, 4
    g = _gen_inputs(rc, B, R, J, 6)
    toks, rounds = rs.generate(rc, W, tc, dc, inp["pending"], g["eps"], g["r"], g["eps_res"], g["u_res"], -1.0, B)
    for rr in rounds:
        assert np.array_equal(rr["n_accept"], np.full(B, rc.K))
        assert not rr["tries"].any()
        assert np.allclose(rr["log_ratio"], 0.0, atol=1e-6)
    # the same tokens come out of plain autoregressive decoding with the target alone (K = 0 drafts kept)
    rc2, W2, tc2, dc2, inp2, _ = _round_setup(same=True)
    n_tok = R * (rc.K + 1)
    ar = []
    pending = np.asarray(inp2["pending"], dtype=np.float64)
    t, j = 0, 0
    for i in range(n_tok):
        # token i is produced from the noise trajectory it has in the speculative run: round t, row j
        eps_t = g["eps"][t][:, :, j:j + 1]
        o = rnd.verify_stage(rc2, W2, tc2, pending, np.zeros((B, rc.K, rc.target.d_latent)), np.zeros((B, rc.K, rc.target.d_latent)),
                             np.zeros(B, dtype=np.int32), np.ones((B, rc.K)), np.concatenate([eps_t] * (rc.K + 1), axis=2),
                             0.0, 0.25, 0.25, B, commit=True)
        s = rc.head.sigma_last * rc.head.temperature
        pending = o["mu_p"][:, 0] + s * g["eps"][t][-1][:, j]
        ar.append(pending.copy())
        j += 1
        if j == rc.K + 1:
            t, j = t + 1, 0
    ar = np.stack(ar, axis=1)                                 # [B, n_tok, D]
    for b in range(B):
        assert np.allclose(toks[b], ar[b], rtol=1e-7, atol=1e-9)
