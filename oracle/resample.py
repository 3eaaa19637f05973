"""Alg. 1 Step 5 and the token a round ends with; multi-round generation (test infrastructure).

S3 item 3 / Alg. 1 Step 5: when draft n+1 is the first rejected one, the token at that position
is drawn from the residual distribution max(0, Sigma p - q) / Z by acceptance-rejection with
proposals from the target's own distribution p_{n+1}:
    repeat  x ~ p_{n+1}(. | x_1^p);  alpha = max(0, Sigma p(x) - q(x)) / (Sigma p(x));  u ~ U(0,1)
    until u <= alpha.
With the isotropic Gaussians of the accept test (oracle/accept.py), q(x) / (Sigma p(x)) = 1 / rho(x),
so alpha(x) = max(0, 1 - exp(-ln rho(x))).

Readings used by this build (the paper leaves them open):
  * the loop is bounded: proposals j = 0 .. J-1 come from pre-drawn noise eps_res[j] and uniforms
    u_res[j]; if none is accepted the last proposal is the token (tries = J);
  * when every kept draft is accepted (n = len), the round ends with the target's own sample of
    row len under the shared noise, mu_p[len] + sigma_p * eps_last[len] (Alg. 1 Step 2 computes
    p_{len+1} for exactly this purpose); tries = 0;
  * a draft model that accepted all K drafts has not read draft K yet; it reads it before the
    next round starts (one extra single-row draft forward).
"""
from __future__ import annotations

import numpy as np

from . import accept as ac
from . import round as rnd
from . import transformer as tf


def residual_accept_prob(x, mu_p, mu_q, log_sigma, sigma_p, sigma_q):
    """alpha(x) = max(0, Sigma p(x) - q(x)) / (Sigma p(x)) for x [..., D] -> [...]."""
    lr = ac.log_ratio(x, mu_p, mu_q, log_sigma, sigma_p, sigma_q)      # ln (Sigma p / q)
    with np.errstate(over="ignore"):
        return np.maximum(0.0, 1.0 - np.exp(-lr))


def resample_one(mu_p, mu_q, eps_res, u_res, log_sigma, sigma_p, sigma_q):
    """One position.  mu_p, mu_q: [D]; eps_res: [J, D]; u_res: [J].  Returns (x [D], tries)."""
    mu_p = np.asarray(mu_p, dtype=np.float64)
    J = len(u_res)
    x = None
    for j in range(J):
        x = mu_p + sigma_p * np.asarray(eps_res[j], dtype=np.float64)
        a = residual_accept_prob(x, mu_p, mu_q, log_sigma, sigma_p, sigma_q)
        if float(u_res[j]) <= a:
            return x, j + 1
    return x, J


def next_token(n_accept, n_keep, mu_p, mu_q, eps_last, eps_res, u_res, log_sigma, sigma_p, sigma_q):
    """The token every sample's round ends with.
    n_accept, n_keep: [B]; mu_p: [B, K+1, D]; mu_q: [B, K, D]; eps_last: [B, K+1, D] (the shared noise of the
    last sampler transition); eps_res: [B, J, D]; u_res: [B, J].  Returns x_next [B, D], tries [B] int32."""
    B, _, D = np.asarray(mu_p).shape
    x_next = np.zeros((B, D))
    tries = np.zeros(B, dtype=np.int32)
    for b in range(B):
        n, nk = int(n_accept[b]), int(n_keep[b])
        if n < nk:
            x_next[b], tries[b] = resample_one(mu_p[b, n], mu_q[b, n], eps_res[b], u_res[b], log_sigma, sigma_p, sigma_q)
        else:
            x_next[b] = np.asarray(mu_p[b, nk], dtype=np.float64) + sigma_p * np.asarray(eps_last[b, nk], dtype=np.float64)
    return x_next, tries


def generate(rc, W, target_cache, draft_cache, x_first, eps_all, r_all, eps_res_all, u_res_all, tau, B,
             log_sigma=0.0, sigma_p=None, sigma_q=None):
    """R = len(eps_all) rounds in a row.  eps_all[t]: [S+1, B, K+1, D]; r_all[t]: [B, K]; eps_res_all[t]:
    [B, J, D]; u_res_all[t]: [B, J].  Returns tokens (list per sample of [n, D] arrays: the accepted drafts and
    the closing token of every round, in order) and per-round dicts (n_keep, n_accept, tries, H, x_next)."""
    s = rc.head.sigma_last * rc.head.temperature
    sigma_p = s if sigma_p is None else sigma_p
    sigma_q = s if sigma_q is None else sigma_q
    K = rc.K
    pending = np.asarray(x_first, dtype=np.float64).copy()
    tokens = [[] for _ in range(B)]
    rounds = []
    for t in range(len(eps_all)):
        o = rnd.spec_round(rc, W, target_cache, draft_cache, pending, eps_all[t], r_all[t], tau, B,
                           log_sigma=log_sigma, sigma_p=sigma_p, sigma_q=sigma_q)
        x_next, tries = next_token(o["n_accept"], o["n_keep"], o["mu_p"], o["mu_q"], eps_all[t][-1], eps_res_all[t],
                                   u_res_all[t], log_sigma, sigma_p, sigma_q)
        for b in range(B):
            n = int(o["n_accept"][b])
            for i in range(n):
                tokens[b].append(o["x"][b, i].copy())
            tokens[b].append(x_next[b].copy())
            if n == K:      # the draft has not read draft K yet
                tf.forward_sample(rc.draft, W, "draft", draft_cache, b, o["x"][b, K - 1][None, :], commit=True)
        rounds.append(dict(n_keep=o["n_keep"].copy(), n_accept=o["n_accept"].copy(), tries=tries, H=o["H"].copy(),
                           x_next=x_next.copy(), mu_p=o["mu_p"].copy(), mu_q=o["mu_q"].copy(), x=o["x"].copy(),
                           log_ratio=o["log_ratio"].copy()))
        pending = x_next
    return [np.stack(t) if t else np.zeros((0, pending.shape[1])) for t in tokens], rounds
