"""One entropy-informed speculative round, Alg. 1 Steps 1-4 (test infrastructure).

Order of operations per sample (Alg. 1): draft up to K tokens one at a time, stopping
at the first draft step whose shallow-layer entropy falls below tau_ent (that draft
and all later ones are dropped before they are decoded); verify the pending token
plus the K' surviving drafts in one target forward; decode the target-side means
with the same noise; accept the longest prefix whose uniforms stay below the ratio.
Step 5 (resampling) is outside this module.

Token bookkeeping: the caches hold every accepted token except the newest one,
the `pending` token.  Draft step i reads token i-1 (pending for i = 1) and produces
token i; verify row j reads token j and yields the target's distribution of token j+1.
eps[:, b, j] is the noise trajectory of token j+1, shared by both models.
"""
from __future__ import annotations

import numpy as np

from . import transformer as tf
from . import entropy as ent
from . import head as hd
from . import accept as ac

ENT_FEATURE, ENT_ATTN = 0, 1


def draft_stage(rc, W, draft_cache, pending, eps, tau, B):
    """Returns dict with H [B,K], keep [B,K], n_keep [B], x [B,K,D], mu_q [B,K,D],
    z_q (list per sample of [K'_b, d_out]) and the shallow features f [B,K,d]."""
    K, D = rc.K, rc.draft.d_latent
    H = np.zeros((B, K))
    keep = np.zeros((B, K), dtype=np.uint8)
    n_keep = np.zeros(B, dtype=np.int32)
    x = np.zeros((B, K, D))
    mu_q = np.zeros((B, K, D))
    feat = np.zeros((B, K, rc.draft.d_model))
    z_q = [[] for _ in range(B)]
    for b in range(B):
        tok = np.asarray(pending[b], dtype=np.float64)
        for i in range(K):
            z, sh, ha = tf.forward_sample(rc.draft, W, "draft", draft_cache, b, tok[None, :],
                                          commit=True, shallow_layer=rc.entropy_layer)
            feat[b, i] = sh[0]
            H[b, i] = ent.softmax_entropy(sh[0]) if rc.entropy_mode == ENT_FEATURE else ha[0]
            if H[b, i] < tau:
                break
            keep[b, i] = 1
            n_keep[b] += 1
            mu, xi = hd.decode(rc.head, W, z, eps[:, b, i][:, None, :])
            mu_q[b, i], x[b, i] = mu[0], xi[0]
            z_q[b].append(z[0])
            tok = xi[0]
    return dict(H=H, keep=keep, n_keep=n_keep, x=x, mu_q=mu_q, z_q=z_q, feat=feat)


def verify_stage(rc, W, target_cache, pending, x, mu_q, n_keep, r, eps,
                 log_sigma, sigma_p, sigma_q, B, commit=False):
    """Target forward over [pending, x_1..x_K'] per sample, head on all K'+1 rows with the
    shared noise, accept test.  Returns n_accept, ln rho, acc, mu_p [B,K+1,D], z_p (list)."""
    K, D = rc.K, rc.target.d_latent
    xs = []
    for b in range(B):
        rows = [np.asarray(pending[b], dtype=np.float64)] + [x[b, i] for i in range(n_keep[b])]
        xs.append(np.stack(rows))
    z_p, _, _ = tf.forward(rc.target, W, "target", target_cache, xs, commit=commit)
    mu_p = np.zeros((B, K + 1, D))
    for b in range(B):
        n_q = n_keep[b] + 1
        mu, _ = hd.decode(rc.head, W, z_p[b], eps[:, b, :n_q])
        mu_p[b, :n_q] = mu
    n_acc, lr, acc = ac.accept(x, mu_p, mu_q, r, n_keep, log_sigma, sigma_p, sigma_q)
    return dict(n_accept=n_acc, log_ratio=lr, acc=acc, mu_p=mu_p, z_p=z_p)


def spec_round(rc, W, target_cache, draft_cache, pending, eps, r, tau, B,
               log_sigma=0.0, sigma_p=None, sigma_q=None):
    """Draft + verify + accept, then roll both caches back to the accepted length."""
    s = rc.head.sigma_last * rc.head.temperature
    sigma_p = s if sigma_p is None else sigma_p
    sigma_q = s if sigma_q is None else sigma_q
    len0_t = [target_cache.length(b) for b in range(B)]
    len0_d = [draft_cache.length(b) for b in range(B)]
    d = draft_stage(rc, W, draft_cache, pending, eps, tau, B)
    v = verify_stage(rc, W, target_cache, pending, d["x"], d["mu_q"], d["n_keep"], r, eps,
                     log_sigma, sigma_p, sigma_q, B, commit=True)
    for b in range(B):
        target_cache.truncate(b, len0_t[b] + 1 + int(v["n_accept"][b]))
        draft_cache.truncate(b, min(draft_cache.length(b), len0_d[b] + 1 + int(v["n_accept"][b])))
    out = dict(d)
    out.update(v)
    return out
