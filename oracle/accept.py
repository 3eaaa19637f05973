"""Continuous accept/reject test of Alg. 1, Steps 3-4 (test infrastructure).

S3 item 2: the density ratio is Sigma * p(x | x_1^p) / q(x | x_1^q) with
Sigma = prod_{t=2..T} sqrt(|Sigma_{q,t}| / |Sigma_{p,t}|).  With the last transition
of each sampler an isotropic Gaussian N(mu, sigma^2 I) (reading used by this build),
ln rho = ln Sigma + D ln(sigma_q / sigma_p) - |x - mu_p|^2 / (2 sigma_p^2)
                                            + |x - mu_q|^2 / (2 sigma_q^2).
Step 4: a draft is rejected when r_i > rho_i; n = number of leading accepted drafts.
"""
from __future__ import annotations

import numpy as np


def log_sigma_factor(sig_q, sig_p, D):
    """ln Sigma for per-step isotropic variances sigma_{.,t}^2 I_D, t = 2..T (empty -> 0)."""
    sq, sp = np.asarray(sig_q, dtype=np.float64), np.asarray(sig_p, dtype=np.float64)
    if sq.size == 0:
        return 0.0
    return float(D * np.sum(np.log(sq) - np.log(sp)))


def log_ratio(x, mu_p, mu_q, log_sigma, sigma_p, sigma_q):
    """x, mu_p, mu_q: [..., D] -> ln rho [...]."""
    x, mu_p, mu_q = (np.asarray(a, dtype=np.float64) for a in (x, mu_p, mu_q))
    D = x.shape[-1]
    dp = ((x - mu_p) ** 2).sum(axis=-1)
    dq = ((x - mu_q) ** 2).sum(axis=-1)
    return (log_sigma + D * (np.log(sigma_q) - np.log(sigma_p))
            - dp / (2.0 * sigma_p ** 2) + dq / (2.0 * sigma_q ** 2))


def accept(x, mu_p, mu_q, r, n_keep, log_sigma, sigma_p, sigma_q):
    """x, mu_q: [B, K, D] drafts and their draft-side means; mu_p: [B, K+1, D] target-side
    means (row i-1 is the target's mean for draft i); r: [B, K] uniforms; n_keep: [B].
    Returns n_accept [B] int32, ln rho [B, K], acc [B, K] uint8."""
    x = np.asarray(x, dtype=np.float64)
    B, K, _ = x.shape
    lr = log_ratio(x, np.asarray(mu_p, dtype=np.float64)[:, :K], mu_q, log_sigma, sigma_p, sigma_q)
    r = np.asarray(r, dtype=np.float64)
    with np.errstate(divide="ignore"):
        acc = (np.log(r) <= lr)
    n_acc = np.zeros(B, dtype=np.int32)
    for b in range(B):
        n = 0
        while n < n_keep[b] and acc[b, n]:
            n += 1
        n_acc[b] = n
    return n_acc, lr, acc.astype(np.uint8)
