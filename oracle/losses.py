"""Training-side losses of the draft model (test infrastructure): the attention-entropy loss and the feature
regression loss, each with its gradient.

Sec. 3 (entropy-informed speculative decoding), Eq. for L_entropy, and S2.1: for the softmax-normalised rows
Omega_r of the penultimate layer's attention map,
    L_entropy = 1 / (R * N) * sum_heads sum_r sum_c Omega_{r,c} ln Omega_{r,c}        (= - mean row entropy),
here also averaged over the batch.  The attention map is that of the causal AR body (Sec. 3.1): row r sees
columns 0..r, scores s_{r,c} = q_r . k_c / sqrt(d_head); with grouped heads, query head h reads kv head h // G.
The gradient is written out from the definition: with H_r = -sum_c Omega ln Omega,
    dH_r / ds_{r,c} = -Omega_{r,c} (ln Omega_{r,c} + H_r),
    dL/ds = -dH/ds / (B N R),   dL/dq_r = sum_c dL/ds_{r,c} k_c / sqrt(d),   dL/dk_c = sum_r dL/ds_{r,c} q_r / sqrt(d).

Feature regression (the Smooth-L1 L_reg the method keeps from EAGLE): mean over elements of
    0.5 d^2 / beta  for |d| < beta,   |d| - 0.5 beta  otherwise,     d = pred - target.
"""
from __future__ import annotations

import numpy as np


def attn_entropy_loss(q, k):
    """q: [B, H, R, dh], k: [B, Hkv, R, dh].  Returns loss, H_rows [B, H, R], dq (like q), dk (like k)."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    B, H, R, dh = q.shape
    Hkv = k.shape[1]
    G = H // Hkv
    scale = 1.0 / np.sqrt(dh)
    H_rows = np.zeros((B, H, R))
    dq = np.zeros_like(q)
    dk = np.zeros_like(k)
    c = 1.0 / (B * H * R)
    causal = np.tril(np.ones((R, R), dtype=bool))
    for b in range(B):
        for h in range(H):
            kk = k[b, h // G]
            s = (q[b, h] @ kk.T) * scale
            s = np.where(causal, s, -np.inf)
            m = s.max(axis=1, keepdims=True)
            e = np.exp(s - m)
            l = e.sum(axis=1, keepdims=True)
            p = e / l
            logp = np.where(causal, (s - m) - np.log(l), 0.0)
            Hr = -(p * logp).sum(axis=1)
            H_rows[b, h] = Hr
            ds = c * p * (logp + Hr[:, None])            # dL/ds, L = -mean H
            dq[b, h] = (ds @ kk) * scale
            dk[b, h // G] += (ds.T @ q[b, h]) * scale
    return -H_rows.mean(), H_rows, dq, dk


def smooth_l1(pred, target, beta=1.0):
    """Returns loss (mean over elements) and dloss/dpred."""
    d = np.asarray(pred, dtype=np.float64) - np.asarray(target, dtype=np.float64)
    a = np.abs(d)
    per = np.where(a < beta, 0.5 * d * d / beta, a - 0.5 * beta)
    g = np.where(a < beta, d / beta, np.sign(d)) / d.size
    return per.mean(), g
