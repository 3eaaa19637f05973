"""Shallow-layer entropy indicator, threshold, prefix rule, survivor list (test infrastructure).

Eq. 1 and S2.1 define L_entropy as the mean over rows (and heads) of
sum_c Omega_{r,c} ln Omega_{r,c} for softmax-normalised rows Omega; the inference
indicator is H = -L_entropy (Alg. 1, Step 1), compared with tau_ent: a draft whose
H < tau_ent ends speculation for its sample and is dropped together with every
later draft of that sample.  The threshold follows Sec. 4.3:
tau = 0.3 * mean(H) - 0.1 * std(H) over a calibration set.

Two bindings of the same operator: FEATURE rows (the d channels of the draft's
layer-l_s output) and ATTN rows (attention rows of layer l_s, head-averaged;
computed in oracle/transformer.py from the softmax rows themselves).
"""
from __future__ import annotations

import numpy as np


def softmax_entropy(rows):
    """H(row) = -sum_c p_c ln p_c, p = softmax(row); rows: [..., L] -> [...]."""
    x = np.asarray(rows, dtype=np.float64)
    m = x.max(axis=-1, keepdims=True)
    e = np.exp(x - m)
    l = e.sum(axis=-1, keepdims=True)
    p = e / l
    logp = (x - m) - np.log(l)
    term = np.where(p > 0, p * logp, 0.0)
    return -term.sum(axis=-1)


def l_entropy(attn):
    """S2.1: attn [N_heads, R, C] of softmax rows -> 1/(R*N) sum_h sum_r sum_c Om ln Om (<= 0)."""
    a = np.asarray(attn, dtype=np.float64)
    t = np.where(a > 0, a * np.log(np.where(a > 0, a, 1.0)), 0.0)
    return t.sum() / (a.shape[0] * a.shape[1])


def threshold(H_cal):
    """tau = 0.3 * E[H] - 0.1 * std(H), population std (Sec. 4.3)."""
    h = np.asarray(H_cal, dtype=np.float64)
    return 0.3 * h.mean() - 0.1 * h.std()


def prefilter(H, tau):
    """H: [B, K].  raw = H >= tau; keep[b, i] = all(raw[b, :i+1]) (Alg. 1: the first
    low-entropy draft stops speculation and is dropped with everything after it).
    Returns keep [B,K] uint8, n_keep [B] int32, surv_idx (row-major flat indices b*K+i
    of kept drafts) int32, n_surv."""
    H = np.asarray(H, dtype=np.float64)
    B, K = H.shape
    keep = np.zeros((B, K), dtype=np.uint8)
    n_keep = np.zeros(B, dtype=np.int32)
    surv = []
    for b in range(B):
        alive = True
        for i in range(K):
            if alive and not (H[b, i] < tau):
                keep[b, i] = 1
                n_keep[b] += 1
                surv.append(b * K + i)
            else:
                alive = False
    return keep, n_keep, np.asarray(surv, dtype=np.int32), len(surv)


def online_entropy(row, splits):
    """Entropy of softmax(row) from blocks processed one after another with the running
    triple (m, l, a), a = sum e^{x-m} (x-m); H = ln l - a / l.  Used to check that a
    streaming evaluation equals the two-pass definition for any split."""
    row = np.asarray(row, dtype=np.float64)
    m, l, a = -np.inf, 0.0, 0.0
    start = 0
    for stop in list(splits) + [len(row)]:
        blk = row[start:stop]
        start = stop
        if len(blk) == 0:
            continue
        m_new = max(m, blk.max())
        if np.isfinite(m):
            delta = m - m_new
            a = np.exp(delta) * (a + delta * l)
            l = np.exp(delta) * l
        e = np.exp(blk - m_new)
        l += e.sum()
        a += (e * (blk - m_new)).sum()
        m = m_new
    return np.log(l) - a / l
