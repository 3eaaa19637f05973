"""Brute-force counterparts used only to pin the vectorised oracle (test infrastructure).

Pure-Python loops for tiny inputs, and a cache-free transformer forward that
recomputes the whole sequence with an explicit causal mask.
"""
from __future__ import annotations

import math

import numpy as np

from . import transformer as tf


def matmul_loops(a, b):
    n, k = len(a), len(a[0])
    m = len(b[0])
    out = [[0.0] * m for _ in range(n)]
    for i in range(n):
        for j in range(m):
            s = 0.0
            for t in range(k):
                s += float(a[i][t]) * float(b[t][j])
            out[i][j] = s
    return out


def causal_attention_loops(q, k, v):
    """q, k, v: [n, d] nested lists / arrays, one head, row i sees keys 0..i."""
    n, d = len(q), len(q[0])
    out = [[0.0] * d for _ in range(n)]
    probs = []
    for i in range(n):
        s = []
        for c in range(i + 1):
            acc = 0.0
            for t in range(d):
                acc += float(q[i][t]) * float(k[c][t])
            s.append(acc / math.sqrt(d))
        m = max(s)
        e = [math.exp(val - m) for val in s]
        z = sum(e)
        p = [val / z for val in e]
        probs.append(p)
        for t in range(d):
            acc = 0.0
            for c in range(i + 1):
                acc += p[c] * float(v[c][t])
            out[i][t] = acc
    return out, probs


def entropy_loops(row):
    m = max(row)
    e = [math.exp(float(x) - m) for x in row]
    z = sum(e)
    h = 0.0
    for val in e:
        p = val / z
        if p > 0.0:
            h -= p * math.log(p)
    return h


def leading_run(flags, limit):
    n = 0
    for i in range(limit):
        if not flags[i]:
            break
        n += 1
    return n


def full_recompute(cfg, W, prefix, x, ids=None, shallow_layer=None):
    """Whole sequence at once, no cache: matrix-form causal attention with a -inf mask.
    x: [n, D].  Returns z [n, d_out], shallow [n, d], attention-row entropies [n]."""
    P = lambda name: np.asarray(W[f"{prefix}.{name}"], dtype=np.float64)
    H, Hk, dh = cfg.n_heads, cfg.n_kv_heads, cfg.d_head
    x = np.asarray(x, dtype=np.float64)
    n = x.shape[0]
    pos = np.arange(n)
    h = x @ P("in.w") + P("in.b")
    if cfg.pos == tf.POS_LEARNED:
        h = h + P("pos")[:n]
    if ids is not None:
        for j in range(n):
            if ids[j] >= 0:
                h[j] = P("cond")[ids[j]]
    mask = np.triu(np.ones((n, n), dtype=bool), k=1)
    shallow, h_attn = None, None

    def norm(name, u):
        if cfg.norm == tf.NORM_LAYER:
            return tf.layer_norm(u, P(name + ".g"), P(name + ".b"), cfg.norm_eps)
        return tf.rms_norm(u, P(name + ".g"), cfg.norm_eps)

    for l in range(cfg.n_layers):
        L = f"L{l}."
        u = norm(L + "n1", h)
        qkv = u @ P(L + "wqkv")
        if cfg.has_bias:
            qkv = qkv + P(L + "bqkv")
        q = qkv[:, :H * dh].reshape(n, H, dh)
        k = qkv[:, H * dh:(H + Hk) * dh].reshape(n, Hk, dh)
        v = qkv[:, (H + Hk) * dh:].reshape(n, Hk, dh)
        if cfg.pos == tf.POS_ROPE:
            q = np.stack([tf.rope(q[:, g], pos, cfg.rope_theta) for g in range(H)], axis=1)
            k = np.stack([tf.rope(k[:, g], pos, cfg.rope_theta) for g in range(Hk)], axis=1)
        o = np.zeros((n, H, dh))
        ent = np.zeros((n, H))
        for g in range(H):
            kv = (g * Hk) // H
            s = q[:, g] @ k[:, kv].T / math.sqrt(dh)
            s = np.where(mask, -np.inf, s)
            p = tf.softmax_rows(s)
            o[:, g] = p @ v[:, kv]
            ent[:, g] = tf.row_entropy(p)
        att = o.reshape(n, H * dh) @ P(L + "wo")
        if cfg.has_bias:
            att = att + P(L + "bo")
        h = h + att
        u = norm(L + "n2", h)
        if cfg.act == tf.ACT_GELU:
            a = u @ P(L + "w1")
            if cfg.has_bias:
                a = a + P(L + "b1")
            m = tf.gelu_erf(a) @ P(L + "w2")
            if cfg.has_bias:
                m = m + P(L + "b2")
        else:
            m = (tf.silu(u @ P(L + "wg")) * (u @ P(L + "wu"))) @ P(L + "wd")
        h = h + m
        if shallow_layer is not None and l + 1 == shallow_layer:
            shallow, h_attn = h.copy(), ent.mean(axis=1)
    z = norm("nf", h)
    if cfg.d_out and cfg.d_out != cfg.d_model:
        z = z @ P("up.w")
    return z, shallow, h_attn
