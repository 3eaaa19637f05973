"""Pre-norm causal transformer forward with a KV cache, float64 (test infrastructure).

The paper treats the AR transformer as a black box z = ART(x_{1:i-1}, c) (Sec. 3.2)
that is evaluated in parallel over len+1 positions during verification (Alg. 1,
Step 2) and one position at a time while drafting (Alg. 1, Step 1), under the
causal factorisation of Sec. 3.1.  Its internals here are the standard ones fixed
by the benchmark configurations: pre-norm blocks, LayerNorm/GELU/learned positions
or RMSNorm/SwiGLU/RoPE/grouped KV heads.

One sample at a time, one layer at a time, one head at a time: no blocking, no
fusion.  A cached forward must equal a full recompute; tests check that.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import erf

ACT_GELU, ACT_SWIGLU = 0, 1
NORM_LAYER, NORM_RMS = 0, 1
POS_LEARNED, POS_ROPE = 0, 1


def f64(x):
    return np.asarray(x, dtype=np.float64)


def layer_norm(u, g, b, eps):
    mean = u.mean(axis=-1, keepdims=True)
    var = ((u - mean) ** 2).mean(axis=-1, keepdims=True)
    y = (u - mean) / np.sqrt(var + eps) * g
    return y + b if b is not None else y


def rms_norm(u, g, eps):
    ms = (u ** 2).mean(axis=-1, keepdims=True)
    return u / np.sqrt(ms + eps) * g


def gelu_erf(x):
    return 0.5 * x * (1.0 + erf(x / math.sqrt(2.0)))


def silu(x):
    return x / (1.0 + np.exp(-x))


def rope(x, pos, theta):
    """x: [n, d_head]; rotate-half pairing (c, c + d_head/2); pos: [n] absolute positions."""
    n, dh = x.shape
    half = dh // 2
    c = np.arange(half, dtype=np.float64)
    inv = theta ** (-2.0 * c / dh)
    ang = f64(pos)[:, None] * inv[None, :]
    cs, sn = np.cos(ang), np.sin(ang)
    a, b = x[:, :half], x[:, half:]
    return np.concatenate([a * cs - b * sn, b * cs + a * sn], axis=1)


def softmax_rows(s):
    m = s.max(axis=-1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=-1, keepdims=True)


def row_entropy(p):
    """-sum p ln p with 0 ln 0 = 0 (natural log)."""
    q = np.where(p > 0, p, 1.0)
    return -(p * np.log(q)).sum(axis=-1)


class KVCache:
    """Per layer, per sample: K and V of the tokens seen so far, [H_kv, len, d_head]."""

    def __init__(self, cfg, B):
        self.cfg = cfg
        self.B = B
        z = lambda: np.zeros((cfg.n_kv_heads, 0, cfg.d_head))
        self.k = [[z() for _ in range(B)] for _ in range(cfg.n_layers)]
        self.v = [[z() for _ in range(B)] for _ in range(cfg.n_layers)]

    def length(self, b):
        return self.k[0][b].shape[1]

    def load(self, layer, k, v):
        """k, v: [B, H_kv, n, d_head]; replaces the layer's content."""
        for b in range(self.B):
            self.k[layer][b] = f64(k[b]).copy()
            self.v[layer][b] = f64(v[b]).copy()

    def truncate(self, b, n):
        for l in range(self.cfg.n_layers):
            self.k[l][b] = self.k[l][b][:, :n]
            self.v[l][b] = self.v[l][b][:, :n]


def _norm(cfg, W, name, u):
    g = f64(W[name + ".g"])
    if cfg.norm == NORM_LAYER:
        return layer_norm(u, g, f64(W[name + ".b"]), cfg.norm_eps)
    return rms_norm(u, g, cfg.norm_eps)


def forward_sample(cfg, W, prefix, cache, b, x, ids=None, commit=True, shallow_layer=None):
    """One sample.  x: [n_q, D] latent rows, ids: [n_q] ints (-1 = latent row) or None.

    Row j sits at position cache_len + j and attends to every cached token and to
    rows 0..j of this call.  Returns z [n_q, d_out], the residual stream after layer
    `shallow_layer` (1-indexed) and the head-averaged attention-row entropy there.
    """
    P = lambda n: W[f"{prefix}.{n}"]
    H, Hk, dh, d = cfg.n_heads, cfg.n_kv_heads, cfg.d_head, cfg.d_model
    x = f64(x)
    n_q = x.shape[0]
    p0 = cache.length(b)
    pos = p0 + np.arange(n_q)

    h = x @ f64(P("in.w")) + f64(P("in.b"))
    if cfg.pos == POS_LEARNED:
        h = h + f64(P("pos"))[pos]
    if ids is not None:
        for j in range(n_q):
            if ids[j] >= 0:
                h[j] = f64(P("cond"))[ids[j]]

    shallow, h_attn = None, None
    for l in range(cfg.n_layers):
        L = f"L{l}."
        u = _norm(cfg, _View(W, prefix), L + "n1", h)
        qkv = u @ f64(P(L + "wqkv"))
        if cfg.has_bias:
            qkv = qkv + f64(P(L + "bqkv"))
        q = qkv[:, :H * dh].reshape(n_q, H, dh)
        k = qkv[:, H * dh:(H + Hk) * dh].reshape(n_q, Hk, dh)
        v = qkv[:, (H + Hk) * dh:].reshape(n_q, Hk, dh)
        if cfg.pos == POS_ROPE:
            q = np.stack([rope(q[:, g], pos, cfg.rope_theta) for g in range(H)], axis=1)
            k = np.stack([rope(k[:, g], pos, cfg.rope_theta) for g in range(Hk)], axis=1)
        K_all = np.concatenate([cache.k[l][b], k.transpose(1, 0, 2)], axis=1)   # [Hk, p0+n_q, dh]
        V_all = np.concatenate([cache.v[l][b], v.transpose(1, 0, 2)], axis=1)
        if commit:
            cache.k[l][b], cache.v[l][b] = K_all, V_all

        o = np.zeros((n_q, H, dh))
        ent = np.zeros((n_q, H))
        for g in range(H):
            kv = (g * Hk) // H
            for j in range(n_q):
                vis = p0 + j + 1                      # keys c <= p_j
                s = (K_all[kv, :vis] @ q[j, g]) / math.sqrt(dh)
                om = softmax_rows(s[None, :])[0]
                o[j, g] = om @ V_all[kv, :vis]
                ent[j, g] = row_entropy(om)
        att = o.reshape(n_q, H * dh) @ f64(P(L + "wo"))
        if cfg.has_bias:
            att = att + f64(P(L + "bo"))
        h = h + att

        u = _norm(cfg, _View(W, prefix), L + "n2", h)
        if cfg.act == ACT_GELU:
            a = u @ f64(P(L + "w1"))
            if cfg.has_bias:
                a = a + f64(P(L + "b1"))
            m = gelu_erf(a) @ f64(P(L + "w2"))
            if cfg.has_bias:
                m = m + f64(P(L + "b2"))
        else:
            m = (silu(u @ f64(P(L + "wg"))) * (u @ f64(P(L + "wu")))) @ f64(P(L + "wd"))
        h = h + m

        if shallow_layer is not None and l + 1 == shallow_layer:
            shallow = h.copy()
            h_attn = ent.mean(axis=1)

    z = _norm(cfg, _View(W, prefix), "nf", h)
    if cfg.d_out and cfg.d_out != cfg.d_model:
        z = z @ f64(P("up.w"))
    return z, shallow, h_attn


class _View:
    """Prefix-stripped read-only view of a weight dict."""

    def __init__(self, W, prefix):
        self.W, self.prefix = W, prefix

    def __getitem__(self, name):
        return self.W[f"{self.prefix}.{name}"]


def forward(cfg, W, prefix, cache, xs, ids=None, commit=True, shallow_layer=None):
    """Batch wrapper: xs is a list (one [n_q_b, D] array per sample; n_q_b may be 0)."""
    zs, shs, hs = [], [], []
    for b, x in enumerate(xs):
        if len(x) == 0:
            zs.append(np.zeros((0, cfg.d_out or cfg.d_model)))
            shs.append(np.zeros((0, cfg.d_model)))
            hs.append(np.zeros((0,)))
            continue
        z, sh, ha = forward_sample(cfg, W, prefix, cache, b, x, None if ids is None else ids[b],
                                   commit=commit, shallow_layer=shallow_layer)
        zs.append(z)
        shs.append(sh)
        hs.append(ha)
    return zs, shs, hs
