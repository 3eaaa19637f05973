"""Few-step diffusion/flow head: AdaLN residual MLP plus its sampler, float64 (test infrastructure).

The paper writes the head as x_0 = Diff_theta(x_t | t, z) conditioned on the AR
feature z (Sec. 3.2), MLP-based for MAR / NextStep-1 (Sec. 5.1), run for very few
steps after distillation (Sec. 4.2), with the per-step Gaussian noise shared by
draft and target (S3 item 1; Alg. 1 initialisation).  Its internals are not given;
this is the reading used by this build: rectified-flow convention
x_t = (1 - t) x_0 + t eps, network output v = eps - x_0, AdaLN-modulated residual
blocks.
"""
from __future__ import annotations

import numpy as np

LN_EPS = 1e-6


def f64(x):
    return np.asarray(x, dtype=np.float64)


def silu(x):
    return x / (1.0 + np.exp(-x))


def ln_plain(h):
    mean = h.mean(axis=-1, keepdims=True)
    var = ((h - mean) ** 2).mean(axis=-1, keepdims=True)
    return (h - mean) / np.sqrt(var + LN_EPS)


def time_embedding(hc, W, t):
    """temb(t) = W_t2 SiLU(W_t1 [cos(t s w), sin(t s w)] + b_t1) + b_t2, w_k = 10000^(-k/half)."""
    half = hc.t_freq_dim // 2
    k = np.arange(half, dtype=np.float64)
    omega = 10000.0 ** (-k / half)
    arg = t * hc.t_scale * omega
    feat = np.concatenate([np.cos(arg), np.sin(arg)])
    a = silu(feat @ f64(W["head.t1.w"]) + f64(W["head.t1.b"]))
    return a @ f64(W["head.t2.w"]) + f64(W["head.t2.b"])


def velocity(hc, W, x_t, t, z):
    """v = head(x_t, t, z); x_t: [n, D], z: [n, d_cond] -> [n, D]."""
    w = hc.width
    c = f64(z) @ f64(W["head.c.w"]) + f64(W["head.c.b"]) + time_embedding(hc, W, t)
    sc = silu(c)
    h = f64(x_t) @ f64(W["head.in.w"]) + f64(W["head.in.b"])
    for j in range(hc.n_blocks):
        p = f"head.B{j}."
        mod = sc @ f64(W[p + "mod.w"]) + f64(W[p + "mod.b"])
        shift, scale, gate = mod[:, :w], mod[:, w:2 * w], mod[:, 2 * w:]
        a = ln_plain(h) * (1.0 + scale) + shift
        a = silu(a @ f64(W[p + "w1"]) + f64(W[p + "b1"]))
        h = h + gate * (a @ f64(W[p + "w2"]) + f64(W[p + "b2"]))
    mod = sc @ f64(W["head.f.mod.w"]) + f64(W["head.f.mod.b"])
    shift, scale = mod[:, :w], mod[:, w:]
    a = ln_plain(h) * (1.0 + scale) + shift
    return a @ f64(W["head.out.w"]) + f64(W["head.out.b"])


def decode(hc, W, z, eps):
    """S-step sampler.  z: [n, d_cond]; eps: [S+1, n, D] (eps[0] start noise, eps[k] the
    fresh noise of step k when renoise=1, eps[S] the noise of the last, stochastic
    transition).  Returns (mu, x): mu = final x0 estimate, x = mu + sigma_last*temp*eps[S]."""
    S = hc.n_steps
    eps = f64(eps)
    x_t = eps[0] * hc.temperature
    x0 = None
    for k in range(S):
        t = 1.0 - k / S
        v = velocity(hc, W, x_t, t, z)
        x0 = x_t - t * v
        if k < S - 1:
            t_next = 1.0 - (k + 1) / S
            e = eps[k + 1] if hc.renoise else x_t + (1.0 - t) * v
            x_t = (1.0 - t_next) * x0 + t_next * e
    mu = x0
    x = mu + hc.sigma_last * hc.temperature * eps[S]
    return mu, x
