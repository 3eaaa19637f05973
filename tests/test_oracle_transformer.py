"""Pins for oracle/transformer.py: brute force, cached == recompute, causality, closed-form
special cases (Sec. 3.1 causal factorisation; Alg. 1 Step 2 parallel verification)."""
import math

import numpy as np
import pytest

from oracle import transformer as tf
from oracle import loops
from synth import gen
from synth.configs import TfCfg, ACT_GELU, ACT_SWIGLU, NORM_LAYER, NORM_RMS, POS_LEARNED, POS_ROPE, DT_F32

RNG = np.random.default_rng(7)


def tiny(kind="ln", L=2):
    if kind == "ln":
        return TfCfg(n_layers=L, d_model=16, n_heads=2, n_kv_heads=2, d_head=8, d_ff=24, act=ACT_GELU,
                     norm=NORM_LAYER, pos=POS_LEARNED, has_bias=1, d_latent=4, n_cond_ids=5, max_pos=32)
    return TfCfg(n_layers=L, d_model=32, n_heads=4, n_kv_heads=2, d_head=8, d_ff=24, act=ACT_SWIGLU,
                 norm=NORM_RMS, pos=POS_ROPE, has_bias=0, norm_eps=1e-6, d_latent=4, d_out=20)


def weights(cfg, seed=0, std=0.3):
    return gen.tf_weights(cfg, seed, "m", DT_F32, w_std=std, affine=True)


# ----------------------------------------------------------------------------- primitives
def test_matmul_matches_triple_loop():
    a, b = RNG.normal(size=(5, 7)), RNG.normal(size=(7, 3))
    assert np.allclose(a @ b, np.array(loops.matmul_loops(a.tolist(), b.tolist())), rtol=1e-13, atol=1e-13)


def test_layer_norm_statistics():
    u = RNG.normal(size=(6, 64)) * 3 + 5
    y = tf.layer_norm(u, np.ones(64), np.zeros(64), 0.0)
    assert np.allclose(y.mean(-1), 0, atol=1e-12) and np.allclose(y.var(-1), 1, atol=1e-12)
    g, b = RNG.normal(size=64), RNG.normal(size=64)
    assert np.allclose(tf.layer_norm(u, g, b, 0.0), y * g + b)
    # eps enters under the square root next to the variance
    c = np.array([[1.0, -1.0]])
    assert np.allclose(tf.layer_norm(c, np.ones(2), np.zeros(2), 3.0), c / 2.0)


def test_rms_norm_statistics():
    u = RNG.normal(size=(6, 64)) * 3 + 5
    y = tf.rms_norm(u, np.ones(64), 0.0)
    assert np.allclose((y ** 2).mean(-1), 1, atol=1e-12)
    assert np.allclose(tf.rms_norm(np.array([[3.0, 4.0]]), np.ones(2), 0.0), [[3 / math.sqrt(12.5), 4 / math.sqrt(12.5)]])


def test_activations():
    assert tf.gelu_erf(np.array(0.0)) == 0.0
    assert tf.gelu_erf(np.array(1.0)) == pytest.approx(0.8413447460685429, rel=1e-12)   # Phi(1)
    assert tf.gelu_erf(np.array(-1.0)) == pytest.approx(-0.15865525393145707, rel=1e-12)
    assert tf.gelu_erf(np.array(40.0)) == 40.0 and tf.gelu_erf(np.array(-40.0)) == 0.0
    assert tf.silu(np.array(0.0)) == 0.0
    assert tf.silu(np.array(2.0)) == pytest.approx(2.0 / (1 + math.exp(-2.0)), rel=1e-14)
    assert tf.silu(np.array(-30.0)) == pytest.approx(-30.0 * math.exp(-30.0), rel=1e-9)


def test_rope_is_a_rotation_by_position_difference():
    # d_head = 2: one pair, frequency theta^0 = 1 -> plain 2-D rotation by `pos` radians
    x = np.array([[1.0, 0.0]])
    y = tf.rope(x, np.array([0.5]), 1e4)
    assert np.allclose(y, [[math.cos(0.5), math.sin(0.5)]])
    q, k = RNG.normal(size=(1, 16)), RNG.normal(size=(1, 16))
    a = tf.rope(q, [3], 1e4) @ tf.rope(k, [10], 1e4).T
    b = tf.rope(q, [103], 1e4) @ tf.rope(k, [110], 1e4).T
    assert np.allclose(a, b, rtol=1e-10)
    assert np.allclose(np.linalg.norm(tf.rope(q, [77], 1e4)), np.linalg.norm(q))
    # pairing is (c, c + d/2) with frequency theta^(-2c/d): check the second pair of d_head = 4
    v = np.array([[0.0, 1.0, 0.0, 0.0]])
    ang = 2.0 * 100.0 ** (-2.0 / 4.0)
    assert np.allclose(tf.rope(v, [2], 100.0), [[0, math.cos(ang), 0, math.sin(ang)]])


def test_matrix_attention_matches_python_loops():
    n, d = 6, 4
    q, k, v = (RNG.normal(size=(n, d)) for _ in range(3))
    s = q @ k.T / math.sqrt(d)
    s = np.where(np.triu(np.ones((n, n), bool), 1), -np.inf, s)
    p = tf.softmax_rows(s)
    out, probs = loops.causal_attention_loops(q.tolist(), k.tolist(), v.tolist())
    assert np.allclose(p @ v, np.array(out), rtol=1e-12)
    for i in range(n):
        assert np.allclose(p[i, :i + 1], probs[i], rtol=1e-12)


# ----------------------------------------------------------------------------- cached forward
@pytest.mark.parametrize("kind", ["ln", "rms"])
def test_cached_forward_equals_full_recompute(kind):
    cfg = tiny(kind)
    W = weights(cfg)
    n = 7
    x = RNG.normal(size=(n, cfg.d_latent))
    ids = np.full(n, -1)
    if cfg.n_cond_ids:
        ids[0] = 3
    z_full, sh_full, ha_full = loops.full_recompute(cfg, W, "m", x, ids, shallow_layer=1)
    for chunks in ([7], [1] * 7, [3, 2, 2], [5, 1, 1], [1, 6]):
        cache = tf.KVCache(cfg, 1)
        zs, shs, has = [], [], []
        start = 0
        for c in chunks:
            z, sh, ha = tf.forward_sample(cfg, W, "m", cache, 0, x[start:start + c], ids[start:start + c],
                                          commit=True, shallow_layer=1)
            zs.append(z); shs.append(sh); has.append(ha)
            start += c
        assert cache.length(0) == n
        assert np.allclose(np.concatenate(zs), z_full, rtol=1e-10, atol=1e-12)
        assert np.allclose(np.concatenate(shs), sh_full, rtol=1e-10, atol=1e-12)
        assert np.allclose(np.concatenate(has), ha_full, rtol=1e-10, atol=1e-12)


def test_commit_false_leaves_cache_untouched():
    cfg = tiny("ln")
    W = weights(cfg)
    cache = tf.KVCache(cfg, 1)
    tf.forward_sample(cfg, W, "m", cache, 0, RNG.normal(size=(3, 4)))
    z1, _, _ = tf.forward_sample(cfg, W, "m", cache, 0, RNG.normal(size=(2, 4)), commit=False)
    assert cache.length(0) == 3
    x = RNG.normal(size=(2, 4))
    a, _, _ = tf.forward_sample(cfg, W, "m", cache, 0, x, commit=False)
    b, _, _ = tf.forward_sample(cfg, W, "m", cache, 0, x, commit=False)
    assert np.array_equal(a, b)


@pytest.mark.parametrize("kind", ["ln", "rms"])
def test_causality(kind):
    cfg = tiny(kind)
    W = weights(cfg)
    x = RNG.normal(size=(6, cfg.d_latent))
    y = x.copy()
    y[4] += 1.0
    za, _, _ = tf.forward_sample(cfg, W, "m", tf.KVCache(cfg, 1), 0, x)
    zb, _, _ = tf.forward_sample(cfg, W, "m", tf.KVCache(cfg, 1), 0, y)
    assert np.array_equal(za[:4], zb[:4])
    assert not np.allclose(za[4:], zb[4:])


def test_zero_query_gives_running_mean_of_values_and_log_count_entropy():
    """W_q = 0 -> uniform attention over the visible keys.  With W_o = I and the MLP output
    projection zero, layer output = h + running mean of V; attention entropy = ln(#visible)."""
    cfg = TfCfg(n_layers=1, d_model=16, n_heads=2, n_kv_heads=2, d_head=8, d_ff=24, act=ACT_GELU,
                norm=NORM_LAYER, pos=POS_LEARNED, has_bias=1, d_latent=4, max_pos=32)
    W = weights(cfg)
    d = cfg.d_model
    W["m.L0.wqkv"][:, :d] = 0
    W["m.L0.bqkv"][:d] = 0
    W["m.L0.wo"] = np.eye(d, dtype=np.float32)
    W["m.L0.bo"][:] = 0
    W["m.L0.w2"][:] = 0
    W["m.L0.b2"][:] = 0
    n = 5
    x = RNG.normal(size=(n, 4))
    cache = tf.KVCache(cfg, 1)
    _, sh, ha = tf.forward_sample(cfg, W, "m", cache, 0, x, shallow_layer=1)
    h0 = x @ W["m.in.w"].astype(float) + W["m.in.b"] + W["m.pos"][:n]
    u = tf.layer_norm(h0, W["m.L0.n1.g"].astype(float), W["m.L0.n1.b"].astype(float), cfg.norm_eps)
    v = u @ W["m.L0.wqkv"][:, 2 * d:].astype(float) + W["m.L0.bqkv"][2 * d:]
    want = h0 + np.cumsum(v, axis=0) / np.arange(1, n + 1)[:, None]
    assert np.allclose(sh, want, rtol=1e-10)
    assert np.allclose(ha, np.log(np.arange(1, n + 1)), atol=1e-12)


def test_gqa_with_repeated_kv_heads_equals_mha():
    g = tiny("rms", L=2)                       # 4 q heads, 2 kv heads
    Wg = weights(g)
    m = TfCfg(**{**g.__dict__, "n_kv_heads": 4})
    Wm = dict(Wg)
    H, Hk, dh = g.n_heads, g.n_kv_heads, g.d_head
    for l in range(g.n_layers):
        w = Wg[f"m.L{l}.wqkv"]
        q = w[:, :H * dh]
        k = w[:, H * dh:(H + Hk) * dh].reshape(-1, Hk, dh)
        v = w[:, (H + Hk) * dh:].reshape(-1, Hk, dh)
        rep = lambda t: np.repeat(t, H // Hk, axis=1).reshape(w.shape[0], H * dh)
        Wm[f"m.L{l}.wqkv"] = np.concatenate([q, rep(k), rep(v)], axis=1)
    x = RNG.normal(size=(5, g.d_latent))
    za, _, _ = tf.forward_sample(g, Wg, "m", tf.KVCache(g, 1), 0, x)
    zb, _, _ = tf.forward_sample(m, Wm, "m", tf.KVCache(m, 1), 0, x)
    assert np.allclose(za, zb, rtol=1e-11)


def test_up_projection_follows_the_final_norm():
    cfg = tiny("rms", L=1)
    W = weights(cfg)
    x = RNG.normal(size=(3, cfg.d_latent))
    z, sh, _ = tf.forward_sample(cfg, W, "m", tf.KVCache(cfg, 1), 0, x, shallow_layer=1)
    assert z.shape == (3, cfg.d_out)
    # z = RMSNorm(h_L) W_up
    want = tf.rms_norm(sh, W["m.nf.g"].astype(float), cfg.norm_eps) @ W["m.up.w"].astype(float)
    assert np.allclose(z, want, rtol=1e-12)


def test_loaded_cache_is_used_and_batch_rows_are_independent():
    cfg = tiny("ln")
    W = weights(cfg)
    B, n = 3, 6
    cache = tf.KVCache(cfg, B)
    for l in range(cfg.n_layers):
        k, v = gen.kv_cache(cfg, 5, "m", l, B, n, DT_F32)
        cache.load(l, k, v)
    xs = [RNG.normal(size=(2, 4)), RNG.normal(size=(0, 4)), RNG.normal(size=(3, 4))]
    zs, _, _ = tf.forward(cfg, W, "m", cache, xs, commit=False)
    assert zs[1].shape == (0, 16)
    solo = tf.KVCache(cfg, 1)
    for l in range(cfg.n_layers):
        k, v = gen.kv_cache(cfg, 5, "m", l, B, n, DT_F32)
        solo.load(l, k[2:3], v[2:3])
    z2, _, _ = tf.forward_sample(cfg, W, "m", solo, 0, xs[2], commit=False)
    assert np.array_equal(zs[2], z2)
    # the cache content matters
    empty, _, _ = tf.forward_sample(cfg, W, "m", tf.KVCache(cfg, 1), 0, xs[2], commit=False)
    assert not np.allclose(empty, z2)


def test_class_id_row_uses_table_lookup():
    cfg = tiny("ln", L=1)
    W = weights(cfg)
    x = RNG.normal(size=(2, 4))
    z_a, _, _ = tf.forward_sample(cfg, W, "m", tf.KVCache(cfg, 1), 0, x, np.array([2, -1]))
    x2 = x.copy()
    x2[0] = 99.0                       # the latent of an id row is ignored
    z_b, _, _ = tf.forward_sample(cfg, W, "m", tf.KVCache(cfg, 1), 0, x2, np.array([2, -1]))
    assert np.array_equal(z_a, z_b)
    z_c, _, _ = tf.forward_sample(cfg, W, "m", tf.KVCache(cfg, 1), 0, x, np.array([4, -1]))
    assert not np.allclose(z_a, z_c)


# ----------------------------------------------------------------------------- MLP branches and the score scale, by hand
def _plain_block_weights(cfg, W):
    """Layer 0 with identity norms' gains, so that what the block adds can be written out by hand."""
    V = {k: np.array(v, dtype=np.float64) for k, v in W.items()}
    return V


def test_swiglu_branch_equals_explicit_two_gemm_composition():
    """h_out - h_mid = (SiLU(u W_g) * (u W_u)) W_d with every product taken by the triple loop and SiLU typed out:
    a dropped SiLU, swapped gate/up, or a transposed operand fails here (no second oracle path is involved)."""
    cfg = tiny("rms", L=1)
    W = weights(cfg)
    # switch the attention branch off (W_o = 0): the residual stream before the MLP is the embedding itself
    W["m.L0.wo"] = np.zeros_like(W["m.L0.wo"])
    x = RNG.normal(size=(3, cfg.d_latent))
    _, sh, _ = tf.forward_sample(cfg, W, "m", tf.KVCache(cfg, 1), 0, x, shallow_layer=1)
    h0 = np.array(loops.matmul_loops(x.tolist(), W["m.in.w"].astype(float).tolist())) + W["m.in.b"].astype(float)
    g2 = W["m.L0.n2.g"].astype(float)
    u = np.zeros_like(h0)
    for i in range(h0.shape[0]):
        ms = sum(float(v) ** 2 for v in h0[i]) / h0.shape[1]
        for c in range(h0.shape[1]):
            u[i, c] = h0[i, c] / math.sqrt(ms + cfg.norm_eps) * g2[c]
    a = np.array(loops.matmul_loops(u.tolist(), W["m.L0.wg"].astype(float).tolist()))
    b = np.array(loops.matmul_loops(u.tolist(), W["m.L0.wu"].astype(float).tolist()))
    act = np.zeros_like(a)
    for i in range(a.shape[0]):
        for j in range(a.shape[1]):
            act[i, j] = a[i, j] / (1.0 + math.exp(-a[i, j])) * b[i, j]
    m = np.array(loops.matmul_loops(act.tolist(), W["m.L0.wd"].astype(float).tolist()))
    assert np.allclose(sh, h0 + m, rtol=1e-11, atol=1e-13)
    assert np.abs(m).max() > 1e-3                                   # the branch is not vacuous


def test_gelu_branch_equals_explicit_composition():
    """h_out - h_mid = GELU(u W_1 + b_1) W_2 + b_2, GELU(a) = a Phi(a) with the standard normal CDF from the
    error function of the math module; products by the triple loop."""
    cfg = tiny("ln", L=1)
    W = weights(cfg)
    W["m.L0.wo"] = np.zeros_like(W["m.L0.wo"])
    W["m.L0.bo"] = np.zeros_like(W["m.L0.bo"])
    n = 3
    x = RNG.normal(size=(n, cfg.d_latent))
    _, sh, _ = tf.forward_sample(cfg, W, "m", tf.KVCache(cfg, 1), 0, x, shallow_layer=1)
    h0 = np.array(loops.matmul_loops(x.tolist(), W["m.in.w"].astype(float).tolist())) + W["m.in.b"].astype(float) \
        + W["m.pos"][:n].astype(float)
    g2, b2n = W["m.L0.n2.g"].astype(float), W["m.L0.n2.b"].astype(float)
    u = np.zeros_like(h0)
    for i in range(n):
        mean = sum(h0[i]) / h0.shape[1]
        var = sum((v - mean) ** 2 for v in h0[i]) / h0.shape[1]
        for c in range(h0.shape[1]):
            u[i, c] = (h0[i, c] - mean) / math.sqrt(var + cfg.norm_eps) * g2[c] + b2n[c]
    a = np.array(loops.matmul_loops(u.tolist(), W["m.L0.w1"].astype(float).tolist())) + W["m.L0.b1"].astype(float)
    act = np.array([[v * 0.5 * (1.0 + math.erf(v / math.sqrt(2.0))) for v in row] for row in a])
    m = np.array(loops.matmul_loops(act.tolist(), W["m.L0.w2"].astype(float).tolist())) + W["m.L0.b2"].astype(float)
    assert np.allclose(sh, h0 + m, rtol=1e-11, atol=1e-13)
    assert np.abs(m).max() > 1e-3


def test_score_scale_is_one_over_sqrt_head_dim_in_closed_form():
    """One head, two keys, weights chosen so that q . k is known: row 1 sees keys 0 and 1 with scores
    s_c = q_1 . k_c / sqrt(d_h); its attention entropy is the binary entropy of sigmoid(s_1 - s_0) and its
    output is the sigmoid-weighted mean of the two values.  A missing or squared scale moves both."""
    dh = 16
    cfg = TfCfg(n_layers=1, d_model=dh, n_heads=1, n_kv_heads=1, d_head=dh, d_ff=8, act=ACT_GELU, norm=NORM_LAYER,
                pos=POS_LEARNED, has_bias=1, d_latent=4, max_pos=8)
    W = weights(cfg)
    d = dh
    # q = k = v = the normalised row itself (identity projections, no bias); W_o = I; MLP output switched off
    W["m.L0.wqkv"] = np.concatenate([np.eye(d), np.eye(d), np.eye(d)], axis=1).astype(np.float32)
    W["m.L0.bqkv"] = np.zeros(3 * d, np.float32)
    W["m.L0.wo"] = np.eye(d, dtype=np.float32)
    W["m.L0.bo"] = np.zeros(d, np.float32)
    W["m.L0.w2"] = np.zeros_like(W["m.L0.w2"])
    W["m.L0.b2"] = np.zeros_like(W["m.L0.b2"])
    W["m.L0.n1.g"] = np.ones(d, np.float32)
    W["m.L0.n1.b"] = np.zeros(d, np.float32)
    x = RNG.normal(size=(2, 4))
    _, sh, ha = tf.forward_sample(cfg, W, "m", tf.KVCache(cfg, 1), 0, x, shallow_layer=1)
    h0 = x @ W["m.in.w"].astype(float) + W["m.in.b"].astype(float) + W["m.pos"][:2].astype(float)
    u = np.zeros_like(h0)
    for i in range(2):
        mean = sum(h0[i]) / d
        var = sum((v - mean) ** 2 for v in h0[i]) / d
        u[i] = [(v - mean) / math.sqrt(var + cfg.norm_eps) for v in h0[i]]
    s0 = sum(u[1][t] * u[0][t] for t in range(d)) / math.sqrt(dh)
    s1 = sum(u[1][t] * u[1][t] for t in range(d)) / math.sqrt(dh)
    p1 = 1.0 / (1.0 + math.exp(-(s1 - s0)))
    p0 = 1.0 - p1
    assert 0.02 < p0 < 0.98                                          # both keys matter
    assert ha[0] == pytest.approx(0.0, abs=1e-14)                    # row 0 sees one key
    assert ha[1] == pytest.approx(-(p0 * math.log(p0) + p1 * math.log(p1)), rel=1e-11)
    assert np.allclose(sh[1], h0[1] + p0 * u[0] + p1 * u[1], rtol=1e-11)
    # with the scale dropped (or applied twice) the same closed form gives another number
    for wrong in (1.0, 1.0 / dh):
        pw = 1.0 / (1.0 + math.exp(-(s1 - s0) * math.sqrt(dh) * wrong))
        assert abs(pw - p1) > 1e-3
