"""GPU parity of the KV-cached transformer forward (spec_forward) against the CPU oracle."""
import numpy as np
import pytest

from synth import gen
from synth.configs import DT_BF16, DT_F32
from tests.harness import build_case, make_ctx, oracle_caches, rel_inf

pytestmark = pytest.mark.gpu

TOL = {DT_BF16: 2e-2, DT_F32: 2e-4}


def _oracle_forward(case, which, xs, ids=None, commit=False, shallow=None, caches=None):
    from oracle import transformer as tf
    tc, dc = caches or oracle_caches(case)
    cfg, cache, prefix = (case.rc.target, tc, "target") if which == 0 else (case.rc.draft, dc, "draft")
    return tf.forward(cfg, case.W, prefix, cache, xs, ids=ids, commit=commit, shallow_layer=shallow)


def _pack(xs):
    return np.concatenate([x for x in xs if len(x)], axis=0).astype(np.float32)


@pytest.mark.parametrize("kind", ["ln-gelu-bf16", "gqa-rope-bf16", "ln-gelu-f32", "mid-bf16"])
@pytest.mark.parametrize("which", [0, 1])
@pytest.mark.parametrize("peaky", [False, True])
def test_forward_matches_oracle_with_ragged_rows(kind, which, peaky):
    """peaky=False: the workload recipe (weights N(0, 0.02)); the attention-row entropy of layer l_s is held to the
    stated 1e-3.  peaky=True: a stress variant outside the recipe (QKV weights scaled until the scores have a standard
    deviation near 2, so that a wrong mask or K/Q layout shows as an error of order 1); there the bf16 rounding of q
    and k alone moves a row's entropy by up to 1e-2, and the entropy bar is 2e-2."""
    case = build_case(kind, seed=21, peaky=peaky)
    rc = case.rc
    ctx = make_ctx(case)
    B, K, D = case.B, rc.K, rc.target.d_latent
    rng = np.random.default_rng(3)
    n_q = rng.integers(0, K + 2, size=B)
    n_q[0] = K + 1
    if B > 1:
        n_q[1] = 0                                       # an empty sample in the middle
    xs = [gen.bf16_round(rng.normal(size=(n, D)).astype(np.float32)) for n in n_q]
    z, sh, ha = ctx.spec_forward(which, ctx.dev_f32(_pack(xs)), n_q, commit=False, want_shallow=True,
                                 want_h_attn=True)
    ctx.sync()
    zo, sho, hao = _oracle_forward(case, which, xs, shallow=rc.entropy_layer)
    zo, sho, hao = np.concatenate(zo), np.concatenate(sho), np.concatenate(hao)
    tol = TOL[rc.dtype]
    ez, es = rel_inf(z.float().cpu().numpy(), zo), rel_inf(sh.cpu().numpy(), sho)
    eh = float(np.abs(ha.cpu().numpy() - hao).max())
    print(f"z {ez:.2e} shallow {es:.2e} h_attn {eh:.2e} (H range {hao.min():.2f}..{hao.max():.2f})")
    assert ez < tol
    assert es < tol
    assert eh < (1e-4 if rc.dtype == DT_F32 else (2e-2 if peaky else 1e-3))
    # commit=False leaves lengths alone
    assert np.array_equal(ctx.spec_kv_lengths(which, B), np.full(B, case.n_ctx))
    ctx.close()


@pytest.mark.parametrize("kind,rows", [("mid-bf16", 80), ("gqa-rope-bf16", 31), ("ln-gelu-bf16", 50)])
@pytest.mark.parametrize("which", [0, 1])
@pytest.mark.parametrize("peaky", [False, True])
def test_forward_with_more_rows_than_one_attention_pass(kind, rows, which, peaky):
    """More rows per sample than one attention workgroup holds (64, or 12 with 5:1 grouped heads): the layers take
    all rows at once and the attention walks them in passes; features, shallow stream and attention-row
    entropies against the oracle's single forward.  peaky=True (scores with a standard deviation near 2, so that a
    wrong mask or pass boundary shows as an error of order 1): later rows attend to K / V rows that this same bf16
    forward produced, single rows are off by up to 2 % (measured), so the bar is twice the stated one there."""
    case = build_case(kind, seed=25, peaky=peaky)
    rc = case.rc
    ctx = make_ctx(case)
    B, D = case.B, rc.target.d_latent
    rng = np.random.default_rng(6)
    room = rc.max_ctx - case.n_ctx
    n_q = rng.integers(1, min(rows, room) + 1, size=B)
    n_q[0] = min(rows, room)
    if B > 2:
        n_q[2] = 0
    xs = [gen.bf16_round(rng.normal(size=(n, D)).astype(np.float32)) for n in n_q]
    z, sh, ha = ctx.spec_forward(which, ctx.dev_f32(_pack(xs)), n_q, commit=True, want_shallow=True, want_h_attn=True)
    ctx.sync()
    zo, sho, hao = _oracle_forward(case, which, xs, shallow=rc.entropy_layer)
    zo, sho, hao = np.concatenate(zo), np.concatenate(sho), np.concatenate(hao)
    ez, es = rel_inf(z.float().cpu().numpy(), zo), rel_inf(sh.cpu().numpy(), sho)
    eh = float(np.abs(ha.cpu().numpy() - hao).max())
    print(f"{kind} which={which} rows {n_q.tolist()}: z {ez:.2e} shallow {es:.2e} h_attn {eh:.2e}")
    tol = 4e-2 if peaky else 2e-2
    assert ez < tol and es < tol and eh < tol
    assert np.array_equal(ctx.spec_kv_lengths(which, B), case.n_ctx + n_q)
    ctx.close()


@pytest.mark.parametrize("kind", ["ln-gelu-bf16", "gqa-rope-bf16", "ln-gelu-f32"])
def test_chunked_prefill_equals_one_shot_and_oracle(kind):
    """Cache built by the library's own forward in chunks (3 + 1 + 4 rows ...) must give the same
    features as the oracle's full recompute: cached == recompute on the GPU path."""
    from oracle import loops
    case = build_case(kind, seed=22, peaky=True)
    rc = case.rc
    ctx = make_ctx(case)
    B, D = case.B, rc.target.d_latent
    rng = np.random.default_rng(4)
    n_tot = 33 if kind != "gqa-rope-bf16" else 30
    x_all = gen.bf16_round(rng.normal(size=(B, n_tot, D)).astype(np.float32))
    ctx.spec_kv_reset(0, np.zeros(B, np.int32))
    outs = [[] for _ in range(B)]
    start = 0
    cmax = rc.K + 1                                     # rows per sample the workspace holds
    chunks, left, pat = [], n_tot, [3, 1, cmax, 2, cmax]
    while left > 0:
        c = min(pat[len(chunks) % len(pat)], left)
        chunks.append(c)
        left -= c
    for c in chunks:
        xs = x_all[:, start:start + c].reshape(B * c, D)
        z, _, _ = ctx.spec_forward(0, ctx.dev_f32(xs), np.full(B, c), commit=True)
        ctx.sync()
        zz = z.float().cpu().numpy().reshape(B, c, -1)
        for b in range(B):
            outs[b].append(zz[b])
        start += c
    assert np.array_equal(ctx.spec_kv_lengths(0, B), np.full(B, n_tot))
    for b in (0, B - 1):
        zo, _, _ = loops.full_recompute(rc.target, case.W, "target", x_all[b])
        err = rel_inf(np.concatenate(outs[b]), zo)
        assert err < TOL[rc.dtype]
    ctx.close()


def test_class_id_rows():
    case = build_case("ln-gelu-bf16", seed=23)
    rc = case.rc
    ctx = make_ctx(case)
    B, D = case.B, rc.target.d_latent
    ctx.spec_kv_reset(0, np.zeros(B, np.int32))
    rng = np.random.default_rng(5)
    xs = [gen.bf16_round(rng.normal(size=(3, D)).astype(np.float32)) for _ in range(B)]
    ids = [np.array([b + 2, -1, -1]) for b in range(B)]
    z, _, _ = ctx.spec_forward(0, ctx.dev_f32(_pack(xs)), np.full(B, 3), cond_id=ctx.dev_i32(np.concatenate(ids)),
                               commit=False)
    ctx.sync()
    from oracle import transformer as tf
    cache = tf.KVCache(rc.target, B)
    zo, _, _ = tf.forward(rc.target, case.W, "target", cache, xs, ids=ids, commit=False)
    err = rel_inf(z.float().cpu().numpy(), np.concatenate(zo))
    assert err < 2e-2
    ctx.close()


def test_capacity_and_argument_errors():
    from paper_2512_08537_amd.binding import FardError
    case = build_case("ln-gelu-bf16", seed=24)
    ctx = make_ctx(case)
    B, D = case.B, 16
    x = ctx.dev_f32(np.zeros((B, D), np.float32))
    ctx.spec_kv_reset(0, np.full(B, case.rc.max_ctx, np.int32))
    with pytest.raises(FardError) as e:
        ctx.spec_forward(0, x, np.ones(B))
    assert e.value.code == -3
    with pytest.raises(FardError) as e:
        ctx.spec_kv_reset(0, np.full(B, case.rc.max_ctx + 1, np.int32))
    assert e.value.code == -3
    # the workspace holds max(max_batch * (K + 1), min(max_batch * max_ctx, 8192)) packed rows
    big = ctx.dev_f32(np.zeros((case.rc.max_batch * case.rc.max_ctx + 1, D), np.float32))
    ctx.spec_kv_reset(0, np.zeros(B, np.int32))
    with pytest.raises(FardError) as e:
        ctx.spec_forward(0, big, np.ones(B))
    assert e.value.code == -3
    with pytest.raises(FardError) as e:
        ctx.spec_kv_commit(-1, ctx.dev_i32(np.zeros(B)))
    assert e.value.code == -6
    ctx.close()


def test_forward_of_72_rows_through_k_slice_planes():
    """72 rows (8 samples x 9) through one 3072-wide layer whose QKV, output and down projections are 19-25 MB each: the
    shapes at which K is split over workgroups of the streaming kernel and the products leave as planes that the RoPE /
    cache-append kernel and the next norm sum (the verify stage of the 5120-wide configuration, reduced).  All samples
    against the oracle, ragged row counts included in a second call."""
    from synth.configs import (RoundCfg, TfCfg, HeadCfg, ACT_SWIGLU, NORM_RMS, POS_ROPE)
    tgt = TfCfg(n_layers=2, d_model=3072, n_heads=24, n_kv_heads=4, d_head=128, d_ff=4096,
                act=ACT_SWIGLU, norm=NORM_RMS, pos=POS_ROPE, has_bias=0, norm_eps=1e-6)
    drf = TfCfg(n_layers=1, d_model=256, n_heads=2, n_kv_heads=1, d_head=128, d_ff=192,
                act=ACT_SWIGLU, norm=NORM_RMS, pos=POS_ROPE, has_bias=0, norm_eps=1e-6, d_out=3072)
    rc = RoundCfg(name="planes-72", target=tgt, draft=drf, head=HeadCfg(1, 128, 3072, n_steps=1), K=8, max_batch=8,
                  max_ctx=64, entropy_layer=1, batch=8, n_ctx=40)
    case = build_case(rc, seed=45, w_std=0.012)            # (a branch gain below one at this width, as trained layers have)
    ctx = make_ctx(case)
    B, D = 8, 16
    rng = np.random.default_rng(12)
    for n_q in (np.full(B, 9), np.array([9, 0, 9, 3, 9, 9, 1, 9])):
        xs = [gen.bf16_round(rng.normal(size=(n, D)).astype(np.float32)) for n in n_q]
        z, sh, _ = ctx.spec_forward(0, ctx.dev_f32(_pack(xs)), n_q, commit=False, want_shallow=True, nq_max=9)
        ctx.sync()
        zo, sho, _ = _oracle_forward(case, 0, xs, shallow=1)
        ez = rel_inf(z.float().cpu().numpy()[:int(n_q.sum())], np.concatenate(zo))
        es = rel_inf(sh.cpu().numpy()[:int(n_q.sum())], np.concatenate(sho))
        print(f"72 rows through planes, n_q {n_q.tolist()}: z {ez:.2e} shallow {es:.2e}")
        assert ez < 2e-2 and es < 2e-2
    ctx.close()


def test_forward_of_72_rows_with_a_split_k_residual_product():
    """72 rows through 1024-wide LayerNorm / GELU layers with a 4096-wide MLP: the down-projection (K = 4096, 8 MB of
    weights: too small for planes, too long for the narrow kernel) runs in the streaming kernel with K split over
    workgroups, one row tile, partial sums added to the residual stream with atomics from the LDS-staged epilogue."""
    from synth.configs import RoundCfg, TfCfg, HeadCfg
    tgt = TfCfg(n_layers=2, d_model=1024, n_heads=16, n_kv_heads=16, d_head=64, d_ff=4096, max_pos=64)
    drf = TfCfg(n_layers=1, d_model=256, n_heads=4, n_kv_heads=4, d_head=64, d_ff=512, d_out=1024, max_pos=64)
    rc = RoundCfg(name="split-72", target=tgt, draft=drf, head=HeadCfg(1, 128, 1024, n_steps=1), K=8, max_batch=8,
                  max_ctx=64, entropy_layer=1, batch=8, n_ctx=40)
    case = build_case(rc, seed=46)
    ctx = make_ctx(case)
    B, D = 8, 16
    rng = np.random.default_rng(13)
    for n_q in (np.full(B, 9), np.array([9, 2, 9, 9, 0, 9, 9, 5])):
        xs = [gen.bf16_round(rng.normal(size=(n, D)).astype(np.float32)) for n in n_q]
        z, sh, _ = ctx.spec_forward(0, ctx.dev_f32(_pack(xs)), n_q, commit=False, want_shallow=True, nq_max=9)
        ctx.sync()
        zo, sho, _ = _oracle_forward(case, 0, xs, shallow=1)
        ez = rel_inf(z.float().cpu().numpy()[:int(n_q.sum())], np.concatenate(zo))
        es = rel_inf(sh.cpu().numpy()[:int(n_q.sum())], np.concatenate(sho))
        print(f"72 rows, split-K residual product, n_q {n_q.tolist()}: z {ez:.2e} shallow {es:.2e}")
        assert ez < 2e-2 and es < 2e-2
    ctx.close()
