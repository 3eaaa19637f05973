"""GPU parity of Alg. 1 Step 5 (residual resampling, closing token) and of multi-round generation against the
CPU oracle, through the C-ABI."""
import numpy as np
import pytest

from synth import gen
from tests.harness import build_case, make_ctx, gpu_inputs, oracle_caches, rel_inf, to_np

pytestmark = pytest.mark.gpu

TOL = 2e-2


def _gen_inputs(rc, B, R, J, seed):
    D, K, S = rc.target.d_latent, rc.K, rc.head.n_steps
    return dict(eps=np.stack([gen.noise(seed, f"g.eps{t}", (S + 1, B, K + 1, D)) for t in range(R)]),
                r=np.stack([gen.uniforms(seed, f"g.r{t}", (B, K)) for t in range(R)]),
                eps_res=np.stack([gen.noise(seed, f"g.er{t}", (B, J, D)) for t in range(R)]),
                u_res=np.stack([gen.uniforms(seed, f"g.ur{t}", (B, J)) for t in range(R)]))


def test_resample_matches_oracle_on_identical_inputs():
    """Unit level: same means, noise and uniforms on both sides; every branch (rejected at each position, all
    accepted, nothing drafted, exhausted loop).  A proposal whose alpha is within 1e-4 of its uniform may flip."""
    from oracle import resample as rs
    case = build_case("ln-gelu-bf16", seed=50)
    ctx = make_ctx(case)
    rc = case.rc
    B, K, D, J, S = case.B, rc.K, rc.target.d_latent, 6, rc.head.n_steps
    rng = np.random.default_rng(8)
    s = rc.head.sigma_last * rc.head.temperature
    checked = 0
    for rep in range(12):
        mu_q = rng.normal(size=(B, K, D)).astype(np.float32)
        mu_p = np.concatenate([mu_q, mu_q[:, :1]], 1) + (rng.normal(size=(B, K + 1, D)) * s * rng.choice([0.0, 0.3, 1.0, 3.0])).astype(np.float32)
        mu_p = mu_p.astype(np.float32)
        eps = rng.normal(size=(S + 1, B, K + 1, D)).astype(np.float32)
        eps_res = rng.normal(size=(B, J, D)).astype(np.float32)
        u_res = rng.random((B, J)).astype(np.float32)
        n_keep = rng.integers(0, K + 1, size=B).astype(np.int32)
        n_acc = np.array([rng.integers(0, k + 1) for k in n_keep], dtype=np.int32)
        xg, tg = ctx.spec_resample(ctx.dev_f32(mu_p), ctx.dev_f32(mu_q), ctx.dev_f32(eps), ctx.dev_i32(n_acc), ctx.dev_i32(n_keep),
                                   ctx.dev_f32(eps_res), ctx.dev_f32(u_res))
        ctx.sync()
        xg, tg = xg.cpu().numpy(), tg.cpu().numpy()
        xo, to = rs.next_token(n_acc, n_keep, mu_p, mu_q, eps[-1], eps_res, u_res, 0.0, s, s)
        for b in range(B):
            if n_acc[b] < n_keep[b]:
                n = n_acc[b]
                prop = mu_p[b, n].astype(np.float64) + s * eps_res[b].astype(np.float64)
                alpha = rs.residual_accept_prob(prop, mu_p[b, n], mu_q[b, n], 0.0, s, s)
                if (np.abs(alpha[:to[b]] - u_res[b, :to[b]]) < 1e-4).any():
                    continue
            assert tg[b] == to[b]
            assert np.allclose(xg[b], xo[b], rtol=1e-5, atol=1e-6)
            checked += 1
    assert checked > 10 * B
    ctx.close()


def _run_generate(case, R, J, seed, tau=-1.0):
    from oracle import resample as rs
    ctx = make_ctx(case)
    gi = gpu_inputs(ctx, case)
    g_in = _gen_inputs(case.rc, case.B, R, J, seed)
    out = ctx.spec_generate(gi["pending"], ctx.dev_f32(g_in["eps"]), ctx.dev_f32(g_in["r"]), ctx.dev_f32(g_in["eps_res"]),
                            ctx.dev_f32(g_in["u_res"]), tau)
    ctx.sync()
    from paper_2512_08537_amd import binding
    g = to_np(out)
    g["len_t"] = ctx.spec_kv_lengths(binding.TARGET, case.B)
    g["len_d"] = ctx.spec_kv_lengths(binding.DRAFT, case.B)
    ctx.close()
    tc, dc = oracle_caches(case)
    toks, rounds = rs.generate(case.rc, case.W, tc, dc, case.inp["pending"], list(g_in["eps"]), list(g_in["r"]),
                               list(g_in["eps_res"]), list(g_in["u_res"]), tau, case.B)
    return g, toks, rounds, g_in


def test_generate_three_rounds_matches_oracle():
    """Round by round; a sample leaves the comparison at its first decision that differs, which must then be one
    the oracle takes with a small margin (bf16 means move ln rho by a few 1e-2)."""
    case = build_case("ln-gelu-bf16", seed=51)
    R, J, K, B = 3, 8, case.rc.K, case.B
    g, toks, rounds, g_in = _run_generate(case, R, J, seed=9)
    # what holds whatever the decisions were
    n_tok = (g["n_accept"] + 1).sum(axis=0)
    assert np.array_equal(g["n_tokens"], n_tok)
    assert np.array_equal(g["len_t"], case.n_ctx + n_tok)
    assert np.array_equal(g["len_d"], case.n_ctx + n_tok)
    assert (g["n_accept"] <= g["n_keep"]).all() and (g["tries"][g["n_accept"] == g["n_keep"]] == 0).all()
    assert np.isfinite(g["tokens"]).all()
    alive = np.ones(B, dtype=bool)
    pos = np.zeros(B, dtype=int)
    compared = 0
    for t, rr in enumerate(rounds):
        for b in range(B):
            if not alive[b]:
                continue
            na_o, na_g = int(rr["n_accept"][b]), int(g["n_accept"][t, b])
            nk = int(rr["n_keep"][b])
            assert int(g["n_keep"][t, b]) == nk
            margin = np.abs(np.log(g_in["r"][t, b, :nk].astype(np.float64)) - rr["log_ratio"][b, :nk])
            if na_o != na_g or g["tries"][t, b] != rr["tries"][b]:
                first = min(na_o, na_g)
                if na_o != na_g:
                    assert margin[first] < 0.3, (t, b, margin)
                alive[b] = False
                continue
            k = na_o
            tol = TOL * (t + 1) * 2
            if k:
                assert rel_inf(g["tokens"][b, pos[b]:pos[b] + k], toks[b][pos[b]:pos[b] + k]) < tol
            assert rel_inf(g["tokens"][b, pos[b] + k], toks[b][pos[b] + k]) < tol
            pos[b] += k + 1
            compared += 1
    assert compared >= B                                     # at least every sample's first round
    assert (g["tries"] > 0).any() and (g["n_accept"] == g["n_keep"]).any()     # both closing branches ran


def test_generate_with_draft_equal_to_target():
    """Identical models: every round accepts all K drafts (up to the rounding of ln rho ~ 0), closes with the
    bonus token, and the draft cache is caught up with draft K before the next round."""
    case = build_case("ln-gelu-bf16", seed=52, same_draft=True)
    R, J, K, B = 3, 4, case.rc.K, case.B
    g, toks, rounds, g_in = _run_generate(case, R, J, seed=10)
    for rr in rounds:
        assert np.array_equal(rr["n_accept"], np.full(B, K))
    # uniforms that clear ln rho ~ 0 by a margin accept on the GPU too
    ok = (np.log(g_in["r"].astype(np.float64)) <= -5e-2).all(axis=(0, 2))
    assert ok.any()
    for b in np.nonzero(ok)[0]:
        assert np.array_equal(g["n_accept"][:, b], np.full(R, K))
        assert not g["tries"][:, b].any()
        assert g["n_tokens"][b] == R * (K + 1)
        assert g["len_t"][b] == case.n_ctx + R * (K + 1) and g["len_d"][b] == case.n_ctx + R * (K + 1)
        for t in range(R):
            sl = slice(t * (K + 1), (t + 1) * (K + 1))
            assert rel_inf(g["tokens"][b, sl], toks[b][sl]) < TOL * (t + 1) * 2


def test_generate_rejects_rounds_beyond_the_cache():
    case = build_case("ln-gelu-bf16", seed=53)
    ctx = make_ctx(case)
    gi = gpu_inputs(ctx, case)
    R = (case.rc.max_ctx - case.n_ctx) // (case.rc.K + 1) + 1
    g_in = _gen_inputs(case.rc, case.B, R, 2, 3)
    with pytest.raises(Exception):
        ctx.spec_generate(gi["pending"], ctx.dev_f32(g_in["eps"]), ctx.dev_f32(g_in["r"]), ctx.dev_f32(g_in["eps_res"]),
                          ctx.dev_f32(g_in["u_res"]), -1.0)
    ctx.close()
