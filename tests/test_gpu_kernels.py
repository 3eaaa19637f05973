"""GPU parity of the single kernels behind the C-ABI: GEMM, entropy pre-filter, head, accept.
Each result is compared element by element with the CPU oracle on the same seeded inputs."""
import math

import numpy as np
import pytest

from synth import gen
from synth.configs import reduced, config, DT_BF16, DT_F32, clone
from tests.harness import build_case, make_ctx, rel_inf, to_np

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx_bf16():
    case = build_case("ln-gelu-bf16", seed=3)
    ctx = make_ctx(case)
    yield ctx, case
    ctx.close()


@pytest.fixture(scope="module")
def ctx_f32():
    case = build_case("ln-gelu-f32", seed=3)
    ctx = make_ctx(case)
    yield ctx, case
    ctx.close()


# ----------------------------------------------------------------------------- GEMM
@pytest.mark.parametrize("M,K,N", [(1, 64, 32), (5, 64, 32), (32, 128, 128), (33, 192, 96), (96, 256, 256),
                                   (97, 128, 160), (288, 1024, 1024), (72, 512, 2048), (200, 2048, 320),
                                   (288, 1024, 3072), (130, 768, 4096), (576, 1280, 3840), (65, 256, 64),
                                   (2304, 1280, 3840), (500, 256, 12288),
                                   # enough 256-column panels and rows for the 128-row tile: ragged rows, ragged last panel
                                   (3900, 128, 7680), (3850, 192, 7712),
                                   # a thousand rows and more (prefill passes): ragged rows, few and ragged column
                                   # blocks
                                   (1025, 64, 32), (1100, 256, 96), (1300, 320, 160), (2048, 1024, 1024),
                                   (4100, 128, 416)])
@pytest.mark.parametrize("act", [0, 1, 2])
def test_gemm_bf16_matches_fp64(ctx_bf16, M, K, N, act):
    from oracle import transformer as otf
    ctx, _ = ctx_bf16
    A = gen.normal(11, f"A{M}{K}", (M, K), 1.0, DT_BF16)
    W = gen.normal(11, f"W{K}{N}", (K, N), 0.05, DT_BF16)
    b = gen.normal(11, f"b{N}", (N,), 0.1, DT_F32)
    out = ctx.spec_gemm(ctx.dev_store(A), ctx.dev_store(W), ctx.dev_f32(b), act)
    ctx.sync()
    ref = A.astype(np.float64) @ W.astype(np.float64) + b
    ref = {0: lambda x: x, 1: otf.gelu_erf, 2: otf.silu}[act](ref)
    got = out.float().cpu().numpy()
    # fp32 accumulation, one bf16 rounding of the result
    assert np.allclose(got, ref, rtol=2 ** -7, atol=2e-3 * np.abs(ref).max())
    assert rel_inf(got, ref) < 1e-2


_NARROW_CASES = [
    # M, K, N, epi
    (32, 1024, 1024, 0), (32, 1024, 1024, 3), (13, 64, 32, 1), (16, 1280, 96, 2), (17, 4096, 1024, 2),
    (64, 1024, 160, 3), (49, 1536, 64, 0), (1, 192, 32, 1), (288, 1024, 1024, 2), (130, 512, 96, 3),
    (97, 256, 64, 0), (32, 1024, 4096, 0), (5, 2048, 64, 2),
    # many row slabs against wide matrices: 64- and 32-column workgroups
    (288, 1024, 4096, 0), (130, 1280, 2048, 3), (97, 512, 2112, 1), (100, 1024, 2080, 0), (70, 1536, 2048, 2),
]


@pytest.mark.parametrize("M,K,N,epi", _NARROW_CASES)
def test_gemm_narrow_matches_fp64(ctx_bf16, M, K, N, epi):
    """Narrow-tile GEMM (no K split): every epilogue, one-shot and ring loops, ragged row slabs."""
    import torch
    from oracle import transformer as otf
    ctx, _ = ctx_bf16
    tag = f"{M}.{K}.{N}.{epi}"
    A = gen.normal(13, "A" + tag, (M, K), 1.0, DT_BF16)
    W = gen.normal(13, "W" + tag, (K, N), 0.05, DT_BF16)
    b = gen.normal(13, "b" + tag, (N,), 0.1, DT_F32)
    ref = A.astype(np.float64) @ W.astype(np.float64) + b
    act, kw = 0, {}
    if epi in (0, 1):
        act = 2 if epi == 0 else 1
        ref = {1: otf.gelu_erf, 2: otf.silu}[act](ref)
        out = ctx.empty((M, N), ctx.tdtype if epi == 0 else torch.float32)
    else:
        base = gen.normal(13, "o" + tag, (M, N), 1.0, DT_F32)
        if epi == 3:
            gate = gen.normal(13, "gt" + tag, (M, N), 1.0, DT_F32)
            ref = ref * gate
            kw["gate"] = ctx.dev_f32(gate)
        ref = base + ref
        out = ctx.dev_f32(base)
    ctx.spec_gemm_narrow(ctx.dev_store(A), ctx.dev_store(W), out, bias=ctx.dev_f32(b), epi=epi, act=act, **kw)
    ctx.sync()
    err = rel_inf(out.float().cpu().numpy(), ref)
    assert err < 1e-2, err


@pytest.mark.parametrize("M,K,N,epi", [(32, 1024, 1024, 2), (288, 1024, 1024, 2), (45, 512, 96, 3), (130, 1280, 2048, 3)])
def test_gemm_narrow_bf16_copy_of_a_residual_update(ctx_bf16, M, K, N, epi):
    import torch
    ctx, _ = ctx_bf16
    tag = f"c{M}.{K}.{N}.{epi}"
    A = ctx.dev_store(gen.normal(15, "A" + tag, (M, K), 1.0, DT_BF16))
    W = ctx.dev_store(gen.normal(15, "W" + tag, (K, N), 0.05, DT_BF16))
    base = gen.normal(15, "o" + tag, (M, N), 1.0, DT_F32)
    gate = ctx.dev_f32(gen.normal(15, "g" + tag, (M, N), 1.0, DT_F32)) if epi == 3 else None
    o1, o2 = ctx.dev_f32(base), ctx.dev_f32(base)
    cp = torch.zeros((M, N), dtype=torch.bfloat16, device=ctx.dev)
    torch.cuda.synchronize()
    ctx.spec_gemm_narrow(A, W, o1, gate=gate, epi=epi)
    ctx.spec_gemm_narrow(A, W, o2, gate=gate, epi=epi, out_bf16=cp)
    ctx.sync()
    assert torch.equal(o1, o2)                                       # the copy changes nothing else
    assert torch.equal(cp, o2.to(torch.bfloat16))                    # and is the rounded new value
    with pytest.raises(Exception):
        ctx.spec_gemm_narrow(A, W, ctx.empty((M, N), ctx.tdtype), epi=0, out_bf16=cp)


def _norm_ref(x, g, beta, norm_type, eps):
    x = x.astype(np.float64)
    if norm_type == 0:
        mu = x.mean(axis=1, keepdims=True)
        var = ((x - mu) ** 2).mean(axis=1, keepdims=True)
        return (x - mu) / np.sqrt(var + eps) * g + (0.0 if beta is None else beta)
    return x / np.sqrt((x ** 2).mean(axis=1, keepdims=True) + eps) * g


@pytest.mark.parametrize("M,K,N,norm_type,act,offset", [
    (32, 1024, 4096, 0, 1, 0.0), (288, 1024, 4096, 0, 1, 0.0), (33, 512, 96, 0, 0, 0.0), (64, 1280, 5120, 0, 1, 0.3),
    (100, 1024, 2080, 1, 2, 0.0), (17, 256, 64, 1, 0, 0.5), (288, 1024, 1024, 0, 0, 1.0), (130, 1536, 2048, 0, 1, 0.0),
])
def test_gemm_with_folded_norm_matches_fp64(ctx_bf16, M, K, N, norm_type, act, offset):
    """norm(x) W + b with the norm applied in the GEMM's epilogue, against the plain definition in fp64 on the same
    bf16-rounded inputs.  offset: mean of the rows in units of their standard deviation (the fold subtracts
    mean * colsum(W') after the product, so a large mean costs accuracy: 1 sigma must still meet the bar)."""
    from oracle import transformer as otf
    ctx, _ = ctx_bf16
    tag = f"n{M}.{K}.{N}.{norm_type}"
    x = gen.bf16_round((gen.normal(16, "x" + tag, (M, K), 1.0, DT_F32) + offset).astype(np.float32))
    W = gen.normal(16, "W" + tag, (K, N), 0.05, DT_BF16)
    g = (1.0 + gen.normal(16, "g" + tag, (K,), 0.2, DT_F32)).astype(np.float32)
    beta = gen.normal(16, "be" + tag, (K,), 0.1, DT_F32) if norm_type == 0 else None
    b = gen.normal(16, "b" + tag, (N,), 0.1, DT_F32)
    out = ctx.spec_gemm_norm(ctx.dev_store(x), ctx.dev_store(W), ctx.dev_f32(g), None if beta is None else ctx.dev_f32(beta),
                             ctx.dev_f32(b), norm_type=norm_type, eps=1e-5, act=act)
    ctx.sync()
    ref = _norm_ref(x, g, beta, norm_type, 1e-5) @ W.astype(np.float64) + b
    ref = {0: lambda v: v, 1: otf.gelu_erf, 2: otf.silu}[act](ref)
    err = rel_inf(out.float().cpu().numpy(), ref)
    print(f"folded norm: {err:.2e}")
    assert err < 1e-2, err


def test_gemm_narrow_is_deterministic_and_rejects_bad_shapes(ctx_bf16):
    import torch
    ctx, _ = ctx_bf16
    A = ctx.dev_store(gen.normal(14, "A", (32, 1024), 1.0, DT_BF16))
    W = ctx.dev_store(gen.normal(14, "W", (1024, 256), 0.05, DT_BF16))
    base = gen.normal(14, "o", (32, 256), 1.0, DT_F32)
    outs = []
    for _ in range(3):
        o = ctx.dev_f32(base)
        ctx.spec_gemm_narrow(A, W, o, epi=2)
        ctx.sync()
        outs.append(o.cpu().numpy())
    assert np.array_equal(outs[0], outs[1]) and np.array_equal(outs[0], outs[2])
    Wbad = torch.zeros((96, 32), dtype=ctx.tdtype, device=ctx.dev)          # K % 64 != 0
    with pytest.raises(Exception):
        ctx.spec_gemm_narrow(torch.zeros((4, 96), dtype=ctx.tdtype, device=ctx.dev), Wbad, ctx.empty((4, 32), ctx.tdtype))
    with pytest.raises(Exception):                                            # epi 3 without gate
        ctx.spec_gemm_narrow(A, W, ctx.dev_f32(base), epi=3)


def test_gemm_f32_matches_fp64(ctx_f32):
    ctx, _ = ctx_f32
    for (M, K, N) in [(5, 16, 7), (33, 100, 65), (16, 256, 48)]:
        A = gen.normal(12, f"A{M}", (M, K), 1.0, DT_F32)
        W = gen.normal(12, f"W{N}", (K, N), 0.05, DT_F32)
        out = ctx.spec_gemm(ctx.dev_store(A), ctx.dev_store(W), None, 0)
        ctx.sync()
        ref = A.astype(np.float64) @ W.astype(np.float64)
        assert rel_inf(out.cpu().numpy(), ref) < 1e-5


# ----------------------------------------------------------------------------- entropy pre-filter
def _check_prefilter(ctx, feat, tau, dtype_tol=1e-3):
    from oracle import entropy as ent
    B, K, L = feat.shape
    H, keep, n_keep, surv, n_surv = ctx.entropy_prefilter(ctx.dev_store(feat), tau)
    ctx.sync()
    H, keep, n_keep, surv, n_surv = (t.cpu().numpy() for t in (H, keep, n_keep, surv, n_surv))
    Ho = ent.softmax_entropy(feat.astype(np.float64))
    assert np.abs(H - Ho).max() <= dtype_tol, np.abs(H - Ho).max()
    ko, nko, so, nso = ent.prefilter(Ho, tau)
    near = np.abs(Ho - tau) <= 1e-3                      # decisions this close to tau may flip
    if not near.any():
        assert np.array_equal(keep, ko)
        assert np.array_equal(n_keep, nko)
        assert int(n_surv[0]) == nso and np.array_equal(surv[:nso], so)
    else:
        # off-threshold rows before the first near-threshold row of a sample must agree
        for b in range(B):
            first = np.argmax(near[b]) if near[b].any() else K
            assert np.array_equal(keep[b, :first], ko[b, :first])
    # what is unique regardless of ties: consistency of the outputs with the kernel's own H
    kg, nkg, sg, nsg = ent.prefilter(H.astype(np.float64), np.float32(tau))
    assert np.array_equal(keep, kg) and np.array_equal(n_keep, nkg)
    assert int(n_surv[0]) == nsg and np.array_equal(surv[:nsg], sg)
    return H, Ho


@pytest.mark.parametrize("B,K,L", [(1, 4, 256), (32, 8, 1024), (64, 8, 1280), (8, 8, 2048), (3, 5, 130), (2, 1, 1),
                                   (7, 3, 9), (1024, 2, 72), (1025, 3, 136), (9001, 2, 40), (2500, 4, 257),
                                   (1500, 8, 1280), (1100, 3, 2048), (4100, 1, 8), (1030, 2, 2056)])
def test_prefilter_shapes(ctx_bf16, B, K, L):
    ctx, _ = ctx_bf16
    feat = gen.normal(5, f"feat{B}{K}{L}", (B, K, L), 2.0, DT_BF16)
    from oracle import entropy as ent
    Ho = ent.softmax_entropy(feat.astype(np.float64))
    tau = float(np.median(Ho)) if Ho.size > 1 else 0.0
    _check_prefilter(ctx, feat, tau + 3e-3)


def test_prefilter_stress_fractions(ctx_bf16):
    """Features built so that 0/25/50/75/100 % of drafts fall below the threshold (uniform and ragged)."""
    from oracle import entropy as ent
    ctx, _ = ctx_bf16
    B, K, d = 256, 8, 1280
    cal = gen.stress_features(1, 64, K, d, np.full(64, K), DT_BF16)
    Hc = ent.softmax_entropy(cal.astype(np.float64))
    tau = ent.threshold(Hc)
    assert abs(tau - 0.3 * 7.12) < 0.02
    for frac in (0.0, 0.25, 0.5, 0.75, 1.0):
        for ragged in (False, True):
            cut = gen.cuts_for_fraction(2, B, K, frac, ragged)
            feat = gen.stress_features(2, B, K, d, cut, DT_BF16)
            H, keep, n_keep, surv, n_surv = ctx.entropy_prefilter(ctx.dev_store(feat), tau)
            ctx.sync()
            assert np.array_equal(n_keep.cpu().numpy(), cut)
            assert int(n_surv.cpu()[0]) == int(cut.sum())
            assert abs(cut.sum() / (B * K) - (1 - frac)) < 1e-9 or ragged
            Ho = ent.softmax_entropy(feat.astype(np.float64))
            assert np.abs(H.cpu().numpy() - Ho).max() < 1e-3


def test_prefilter_closed_forms_and_edges(ctx_bf16):
    ctx, _ = ctx_bf16
    B, K, L = 4, 3, 512
    feat = np.zeros((B, K, L), np.float32)
    feat[1, 1, 7] = 60.0                                   # one-hot row: H = 0 -> sample 1 keeps 1 draft
    feat[2, 0, :] = 3.25                                   # constant rows are uniform: H = ln L
    H, keep, n_keep, surv, n_surv = ctx.entropy_prefilter(ctx.dev_store(feat), 1.0)
    ctx.sync()
    H = H.cpu().numpy()
    assert np.allclose(np.delete(H.reshape(-1), 4), math.log(L), atol=1e-4)
    assert abs(H[1, 1]) < 1e-6
    assert n_keep.cpu().tolist() == [3, 1, 3, 3]
    assert surv.cpu().numpy()[:int(n_surv.cpu()[0])].tolist() == [0, 1, 2, 3, 6, 7, 8, 9, 10, 11]
    # everything filtered / empty batch
    H, keep, n_keep, surv, n_surv = ctx.entropy_prefilter(ctx.dev_store(feat), 100.0)
    ctx.sync()
    assert int(n_surv.cpu()[0]) == 0 and not keep.cpu().numpy().any()
    import torch
    empty = torch.empty((0, 3, 16), dtype=ctx.tdtype, device=ctx.dev)
    H, keep, n_keep, surv, n_surv = ctx.entropy_prefilter(empty, 1.0)
    ctx.sync()
    assert int(n_surv.cpu()[0]) == 0


def test_prefilter_near_threshold_rows(ctx_bf16):
    """Rows whose entropy is bisected onto tau +- 1e-3: only those may disagree with the oracle."""
    from oracle import entropy as ent
    ctx, _ = ctx_bf16
    B, K, d = 16, 8, 1280
    tau = 2.14
    rng = np.random.default_rng(0)
    feat = gen.stress_features(4, B, K, d, np.full(B, K), DT_BF16)
    for b in range(0, B, 2):
        i = int(rng.integers(0, K))
        base = feat[b, i].astype(np.float64).copy()
        j = int(rng.integers(0, d))
        lo, hi = 0.0, 14.0
        target = tau + 1e-3 * rng.uniform(-1, 1)
        for _ in range(60):
            mid = 0.5 * (lo + hi)
            row = base.copy()
            row[j] += mid
            if ent.softmax_entropy(gen.bf16_round(row.astype(np.float32))) > target:
                lo = mid
            else:
                hi = mid
        base[j] += lo
        feat[b, i] = gen.bf16_round(base.astype(np.float32))
    _check_prefilter(ctx, feat, tau)


def test_prefilter_f32(ctx_f32):
    ctx, _ = ctx_f32
    feat = gen.normal(6, "featf32", (4, 4, 256), 3.0, DT_F32)
    _check_prefilter(ctx, feat, 3.0, dtype_tol=1e-4)
    feat = gen.normal(6, "featf32big", (1300, 3, 100), 3.0, DT_F32)     # wave-per-sample path, ragged pieces
    _check_prefilter(ctx, feat, 2.5, dtype_tol=1e-4)


# ----------------------------------------------------------------------------- head
@pytest.mark.parametrize("fix", ["ctx_bf16", "ctx_f32"])
def test_diffhead_decode_matches_oracle(fix, request):
    from oracle import head as ohd
    ctx, case = request.getfixturevalue(fix)
    rc = case.rc
    n, D, S = 11, rc.head.d_latent, rc.head.n_steps
    z = gen.normal(8, "z", (n, rc.head.d_cond), 1.0, rc.dtype)
    eps = gen.noise(8, "eps", (S + 1, n, D))
    mu, x = ctx.diffhead_decode(ctx.dev_store(z), ctx.dev_f32(eps))
    ctx.sync()
    mu_o, x_o = ohd.decode(rc.head, case.W, z, eps)
    tol = 2e-2 if rc.dtype == DT_BF16 else 1e-4
    assert rel_inf(mu.cpu().numpy(), mu_o) < tol
    assert rel_inf(x.cpu().numpy(), x_o) < tol
    # device-side row count: rows beyond it stay untouched (zero-initialised by the binding)
    import torch
    cnt = torch.tensor([4], dtype=torch.int32, device=ctx.dev)
    mu2, x2 = ctx.diffhead_decode(ctx.dev_store(z), ctx.dev_f32(eps), n_rows=cnt)
    ctx.sync()
    assert rel_inf(mu2.cpu().numpy()[:4], mu_o[:4]) < tol
    assert not mu2.cpu().numpy()[4:].any()


@pytest.mark.parametrize("shift,n", [(2.0, 11), (4.0, 15), (8.0, 7)])   # in units of the rows' standard deviation (about 0.1)
def test_diffhead_decode_with_rows_far_from_zero_mean(shift, n):
    """The head's residual rows get a mean of `shift` standard deviations (bias of the input projection): from the
    second block of a step on the modulated norm is folded into the block's first GEMM (up to 64 rows), which
    subtracts mean x (1 + scale) W1 from a product of rounded rows."""
    from oracle import head as ohd
    case = build_case("ln-gelu-bf16", seed=5)
    rc = case.rc
    w = rc.head.width
    case.W["head.in.b"] = gen.bf16_round((np.asarray(case.W["head.in.b"], dtype=np.float32) + 0.1 * shift).astype(np.float32))
    ctx = make_ctx(case)
    D, S = rc.head.d_latent, rc.head.n_steps
    z = gen.normal(12, "zs", (n, rc.head.d_cond), 1.0, rc.dtype)
    eps = gen.noise(12, "es", (S + 1, n, D))
    mu, x = ctx.diffhead_decode(ctx.dev_store(z), ctx.dev_f32(eps))
    ctx.sync()
    mu_o, x_o = ohd.decode(rc.head, case.W, z, eps)
    assert rel_inf(mu.cpu().numpy(), mu_o) < 2e-2
    assert rel_inf(x.cpu().numpy(), x_o) < 2e-2
    ctx.close()


def test_diffhead_decode_of_72_rows_in_tile_order():
    """72 rows (not a multiple of the narrow kernel's 32-row workgroups) through a 256-wide head: the rows between the
    norm and the GEMMs are in tile order, and the last workgroup's second row tile lies past the matrix."""
    from oracle import head as ohd
    from synth.configs import RoundCfg, TfCfg, HeadCfg
    tf = TfCfg(n_layers=1, d_model=128, n_heads=2, n_kv_heads=2, d_head=64, d_ff=256, max_pos=32)
    rc = RoundCfg(name="head-72", target=tf, draft=tf, head=HeadCfg(3, 256, 128, n_steps=2), K=8, max_batch=8, max_ctx=32,
                  entropy_layer=1, batch=8, n_ctx=8)
    case = build_case(rc, seed=7)
    ctx = make_ctx(case)
    n, D, S = 72, rc.head.d_latent, rc.head.n_steps
    z = gen.normal(14, "z72", (n, rc.head.d_cond), 1.0, rc.dtype)
    eps = gen.noise(14, "e72", (S + 1, n, D))
    mu, x = ctx.diffhead_decode(ctx.dev_store(z), ctx.dev_f32(eps))
    ctx.sync()
    mu_o, x_o = ohd.decode(rc.head, case.W, z, eps)
    assert rel_inf(mu.cpu().numpy(), mu_o) < 2e-2
    assert rel_inf(x.cpu().numpy(), x_o) < 2e-2
    ctx.close()


def test_head_closed_form_zero_weights():
    """All head weights zero except the output bias: mu = temperature*eps0 - b_out (1 step)."""
    case = build_case("ln-gelu-bf16", seed=1)
    case.rc.head.n_steps = 1
    for k in list(case.W):
        if k.startswith("head."):
            case.W[k] = np.zeros_like(case.W[k])
    b = gen.bf16_round(np.linspace(-1, 1, 16).astype(np.float32))
    case.W["head.out.b"] = b
    ctx = make_ctx(case)
    eps = gen.noise(9, "e", (2, 5, 16))
    z = gen.normal(9, "z", (5, case.rc.head.d_cond), 1.0, DT_BF16)
    mu, x = ctx.diffhead_decode(ctx.dev_store(z), ctx.dev_f32(eps))
    ctx.sync()
    assert np.allclose(mu.cpu().numpy(), eps[0] - b, atol=1e-6)
    assert np.allclose(x.cpu().numpy(), eps[0] - b + 0.25 * eps[1], atol=1e-6)
    ctx.close()


# ----------------------------------------------------------------------------- accept
def test_accept_matches_oracle_on_identical_inputs(ctx_bf16):
    from oracle import accept as oac
    ctx, case = ctx_bf16
    K, D, B = case.rc.K, 16, 64
    rng = np.random.default_rng(5)
    x = rng.normal(size=(B, K, D)).astype(np.float32)
    mu_q = (x + 0.2 * rng.normal(size=(B, K, D))).astype(np.float32)
    mu_p = np.concatenate([mu_q + 0.08 * rng.normal(size=(B, K, D)), rng.normal(size=(B, 1, D))], 1).astype(np.float32)
    r = rng.random((B, K)).astype(np.float32)
    r[0, 0] = 0.0
    n_keep = rng.integers(0, K + 1, size=B).astype(np.int32)
    for (ls, sp, sq) in [(0.0, 0.25, 0.25), (0.3, 0.3, 0.25)]:
        n_acc, lr, acc = ctx.spec_accept(ctx.dev_f32(x), ctx.dev_f32(mu_p), ctx.dev_f32(mu_q), ctx.dev_f32(r),
                                         ctx.dev_i32(n_keep), ls, sp, sq)
        ctx.sync()
        n_o, lr_o, acc_o = oac.accept(x, mu_p, mu_q, r, n_keep, ls, sp, sq)
        lr = lr.cpu().numpy()
        assert np.allclose(lr, lr_o, rtol=1e-4, atol=1e-3)
        with np.errstate(divide="ignore"):
            margin = np.abs(lr_o - np.log(r.astype(np.float64)))
        safe = margin > 1e-3 * np.maximum(1.0, np.abs(lr_o))
        assert np.array_equal(acc.cpu().numpy()[safe], acc_o[safe])
        rows_safe = safe.all(axis=1)
        assert np.array_equal(n_acc.cpu().numpy()[rows_safe], n_o[rows_safe])
        assert rows_safe.sum() > B // 2
    # equal means: ratio 1, everything kept is accepted
    mu_same = np.concatenate([mu_q, mu_q[:, :1]], 1)
    n_acc, lr, _ = ctx.spec_accept(ctx.dev_f32(x), ctx.dev_f32(mu_same), ctx.dev_f32(mu_q), ctx.dev_f32(r),
                                   ctx.dev_i32(n_keep), 0.0, 0.25, 0.25)
    ctx.sync()
    assert np.array_equal(n_acc.cpu().numpy(), n_keep)
    assert np.abs(lr.cpu().numpy()).max() == 0.0


def test_peak_probes_report_physical_rates(ctx_bf16):
    """The probes time real work: a read of a buffer far larger than every cache stays under the published HBM peak,
    the MFMA loop under the published bf16 peak, and both are within an order of magnitude of them."""
    import torch
    ctx, _ = ctx_bf16
    from paper_2512_08537_amd.binding import FardError
    buf = torch.zeros(1 << 28, device="cuda", dtype=torch.float32)      # 1 GiB
    torch.cuda.synchronize()
    ms, nbytes = ctx.spec_peak_probe(0, buf, reps=5)
    assert nbytes == float(1 << 30) and ms > 0
    gbs = nbytes / (ms * 1e-3) / 1e9
    assert 800.0 < gbs < 8000.0 * 1.02, gbs
    ms, flop = ctx.spec_peak_probe(1, iters=2048, reps=3)
    assert flop == 2048.0 * 16 * 2048 * 32768 and ms > 0
    tf = flop / (ms * 1e-3) / 1e12
    assert 250.0 < tf < 2500.0 * 1.02, tf
    with pytest.raises(FardError):
        ctx.spec_peak_probe(0, buf[1:9], reps=1)                   # 32 bytes at a 4-byte offset: misaligned
    with pytest.raises(FardError):
        ctx.spec_peak_probe(1, iters=0, reps=1)
    with pytest.raises(FardError):
        ctx.spec_peak_probe(2, buf, reps=1)
