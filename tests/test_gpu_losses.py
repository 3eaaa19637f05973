"""GPU parity of the training-side losses (spec_entropy_loss, spec_smooth_l1) against oracle/losses.py, through the
C-ABI.  Inputs are bf16-rounded before either side sees them; the library accumulates scores in fp32 and rounds
dL/ds to bf16 for its second product, so entropies are held to 1e-3 (the bar of the inference indicator) and
gradients to the bf16 bar of the forward tests (max-rel 2e-2 over the tensor)."""
import numpy as np
import pytest

from synth import gen
from synth.configs import DT_BF16
from tests.harness import build_case, make_ctx, rel_inf

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def ctx():
    case = build_case("ln-gelu-bf16", seed=3)
    c = make_ctx(case)
    yield c
    c.close()


def _inputs(seed, B, H, Hkv, R, dh, std):
    q = gen.normal(seed, f"q{B}{H}{R}{dh}", (B, H, R, dh), std, DT_BF16)
    k = gen.normal(seed, f"k{B}{Hkv}{R}{dh}", (B, Hkv, R, dh), std, DT_BF16)
    return q, k


@pytest.mark.parametrize("B,H,Hkv,R,dh,std", [
    (1, 1, 1, 1, 32, 1.0),          # a single row: H = 0, no gradient
    (2, 2, 2, 32, 64, 1.0),         # exactly one tile
    (2, 3, 3, 33, 64, 1.5),         # ragged tail of one row
    (1, 4, 2, 95, 32, 1.0),         # grouped heads, ragged
    (2, 5, 1, 70, 128, 0.7),        # 5:1 groups, head dim 128
    (3, 4, 4, 256, 64, 1.2),        # several tiles, the sequence length of the 256-token setting
    (1, 2, 2, 300, 64, 2.0),        # peaky rows
    (32, 16, 16, 256, 64, 1.0),     # the shape kernel_bench times (draft of configs[1]: 16 heads, 256 tokens)
])
def test_entropy_loss_and_gradients_match_oracle(ctx, B, H, Hkv, R, dh, std):
    from oracle import losses
    q, k = _inputs(5, B, H, Hkv, R, dh, std)
    loss, hr, dq, dk = ctx.spec_entropy_loss(ctx.dev_store(q), ctx.dev_store(k))
    ctx.sync()
    lo, hro, dqo, dko = losses.attn_entropy_loss(q, k)
    eh = float(np.abs(hr.cpu().numpy() - hro).max())
    el = abs(float(loss.item()) - lo)
    print(f"H rows {eh:.2e} (range {hro.min():.2f}..{hro.max():.2f}), loss {el:.2e}")
    assert eh < 1e-3
    assert el < 1e-4
    if R > 1:
        eq, ek = rel_inf(dq.cpu().numpy(), dqo), rel_inf(dk.cpu().numpy(), dko)
        print(f"dq {eq:.2e} dk {ek:.2e}")
        assert eq < 2e-2 and ek < 2e-2
    else:
        # a single column: Omega = 1 up to the rounding of s - ln sum exp in fp32
        assert np.abs(dq.cpu().numpy()).max() < 1e-6 and np.abs(dk.cpu().numpy()).max() < 1e-6


def test_entropy_loss_outputs_are_optional_and_errors(ctx):
    from paper_2512_08537_amd.binding import FardError
    from oracle import losses
    q, k = _inputs(6, 1, 2, 2, 40, 64, 1.0)
    qd, kd = ctx.dev_store(q), ctx.dev_store(k)
    loss, hr, dq, dk = ctx.spec_entropy_loss(qd, kd, want_rows=False, want_dq=False, want_dk=True)
    ctx.sync()
    lo, _, _, dko = losses.attn_entropy_loss(q, k)
    assert hr is None and dq is None
    assert abs(float(loss.item()) - lo) < 1e-4
    assert rel_inf(dk.cpu().numpy(), dko) < 2e-2
    with pytest.raises(FardError):
        ctx.spec_entropy_loss(ctx.dev_store(q[..., :48]), ctx.dev_store(k[..., :48]))      # head dim 48
    with pytest.raises(FardError):
        ctx.spec_entropy_loss(ctx.dev_store(np.concatenate([q, q[:, :1]], axis=1)), kd)     # 3 heads over 2 kv heads


def test_entropy_loss_needs_a_bf16_context():
    from paper_2512_08537_amd.binding import FardError
    case = build_case("ln-gelu-f32", seed=3)
    c = make_ctx(case)
    x = c.dev_f32(np.zeros((1, 1, 32, 64), np.float32))
    with pytest.raises(FardError) as e:
        c.spec_entropy_loss(x, x)
    assert "FARD_ESTATE" in str(e.value)
    c.close()


@pytest.mark.parametrize("n,beta", [(1, 1.0), (257, 0.5), (100003, 1.0), (300000, 0.05)])
def test_smooth_l1_matches_oracle(ctx, n, beta):
    from oracle import losses
    p = gen.normal(7, f"p{n}", (n,), 1.0, DT_BF16)
    t = gen.normal(7, f"t{n}", (n,), 1.0, DT_BF16)
    loss, g = ctx.spec_smooth_l1(ctx.dev_store(p), ctx.dev_store(t), beta=beta)
    ctx.sync()
    lo, go = losses.smooth_l1(p, t, beta)
    assert float(loss.item()) == pytest.approx(lo, rel=2e-5)
    # elements within rounding of the kink may sit on either branch: both branches agree there to O(eps)
    assert np.allclose(g.cpu().numpy(), go, rtol=1e-5, atol=1e-6 / n)
