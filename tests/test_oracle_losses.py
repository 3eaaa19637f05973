"""Pins for oracle/losses.py (the draft's training losses: L_entropy of Sec. 3 / S2.1 and the Smooth-L1 L_reg)."""
import math

import numpy as np
import pytest

from oracle import entropy as ent
from oracle import losses

RNG = np.random.default_rng(77)


def _qk(B=2, H=4, Hkv=2, R=9, dh=8, scale=1.0):
    return RNG.normal(size=(B, H, R, dh)) * scale, RNG.normal(size=(B, Hkv, R, dh)) * scale


def test_zero_queries_give_log_count_entropies_and_zero_gradient():
    """q = 0: every causal row is uniform over its r+1 columns: H_r = ln(r+1), the maximum, where the gradient
    vanishes."""
    q, k = _qk()
    q[:] = 0.0
    loss, Hr, dq, dk = losses.attn_entropy_loss(q, k)
    want = np.log(np.arange(1, q.shape[2] + 1))
    assert np.allclose(Hr, want[None, None, :], atol=1e-12)
    assert loss == pytest.approx(-want.mean(), abs=1e-12)
    assert np.abs(dq).max() < 1e-15 and np.abs(dk).max() < 1e-15


def test_loss_is_the_l_entropy_of_the_softmax_rows():
    """Against the S2.1 formula applied to explicitly built causal softmax rows (one batch element), by the
    function that the inference indicator's pins already cover."""
    q, k = _qk(B=1, H=3, Hkv=3, R=7, dh=4, scale=2.0)
    loss, Hr, _, _ = losses.attn_entropy_loss(q, k)
    maps = np.zeros((3, 7, 7))
    for h in range(3):
        for r in range(7):
            s = np.array([q[0, h, r] @ k[0, h, c] / math.sqrt(4) for c in range(r + 1)])
            p = np.exp(s - s.max())
            maps[h, r, :r + 1] = p / p.sum()
            assert Hr[0, h, r] == pytest.approx(ent.softmax_entropy(s), abs=1e-12)
    assert loss == pytest.approx(ent.l_entropy(maps), abs=1e-12)


@pytest.mark.parametrize("H,Hkv", [(4, 4), (4, 2), (6, 1)])
def test_gradients_match_central_differences(H, Hkv):
    q, k = _qk(B=2, H=H, Hkv=Hkv, R=6, dh=4, scale=1.5)
    _, _, dq, dk = losses.attn_entropy_loss(q, k)
    eps = 1e-6
    for arr, grad in ((q, dq), (k, dk)):
        idx = [tuple(RNG.integers(0, n) for n in arr.shape) for _ in range(25)]
        for i in idx:
            old = arr[i]
            arr[i] = old + eps
            lp = losses.attn_entropy_loss(q, k)[0]
            arr[i] = old - eps
            lm = losses.attn_entropy_loss(q, k)[0]
            arr[i] = old
            assert grad[i] == pytest.approx((lp - lm) / (2 * eps), rel=1e-5, abs=1e-9)


def test_future_keys_and_queries_do_not_leak():
    """Causality: row r's entropy and dq_r do not change when later keys change; dk of the last key only sees
    the last row."""
    q, k = _qk(B=1, H=2, Hkv=2, R=8, dh=4)
    _, H0, dq0, dk0 = losses.attn_entropy_loss(q, k)
    k2 = k.copy()
    k2[:, :, 5:] += 3.0
    _, H1, dq1, _ = losses.attn_entropy_loss(q, k2)
    assert np.array_equal(H0[:, :, :5], H1[:, :, :5]) and np.array_equal(dq0[:, :, :5], dq1[:, :, :5])
    q2 = q.copy()
    q2[:, :, :7] = 0.0                                   # only the last row keeps a non-uniform distribution
    _, _, _, dk2 = losses.attn_entropy_loss(q2, k)
    q3 = q2.copy()
    q3[:, :, 7] = 0.0
    assert np.abs(losses.attn_entropy_loss(q3, k)[3]).max() < 1e-15
    assert np.abs(dk2[:, :, 7]).max() > 0


def test_shift_of_all_keys_along_a_query_changes_nothing():
    """Softmax rows are invariant to adding a constant to a row's scores: k_c -> k_c + v adds q_r . v to every
    score of row r."""
    q, k = _qk(B=1, H=2, Hkv=1, R=7, dh=4)
    v = RNG.normal(size=4)
    a = losses.attn_entropy_loss(q, k)
    b = losses.attn_entropy_loss(q, k + v)
    assert a[0] == pytest.approx(b[0], abs=1e-12)
    assert np.allclose(a[1], b[1], atol=1e-12)
    # ... and therefore dL/dv = sum_c dL/dk_c must vanish for every direction v
    assert np.allclose(a[3].sum(axis=2), 0.0, atol=1e-12)


def test_smooth_l1_values_branches_and_gradient():
    pred = np.array([0.0, 0.25, -0.5, 2.0, -3.0, 1.0])
    tgt = np.zeros(6)
    loss, g = losses.smooth_l1(pred, tgt, beta=1.0)
    per = [0.0, 0.03125, 0.125, 1.5, 2.5, 0.5]
    assert loss == pytest.approx(sum(per) / 6, abs=1e-15)
    assert np.allclose(g * 6, [0.0, 0.25, -0.5, 1.0, -1.0, 1.0])
    # beta -> 0 is the L1 loss; large beta is 0.5 d^2 / beta
    loss, _ = losses.smooth_l1(pred, tgt, beta=1e-12)
    assert loss == pytest.approx(np.abs(pred).mean(), abs=1e-9)
    loss, _ = losses.smooth_l1(pred, tgt, beta=100.0)
    assert loss == pytest.approx((0.5 * pred ** 2 / 100.0).mean(), abs=1e-15)
    # gradient by central differences away from the kinks
    p = RNG.normal(size=50) * 2
    t = RNG.normal(size=50)
    _, g = losses.smooth_l1(p, t, beta=0.7)
    for i in range(50):
        if abs(abs(p[i] - t[i]) - 0.7) < 1e-3:
            continue
        pp, pm = p.copy(), p.copy()
        pp[i] += 1e-6
        pm[i] -= 1e-6
        fd = (losses.smooth_l1(pp, t, 0.7)[0] - losses.smooth_l1(pm, t, 0.7)[0]) / 2e-6
        assert g[i] == pytest.approx(fd, rel=1e-6, abs=1e-10)
