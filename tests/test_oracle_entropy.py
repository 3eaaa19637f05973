"""Pins for oracle/entropy.py: closed forms, invariances, brute force (Eq. 1, S2.1, Sec. 4.3, Alg. 1 Step 1)."""
import math
import os

import numpy as np
import pytest

from oracle import entropy as ent
from oracle import loops

RNG = np.random.default_rng(1234)


def test_uniform_row_is_log_length():
    for L in (1, 2, 7, 256, 1280):
        for c in (0.0, 3.5, -100.0):
            assert ent.softmax_entropy(np.full(L, c)) == pytest.approx(math.log(L), abs=1e-12)


def test_one_hot_row_is_zero():
    row = np.zeros(1280)
    row[17] = 800.0
    assert ent.softmax_entropy(row) == pytest.approx(0.0, abs=1e-12)
    row[17] = 40.0          # finite gap: H = ln(1 + (L-1)e^-g) + g (L-1) e^-g / (1 + (L-1) e^-g)
    g, L = 40.0, 1280
    z = 1.0 + (L - 1) * math.exp(-g)
    want = math.log(z) + g * (L - 1) * math.exp(-g) / z
    assert ent.softmax_entropy(row) == pytest.approx(want, rel=1e-9)


def test_two_level_row_closed_form():
    # k entries at logit a, L-k at logit 0: p_hi = e^a/(k e^a + L-k), blocked entropy
    L, k, a = 64, 5, 2.3
    row = np.zeros(L)
    row[:k] = a
    z = k * math.exp(a) + (L - k)
    p_hi, p_lo = math.exp(a) / z, 1.0 / z
    want = -(k * p_hi * math.log(p_hi) + (L - k) * p_lo * math.log(p_lo))
    assert ent.softmax_entropy(row) == pytest.approx(want, rel=1e-12)


def test_binary_entropy():
    # two logits (x, 0): H = binary entropy of sigmoid(x)
    for x in (-3.0, 0.0, 0.7, 5.0):
        p = 1.0 / (1.0 + math.exp(-x))
        want = -(p * math.log(p) + (1 - p) * math.log(1 - p))
        assert ent.softmax_entropy(np.array([x, 0.0])) == pytest.approx(want, rel=1e-12)


def test_shift_and_permutation_invariance():
    row = RNG.normal(size=300) * 3
    h = ent.softmax_entropy(row)
    assert ent.softmax_entropy(row + 123.25) == pytest.approx(h, abs=1e-10)
    assert ent.softmax_entropy(RNG.permutation(row)) == pytest.approx(h, abs=1e-12)


def test_monotone_in_scale_and_small_beta_expansion():
    g = RNG.normal(size=1280)
    hs = [ent.softmax_entropy(b * g) for b in (0.0, 0.25, 0.5, 1, 2, 4, 8, 16)]
    assert all(a > b for a, b in zip(hs, hs[1:]))
    beta = 1e-2
    want = math.log(1280) - beta ** 2 * g.var() / 2.0
    assert ent.softmax_entropy(beta * g) == pytest.approx(want, abs=1e-7)


def test_matches_python_loops():
    for L in (1, 3, 50):
        row = RNG.normal(size=L) * 4
        assert ent.softmax_entropy(row) == pytest.approx(loops.entropy_loops(list(row)), rel=1e-12, abs=1e-14)


def test_batched_rows():
    rows = RNG.normal(size=(4, 6, 33))
    H = ent.softmax_entropy(rows)
    assert H.shape == (4, 6)
    assert H[2, 3] == pytest.approx(loops.entropy_loops(list(rows[2, 3])), rel=1e-12)


def test_online_triple_equals_two_pass():
    row = RNG.normal(size=137) * 5
    want = ent.softmax_entropy(row)
    for splits in ([], [1], [32, 64, 96, 128], [5, 6, 100], list(range(1, 137))):
        assert ent.online_entropy(row, splits) == pytest.approx(want, rel=1e-11)
    # increasing row forces a max update in every block
    inc = np.arange(64, dtype=float)
    assert ent.online_entropy(inc, [16, 32, 48]) == pytest.approx(ent.softmax_entropy(inc), rel=1e-11)


def test_l_entropy_sign_and_uniform_map():
    # S2.1: a uniform attention map with C visible columns gives L = -ln C (mean over heads and rows)
    N, R, C = 3, 5, 9
    a = np.full((N, R, C), 1.0 / C)
    assert ent.l_entropy(a) == pytest.approx(-math.log(C), rel=1e-12)
    # H = -L equals the mean row entropy
    logits = RNG.normal(size=(N, R, C))
    p = np.exp(logits) / np.exp(logits).sum(-1, keepdims=True)
    assert -ent.l_entropy(p) == pytest.approx(ent.softmax_entropy(logits).mean(), rel=1e-12)


def test_threshold_constant_stats_and_golden_example():
    assert ent.threshold(np.full(10, 7.12)) == pytest.approx(0.3 * 7.12, rel=1e-12)
    path = os.path.join(os.path.dirname(__file__), "golden", "threshold_example.txt")
    vals, want = None, None
    for line in open(path):
        if line.startswith("H:"):
            vals = [float(t) for t in line[2:].split()]
        if line.startswith("tau:"):
            want = float(line[4:])
    assert ent.threshold(vals) == pytest.approx(want, abs=1e-9)


def _prefilter_brute(H, tau):
    B, K = H.shape
    keep = np.zeros((B, K), np.uint8)
    for b in range(B):
        for i in range(K):
            keep[b, i] = all(H[b, j] >= tau for j in range(i + 1))
    return keep


def test_prefilter_prefix_rule_and_compaction():
    H = RNG.uniform(0, 2, size=(37, 8))
    tau = 0.6
    keep, n_keep, surv, n_surv = ent.prefilter(H, tau)
    assert np.array_equal(keep, _prefilter_brute(H, tau))
    assert n_keep.sum() == n_surv == len(surv)
    assert np.all(np.diff(surv) > 0)
    assert np.array_equal(np.flatnonzero(keep.reshape(-1)), surv)
    assert np.array_equal(n_keep, keep.sum(1))


def test_prefilter_edges():
    K = 4
    keep, n_keep, surv, n = ent.prefilter(np.full((3, K), 5.0), 1.0)
    assert keep.all() and n == 3 * K and np.array_equal(surv, np.arange(3 * K))
    H = np.full((2, K), 5.0)
    H[0, 0] = 0.0                       # first draft fails: nothing of sample 0 survives
    H[1, 2] = 0.0
    keep, n_keep, surv, n = ent.prefilter(H, 1.0)
    assert list(n_keep) == [0, 2] and list(surv) == [K + 0, K + 1]
    # tie: H == tau is kept (the paper stops on strict H < tau)
    keep, n_keep, _, _ = ent.prefilter(np.array([[1.0, 1.0]]), 1.0)
    assert list(n_keep) == [2]
    # recovery after a failure is ignored
    H = np.array([[5.0, 0.0, 5.0, 5.0]])
    keep, _, _, _ = ent.prefilter(H, 1.0)
    assert list(keep[0]) == [1, 0, 0, 0]
