"""Pins for the oracle's LayerNorm-folded linear (the fused form of Sec. 5.5's LayerNorm + QKV
kernel): the identity against the separately pinned layer_norm and linear, a case worked by
hand, and the rule that the column sums follow the rounded weights."""
import numpy as np

from oracle import energon_oracle as O


def test_identity_against_layer_norm_then_linear():
    rng = np.random.default_rng(5)
    x = rng.normal(3.0, 2.0, (37, 96))            # a mean far from zero: the mu * c term matters
    w = rng.normal(0, 0.2, (50, 96)); b = rng.normal(0, 1, 50)
    g = rng.normal(1.0, 0.3, 96); beta = rng.normal(0, 0.5, 96)
    eps = 1e-5
    want = O.linear(O.layer_norm(x, g, beta, eps), w, b)
    mu, r = O.row_stats(x, eps)
    wf, c, bf = O.fold_layer_norm(w, b, g, beta)
    got = O.linear_ln_folded(x, wf, c, bf, mu, r)
    assert np.abs(got - want).max() <= 1e-11 * np.abs(want).max()
    # a dropped beta term, a dropped mean term or an unscaled weight must all show
    assert np.abs(O.linear_ln_folded(x, wf, c, bf - w @ beta, mu, r) - want).max() > 1e-3
    assert np.abs(O.linear_ln_folded(x, wf, 0 * c, bf, mu, r) - want).max() > 1e-3
    assert np.abs(O.linear_ln_folded(x, w, w.sum(1), bf, mu, r) - want).max() > 1e-3


def test_no_bias_is_zero_bias():
    rng = np.random.default_rng(6)
    w = rng.normal(0, 1, (4, 8)); g = rng.normal(1, 0.1, 8); beta = rng.normal(0, 1, 8)
    _, _, bf0 = O.fold_layer_norm(w, None, g, beta)
    _, _, bf1 = O.fold_layer_norm(w, np.zeros(4), g, beta)
    assert np.array_equal(bf0, bf1)


def test_hand_computed_case():
    # x = (1, 3): mean 2, variance 1, eps 0 -> r = 1, normalised (-1, 1).
    # gamma = (2, 1), beta = (0, 1) -> LayerNorm output (-2, 2).
    # W = [[1, 1], [0, 2]], b = (10, 20) -> y = (-2 + 2 + 10, 4 + 20) = (10, 24).
    x = np.array([[1.0, 3.0]]); g = np.array([2.0, 1.0]); beta = np.array([0.0, 1.0])
    w = np.array([[1.0, 1.0], [0.0, 2.0]]); b = np.array([10.0, 20.0])
    mu, r = O.row_stats(x, 0.0)
    assert mu[0] == 2.0 and r[0] == 1.0
    wf, c, bf = O.fold_layer_norm(w, b, g, beta)
    assert np.array_equal(wf, [[2.0, 1.0], [0.0, 2.0]])
    assert np.array_equal(c, [3.0, 2.0])
    assert np.array_equal(bf, [11.0, 22.0])
    assert np.array_equal(O.linear_ln_folded(x, wf, c, bf, mu, r), [[10.0, 24.0]])


def test_row_stats_closed_forms():
    # a constant row: variance 0, r = 1/sqrt(eps); the row 0..n-1: mean (n-1)/2, variance (n^2-1)/12
    mu, r = O.row_stats(np.full((1, 16), 7.0), 0.25)
    assert mu[0] == 7.0 and r[0] == 2.0
    n = 12
    mu, r = O.row_stats(np.arange(n, dtype=np.float64)[None, :], 0.0)
    assert mu[0] == (n - 1) / 2
    assert abs(r[0] - 1.0 / np.sqrt((n * n - 1) / 12.0)) < 1e-15


def test_column_sums_follow_the_rounded_weights():
    rng = np.random.default_rng(7)
    w = rng.normal(0, 1, (6, 64)); g = rng.normal(1, 0.2, 64); beta = np.zeros(64)
    rnd = lambda a: np.round(a * 8) / 8          # a coarse grid stands in for a 16-bit format
    wf, c, _ = O.fold_layer_norm(w, None, g, beta, round_weights=rnd)
    assert np.array_equal(wf, rnd(w * g))
    assert np.array_equal(c, wf.sum(axis=1))
    # with rounded weights the identity still holds exactly for THOSE weights
    x = rng.normal(1.0, 1.0, (5, 64)); mu, r = O.row_stats(x, 1e-5)
    want = O.linear((x - mu[:, None]) * r[:, None], wf, None)
    assert np.abs(O.linear_ln_folded(x, wf, c, np.zeros(6), mu, r) - want).max() < 1e-12
