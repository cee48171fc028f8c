"""Pins for the three shadow-sync rules: conservation laws, fixed points, contraction
factors and scalar recurrences that follow from Algorithms 2-4 by algebra."""
import numpy as np
import pytest

from oracle import sync


def _state(seed, K=4, P=37):
    rng = np.random.default_rng(seed)
    return (rng.standard_normal((K, P)), rng.standard_normal(P), rng.standard_normal(P),
            rng.standard_normal(P))


# ----------------------------------------------------------------------------- S-EASGD
@pytest.mark.parametrize("K", [1, 2, 4, 8])
def test_easgd_conserves_total_mass(K):
    W, w_ps, _, _ = _state(0, K)
    total = W.sum(axis=0) + w_ps
    for _ in range(3):
        sync.easgd_round(W, w_ps, 0.1)
    np.testing.assert_allclose(W.sum(axis=0) + w_ps, total, rtol=0, atol=1e-13)


def test_easgd_special_cases():
    W, w_ps, _, _ = _state(1, 3)
    W0, p0 = W.copy(), w_ps.copy()
    sync.easgd_round(W, w_ps, 0.0)                       # alpha = 0: nothing moves
    assert np.array_equal(W, W0) and np.array_equal(w_ps, p0)
    W1, p1 = W0[:1].copy(), p0.copy()                    # K = 1, alpha = 1/2: both -> average
    sync.easgd_round(W1, p1, 0.5)
    np.testing.assert_allclose(W1[0], (W0[0] + p0) / 2, atol=1e-15)
    np.testing.assert_allclose(p1, (W0[0] + p0) / 2, atol=1e-15)
    W2, p2 = W0[:1].copy(), p0.copy()                    # gap contracts by (1 - 2 alpha)
    sync.easgd_round(W2, p2, 0.1)
    np.testing.assert_allclose(W2[0] - p2, (1 - 0.2) * (W0[0] - p0), atol=1e-15)
    assert not np.allclose(W2[0], p2)                    # asymmetric: not equal afterwards
    We = np.tile(p0, (3, 1)); pe = p0.copy()             # all-equal state is a fixed point
    sync.easgd_round(We, pe, 0.3)
    assert np.array_equal(We, np.tile(p0, (3, 1))) and np.array_equal(pe, p0)


def test_easgd_replicas_meet_the_centre_in_ascending_order():
    W = np.array([[1.0], [0.0]]); w_ps = np.array([0.0])
    sync.easgd_round(W, w_ps, 0.5)
    # replica 0: delta = .5 -> centre .5, w0 = .5; replica 1 then sees centre .5:
    # delta = -.25 -> centre .25, w1 = .25
    assert W.ravel().tolist() == [0.5, 0.25] and w_ps.tolist() == [0.25]


def test_easgd_literal_variant_drifts_by_alpha_squared():
    W, w_ps, _, _ = _state(2, 1)
    W0, p0 = W.copy(), w_ps.copy()
    a = 0.2
    sync.easgd_round_literal(W, w_ps, a)
    np.testing.assert_allclose((W[0] + w_ps) - (W0[0] + p0), a * a * (W0[0] - p0), atol=1e-15)
    np.testing.assert_allclose(W[0] - w_ps, (1 - a) ** 2 * (W0[0] - p0), atol=1e-15)


# ----------------------------------------------------------------------------- S-MA
@pytest.mark.parametrize("alpha", [0.25, 0.5, 1.0])
def test_ma_preserves_mean_and_scales_deviation(alpha):
    W, _, wg, _ = _state(3, 5)
    mean0 = W.mean(axis=0)
    dev0 = W - mean0
    sync.ma_round(W, wg, alpha)
    np.testing.assert_allclose(W.mean(axis=0), mean0, atol=1e-14)
    np.testing.assert_allclose(W - mean0, (1 - alpha) * dev0, atol=1e-14)
    np.testing.assert_allclose(wg, mean0, atol=1e-14)


def test_ma_alpha_one_makes_all_replicas_the_mean_and_is_idempotent():
    W, _, wg, _ = _state(4, 4)
    mean0 = W.mean(axis=0)
    sync.ma_round(W, wg, 1.0)
    for i in range(4):
        np.testing.assert_allclose(W[i], mean0, atol=1e-15)
    W1 = W.copy()
    sync.ma_round(W, wg, 1.0)
    np.testing.assert_allclose(W, W1, atol=1e-15)
    Wk, _, wgk, _ = _state(5, 1)                          # K = 1: no-op
    Wk0 = Wk.copy()
    sync.ma_round(Wk, wgk, 0.7)
    np.testing.assert_allclose(Wk, Wk0, atol=1e-15)


# ----------------------------------------------------------------------------- S-BMUF
@pytest.mark.parametrize("alpha", [0.3, 1.0])
def test_bmuf_without_momentum_and_unit_step_is_ma(alpha):
    W, _, wg, v = _state(6, 4)
    Wm, wgm = W.copy(), wg.copy()
    v[:] = 0
    sync.bmuf_round(W, wg, v, alpha, eta=1.0, mu=0.0)
    sync.ma_round(Wm, wgm, alpha)
    np.testing.assert_allclose(W, Wm, atol=1e-14)
    np.testing.assert_allclose(wg, wgm, atol=1e-14)


def test_bmuf_plain_step_is_algorithm_4():
    """mu = 0: w_global moves a fraction eta of the way to the mean."""
    W, _, wg, v = _state(7, 3)
    v[:] = 0
    m, g0 = W.mean(axis=0), wg.copy()
    sync.bmuf_round(W, wg, v, 0.0, eta=0.4, mu=0.0)
    np.testing.assert_allclose(wg, g0 + 0.4 * (m - g0), atol=1e-14)


def test_bmuf_momentum_follows_scalar_recurrence_with_frozen_replicas():
    """alpha = 0 freezes the replicas, so e = w_global - mean obeys v <- mu v - eta e,
    e <- e + v."""
    W, _, wg, v = _state(8, 4, P=5)
    v[:] = 0
    m = W.mean(axis=0)
    mu, eta = 0.9, 0.5
    e = wg - m
    vs = np.zeros_like(e)
    for _ in range(6):
        sync.bmuf_round(W, wg, v, 0.0, eta, mu)
        vs = mu * vs - eta * e
        e = e + vs
        np.testing.assert_allclose(wg - m, e, atol=1e-13)
        np.testing.assert_allclose(v, vs, atol=1e-13)


def test_bmuf_fixed_point():
    w = np.random.default_rng(9).standard_normal(11)
    W = np.tile(w, (4, 1)); wg = w.copy(); v = np.zeros(11)
    sync.bmuf_round(W, wg, v, 0.5, 1.0, 0.9)
    assert np.array_equal(W, np.tile(w, (4, 1))) and np.array_equal(wg, w) and not v.any()


# ----------------------------------------------------------------------------- Nesterov BMUF
def test_bmuf_nesterov_without_momentum_is_bmuf():
    W, _, wg, v = _state(10, 4)
    v[:] = 0
    W2, wg2, v2 = W.copy(), wg.copy(), v.copy()
    for _ in range(3):
        sync.bmuf_nesterov_round(W, wg, v, 0.4, eta=0.7, mu=0.0)
        sync.bmuf_round(W2, wg2, v2, 0.4, eta=0.7, mu=0.0)
    np.testing.assert_allclose(W, W2, atol=1e-14)
    np.testing.assert_allclose(wg, wg2, atol=1e-14)


def test_bmuf_nesterov_pulls_towards_the_look_ahead_point():
    """Same w_global and v as plain BMUF from the same state; with alpha = 1 every replica
    lands on w_global + mu v, i.e. it differs from plain BMUF's replicas by exactly mu v."""
    W, _, wg, v = _state(11, 3, P=6)
    v[:] = np.random.default_rng(12).standard_normal(6) * 0.1
    W2, wg2, v2 = W.copy(), wg.copy(), v.copy()
    mu = 0.8
    sync.bmuf_nesterov_round(W, wg, v, 1.0, eta=0.5, mu=mu)
    sync.bmuf_round(W2, wg2, v2, 1.0, eta=0.5, mu=mu)
    np.testing.assert_allclose(wg, wg2, atol=1e-14)
    np.testing.assert_allclose(v, v2, atol=1e-14)
    np.testing.assert_allclose(W, W2 + mu * v2, atol=1e-14)
    np.testing.assert_allclose(W, np.tile(wg + mu * v, (3, 1)), atol=1e-14)


def test_bmuf_nesterov_single_trainer_scalar_recurrence():
    """K = 1, alpha = 1, eta = 1: the replica is the look-ahead point x = g + mu v, and the
    next round does v <- mu v + (x - g) = 2 mu v... written out: v' = mu v + mu v, g' = g + v',
    x' = g' + mu v'."""
    g, v, mu = 0.3, 0.05, 0.5
    x = g + mu * v
    W = np.array([[x]]); wg = np.array([g]); vv = np.array([v])
    for _ in range(5):
        sync.bmuf_nesterov_round(W, wg, vv, 1.0, 1.0, mu)
        v = mu * v + (x - g)
        g = g + v
        x = g + mu * v
        assert abs(wg[0] - g) < 1e-14 and abs(vv[0] - v) < 1e-14 and abs(W[0, 0] - x) < 1e-14


def test_bmuf_nesterov_fixed_point():
    w = np.random.default_rng(13).standard_normal(7)
    W = np.tile(w, (4, 1)); wg = w.copy(); v = np.zeros(7)   # K = 4: the mean is exact
    sync.bmuf_nesterov_round(W, wg, v, 0.5, 1.0, 0.9)
    assert np.array_equal(W, np.tile(w, (4, 1))) and np.array_equal(wg, w) and not v.any()
