"""Pins for the oracle's Alg. 1 loop, momentum rule (Sec. 4.2) and normalized variance (App. J).

The rules are checked against what fixes them from outside: closed forms of the linear recurrences that
heavy ball and Nesterov's method become on a quadratic, the plain step as the mu = 0 case, two-point
sample sets whose moments are known exactly, the exact two-point law of the quantizer (Def. 1), and
gradients the quantizer reproduces exactly, for which Alg. 1 must follow full-precision SGD.
"""
from fractions import Fraction

import numpy as np
import pytest

import oracle


def test_momentum_zero_mu_is_plain_step():
    rng = np.random.default_rng(1)
    w, yl, g = rng.standard_normal((3, 257))
    for l in (0.0, 0.5, 1.0):
        w1, yl1 = oracle.momentum_step(w, yl, g, 0.125, 0.0, l)
        assert np.array_equal(w1, w - 0.125 * g)
        assert np.array_equal(yl1, w - (l * 0.125) * g)


def _companion_closed_form(a: float, b: float, w0: float, w1: float, T: int) -> float:
    """w_T of w_{t+1} = a w_t + b w_{t-1} through the T-1'th power of the companion matrix."""
    M = np.array([[a, b], [1.0, 0.0]])
    return float((np.linalg.matrix_power(M, T - 1) @ np.array([w1, w0]))[0])


@pytest.mark.parametrize("l", [0.0, 1.0])
@pytest.mark.parametrize("alpha,mu,h", [(0.25, 0.5, 1.0), (0.0625, 0.875, 3.0), (0.5, 0.25, 0.75)])
def test_momentum_on_a_quadratic_matches_linear_recurrence(l, alpha, mu, h):
    # f(w) = h w^2 / 2, g = h w.  Heavy ball (l = 0): w_{t+1} = (1 + mu - alpha h) w_t - mu w_{t-1};
    # Nesterov (l = 1): w_{t+1} = (1 + mu)(1 - alpha h) w_t - mu (1 - alpha h) w_{t-1};
    # both start from y^l_0 = w_0, i.e. w_1 = (1 - alpha h - mu l alpha h) w_0.
    w0 = 1.75
    c = 1.0 - alpha * h
    a, b = ((1.0 + mu - alpha * h), -mu) if l == 0.0 else ((1.0 + mu) * c, -mu * c)
    w = np.array([w0])
    yl = w.copy()
    T = 25
    for _ in range(T):
        w, yl = oracle.momentum_step(w, yl, h * w, alpha, mu, l)
    assert w[0] == pytest.approx(_companion_closed_form(a, b, w0, (c - mu * l * alpha * h) * w0, T),
                                 rel=1e-11, abs=1e-14)


def test_heavy_ball_textbook_form():
    # w_{t+1} = w_t - alpha g_t + mu (w_t - w_{t-1}) with arbitrary gradients
    rng = np.random.default_rng(2)
    alpha, mu = 0.375, 0.75
    w_prev = w = rng.standard_normal(33)
    yl = w.copy()
    for t in range(6):
        g = rng.standard_normal(33)
        want = w - alpha * g + mu * (w - w_prev)
        w_prev = w
        w, yl = oracle.momentum_step(w, yl, g, alpha, mu, 0.0)
        np.testing.assert_allclose(w, want, rtol=0, atol=1e-14)


def test_normalized_variance_two_point_samples():
    # coordinate i takes m_i + a_i and m_i - a_i equally often: variance a_i^2, second moment m_i^2 + a_i^2
    m = np.array([1.0, -2.0, 0.5, 0.0])
    a = np.array([0.5, 1.0, 0.0, 3.0])
    x = np.stack([m + a, m - a] * 5)
    want = Fraction(1, 4) + 1 + 0 + 9
    want = want / (want + 1 + 4 + Fraction(1, 4) + 0)
    assert oracle.normalized_variance(x) == pytest.approx(float(want), rel=1e-14)


def test_normalized_variance_invariances():
    rng = np.random.default_rng(3)
    x = rng.standard_normal((40, 19)) + 0.3
    nv = oracle.normalized_variance(x)
    assert 0.0 < nv < 1.0
    assert oracle.normalized_variance(-2.5 * x) == pytest.approx(nv, rel=1e-13)
    assert oracle.normalized_variance(x[:, ::-1]) == pytest.approx(nv, rel=1e-13)
    assert oracle.normalized_variance(np.tile(x[:1], (8, 1))) < 1e-30       # no randomness: zero variance
    assert oracle.normalized_variance(x - x.mean(axis=0)) == pytest.approx(1.0, rel=1e-13)  # zero mean: all noise


def test_normalized_variance_of_the_quantizer_matches_def1():
    # Def. 1: Q(v)_i is norm * l_j or norm * l_{j+1}, the upper one with probability p = (r - l_j) / (l_{j+1} - l_j):
    # variance norm^2 (l_{j+1} - r)(r - l_j), second moment v_i^2 + variance.
    s, n = 3, 64
    rng = np.random.default_rng(4)
    v = (rng.standard_normal(n) * np.exp(rng.standard_normal(n))).astype(np.float32)
    norms = oracle.bucket_norms(v, n)
    norm = float(norms[0])
    lev = [float(x) for x in oracle.levels(s)]
    var = np.zeros(n)
    for i in range(n):
        r = abs(float(v[i])) / norm
        j = max(t for t in range(s + 1) if lev[t] <= r)
        var[i] = norm * norm * (lev[j + 1] - r) * (r - lev[j])
    want = var.sum() / (var.sum() + float((v.astype(np.float64) ** 2).sum()))
    M = 3000
    draws = np.stack([oracle.dequantize(oracle.quantize(v, n, s, 1000 + m, norms), n, s, norms) for m in range(M)])
    got = oracle.normalized_variance(draws)
    assert got == pytest.approx(want, rel=0.04)
    # the mean of the draws is v (unbiasedness), coordinate by coordinate, within 5 standard errors
    assert np.all(np.abs(draws.mean(axis=0) - v) <= 5 * np.sqrt(var / M) + 1e-7 * norm)


def test_alg1_follows_full_precision_sgd_when_quantization_is_exact():
    # gradient with one nonzero coordinate per bucket: r = 1 is the top level, Q(g) = g with certainty,
    # so w_T[i] = (1 - alpha h_i)^T w_0[i] on f(w) = sum_i h_i w_i^2 / 2 restricted to those coordinates
    n, nb, K, T, alpha = 16, 5, 3, 12, 0.25
    d = n * nb - 3
    hot = np.arange(nb) * n + np.array([0, 3, 7, 15, 2])
    h = np.zeros(d, dtype=np.float32)
    h[hot] = [1.0, 0.5, 2.0, 1.5, 0.25]
    w0 = np.linspace(-1.0, 1.0, d).astype(np.float32)

    def grad(w, t, k):
        return h * w

    for s in (1, 3):
        wT = oracle.data_parallel_sgd(w0, grad, K, T, alpha, n, s, seed0=77)
        want = w0.astype(np.float64) * (1.0 - alpha * h.astype(np.float64)) ** T
        np.testing.assert_allclose(wT, want, rtol=2e-6, atol=1e-30)
        cold = np.setdiff1d(np.arange(d), hot)
        assert np.array_equal(wT[cold], w0[cold])


def test_alg1_with_momentum_reduces_to_momentum_recurrence_when_exact():
    n, K, T, alpha, mu = 8, 2, 10, 0.25, 0.5
    h = np.zeros(n, dtype=np.float32)
    h[5] = 1.0
    w0 = np.ones(n, dtype=np.float32) * 0.75
    for l, (a, b) in ((0.0, (1.0 + mu - alpha, -mu)), (1.0, ((1.0 + mu) * (1 - alpha), -mu * (1 - alpha)))):
        wT = oracle.data_parallel_sgd(w0, lambda w, t, k: h * w, K, T, alpha, n, 3, seed0=5, mu=mu, l=l)
        assert wT[5] == pytest.approx(_companion_closed_form(a, b, 0.75, (1 - alpha - mu * l * alpha) * 0.75, T),
                                     rel=5e-6)
        assert np.all(wT[np.arange(n) != 5] == 0.75)


def test_alg1_step_is_unbiased_and_averaging_divides_the_variance():
    # one step from the same w with fresh seeds: the mean over runs is the full-precision step, and the spread
    # of the K-worker average is 1/K of one worker's (independent quantizers, Sec. 2)
    n, d, s, alpha = 32, 96, 3, 0.5
    rng = np.random.default_rng(6)
    w0 = rng.standard_normal(d).astype(np.float32)
    g = (rng.standard_normal(d) * 0.3).astype(np.float32)
    runs = 600

    def spread(K):
        ws = np.stack([oracle.data_parallel_sgd(w0, lambda w, t, k: g, K, 1, alpha, n, s, seed0=10_000 * K + 97 * r)
                       for r in range(runs)]).astype(np.float64)
        return ws.mean(axis=0), ws.var(axis=0).sum()

    m1, v1 = spread(1)
    m4, v4 = spread(4)
    full = w0.astype(np.float64) - alpha * g
    assert np.abs(m1 - full).max() < 5 * np.sqrt(v1 / d / runs) + 1e-6
    assert np.abs(m4 - full).max() < 5 * np.sqrt(v4 / d / runs) + 1e-6
    assert v1 / v4 == pytest.approx(4.0, rel=0.15)


def test_alg1_converges_on_least_squares():
    # strongly convex quadratic with per-worker noise: the quantized run reaches the noise floor of the
    # full-precision run (Theorem 4's message: same rate up to the variance blow-up), far below the start
    d, n, s, K, T, alpha = 256, 64, 3, 4, 300, 0.2
    rng = np.random.default_rng(8)
    hdiag = rng.uniform(0.5, 2.0, d).astype(np.float32)
    wstar = rng.standard_normal(d).astype(np.float32)
    noise = (0.01 * rng.standard_normal((T, K, d))).astype(np.float32)

    def grad(w, t, k):
        return hdiag * (w - wstar) + noise[t, k]

    loss = lambda w: 0.5 * float((hdiag.astype(np.float64) * (w.astype(np.float64) - wstar) ** 2).sum())
    w0 = np.zeros(d, dtype=np.float32)
    wq = oracle.data_parallel_sgd(w0, grad, K, T, alpha, n, s, seed0=123)
    wf = w0.copy()
    for t in range(T):
        wf = (wf - alpha * np.mean([grad(wf, t, k) for k in range(K)], axis=0)).astype(np.float32)
    assert loss(wq) < 1e-3 * loss(w0)
    assert loss(wf) < loss(wq) < 50 * loss(wf) + 1e-6
