"""Pins the oracle's ridge regressor (no GPU needed): scikit-learn's Ridge as a library
opinion, closed forms, limits and invariances."""
import numpy as np
from sklearn.linear_model import Ridge

import oracle


def _data(seed, n, p):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((n, p)) * rng.uniform(0.5, 2.0, p) + rng.uniform(-1, 1, p)
    y = X[:, : min(p, 5)].sum(axis=1) * 0.3 + 1.5 + 0.1 * rng.standard_normal(n)
    return X, y


def test_matches_sklearn_ridge_tall_and_wide():
    """wrong centring, a penalised intercept or a transposed system all disagree with sklearn"""
    for n, p, alpha in ((60, 7, 0.5), (40, 40, 2.0), (25, 90, 1.0), (30, 200, 10.0)):
        X, y = _data(n + p, n, p)
        w, b = oracle.ridge_fit(X, y, alpha)
        ref = Ridge(alpha=alpha, fit_intercept=True, solver="svd").fit(X, y)
        np.testing.assert_allclose(w, ref.coef_, rtol=1e-8, atol=1e-10)
        assert abs(b - ref.intercept_) < 1e-9
        np.testing.assert_allclose(oracle.ridge_predict(X, w, b), ref.predict(X), rtol=1e-9, atol=1e-9)


def test_single_feature_closed_form():
    """p = 1: w = Sxy / (Sxx + alpha), b = ybar - xbar * w"""
    rng = np.random.default_rng(3)
    x = rng.standard_normal(50) + 2.0
    y = 3.0 * x - 1.0 + 0.05 * rng.standard_normal(50)
    alpha = 4.0
    w, b = oracle.ridge_fit(x[:, None], y, alpha)
    sxx = ((x - x.mean()) ** 2).sum()
    sxy = ((x - x.mean()) * (y - y.mean())).sum()
    assert abs(w[0] - sxy / (sxx + alpha)) < 1e-12
    assert abs(b - (y.mean() - x.mean() * w[0])) < 1e-12


def test_limits_and_invariances():
    X, y = _data(5, 80, 6)
    # alpha -> 0 with n > p: ordinary least squares
    w0, b0 = oracle.ridge_fit(X, y, 1e-10)
    sol = np.linalg.lstsq(np.c_[X, np.ones(len(y))], y, rcond=None)[0]
    np.testing.assert_allclose(np.r_[w0, b0], sol, rtol=1e-6, atol=1e-8)
    # alpha -> infinity: coefficients vanish, the intercept is the mean target
    wi, bi = oracle.ridge_fit(X, y, 1e12)
    assert np.abs(wi).max() < 1e-8 and abs(bi - y.mean()) < 1e-6
    # shifting the targets moves only the intercept; shifting a feature leaves w unchanged
    w1, b1 = oracle.ridge_fit(X, y, 3.0)
    w2, b2 = oracle.ridge_fit(X, y + 7.0, 3.0)
    np.testing.assert_allclose(w2, w1, atol=1e-12)
    assert abs(b2 - b1 - 7.0) < 1e-10
    Xs = X.copy()
    Xs[:, 2] += 5.0
    w3, b3 = oracle.ridge_fit(Xs, y, 3.0)
    np.testing.assert_allclose(w3, w1, atol=1e-10)
    assert abs(b3 - (b1 - 5.0 * w1[2])) < 1e-9
    # the penalty shrinks the coefficient norm monotonically
    norms = [np.linalg.norm(oracle.ridge_fit(X, y, a)[0]) for a in (0.1, 1.0, 10.0, 100.0)]
    assert all(norms[i] > norms[i + 1] for i in range(3))
