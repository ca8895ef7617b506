"""Ridge regressor on the pooled features -- oracle side (paper section 3 part (3),
section 3.3: "a simple ridge regressor" on the 20,000 features).

TEST INFRASTRUCTURE ONLY: part of the CPU oracle; shares no code with the library.

The paper does not give the penalty or the treatment of the intercept; the reading
used here is the textbook one: minimise ||y - X w - b||^2 + alpha * ||w||^2 over
(w, b) with an unpenalised intercept b.  Written out plainly in fp64: centre the
columns of X and y, solve the normal equations (Xc^T Xc + alpha I) w = Xc^T yc,
and set b = mean(y) - mean(X) . w.  With more features than examples (the paper has
677 training examples and 20,000 features) the same w is obtained from the n x n
system  w = Xc^T (Xc Xc^T + alpha I)^-1 yc  (push-through identity), which is what makes
the full-size case computable; both branches are pinned against scikit-learn.
"""
import numpy as np


def ridge_fit(X, y, alpha):
    """Returns (w [p], b) in fp64 for features X (n x p) and targets y (n)."""
    X = np.asarray(X, dtype=np.float64)
    y = np.asarray(y, dtype=np.float64)
    n, p = X.shape
    if y.shape != (n,) or not alpha > 0:
        raise ValueError("need y of length n and alpha > 0")
    x_mean = X.mean(axis=0)
    y_mean = y.mean()
    Xc = X - x_mean
    yc = y - y_mean
    if p <= n:
        w = np.linalg.solve(Xc.T @ Xc + alpha * np.eye(p), Xc.T @ yc)
    else:
        w = Xc.T @ np.linalg.solve(Xc @ Xc.T + alpha * np.eye(n), yc)
    return w, y_mean - x_mean @ w


def ridge_predict(X, w, b):
    return np.asarray(X, dtype=np.float64) @ np.asarray(w, dtype=np.float64) + b
