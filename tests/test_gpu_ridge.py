"""GPU parity of rocket_ridge_fit / rocket_ridge_predict against the oracle's ridge
regressor (needs an MI355X).  Both sides work in fp64 on the same fp32 features, so the
results agree to rounding-order level."""
import numpy as np
import pytest

import oracle
from paper_2301_08527_amd import rocket, synth

pytestmark = pytest.mark.gpu


def _fit(X, y, alpha):
    import torch
    Xd, yd = torch.from_numpy(X).cuda(), torch.from_numpy(y).cuda()
    coef, b = rocket.rocket_ridge_fit(Xd, yd, alpha)
    pred = rocket.rocket_ridge_predict(Xd, coef, b)
    torch.cuda.synchronize()
    return coef.cpu().numpy(), float(b.cpu().numpy()[0]), pred.cpu().numpy()


def _check(X, y, alpha):
    w, b, pred = _fit(X, y, alpha)
    w_ref, b_ref = oracle.ridge_fit(X, y, alpha)
    scale = max(np.abs(w_ref).max(), 1e-30)
    assert np.abs(w - w_ref).max() <= 1e-8 * scale, np.abs(w - w_ref).max() / scale
    assert abs(b - b_ref) <= 1e-8 * max(1.0, abs(b_ref))
    ref_pred = oracle.ridge_predict(X, w_ref, b_ref)
    assert np.abs(pred - ref_pred).max() <= 1e-8 * max(1.0, np.abs(ref_pred).max())


@pytest.mark.parametrize("n,p,alpha", [(1, 3, 1.0), (2, 1, 0.5), (33, 31, 0.1), (64, 40, 2.0), (120, 500, 1.0),
                                       (257, 1000, 10.0), (100, 65, 1e-3)])
def test_small_systems(n, p, alpha):
    rng = np.random.default_rng(n * 1000 + p)
    X = (rng.standard_normal((n, p)) * rng.uniform(0.2, 3.0, p) + rng.uniform(-2, 2, p)).astype(np.float32)
    y = (X[:, : min(p, 4)].sum(axis=1) * 0.25 + 1.0 + 0.05 * rng.standard_normal(n)).astype(np.float32)
    _check(X, y, alpha)


def test_paper_sized_fit_on_transform_features():
    """677 training examples x 20,000 features, the paper's sizes (sections 3.3 and 4):
    features of a short synthetic workload, max + PPV planes of K = 10,000 kernels"""
    import torch
    n, C, L, K = 677, 3, 400, 10000
    rng = np.random.default_rng(77)
    x = rng.standard_normal((n, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(5, K, C, L)
    feats = rocket.rocket_transform(h, torch.from_numpy(x).cuda(), 3)
    torch.cuda.synchronize()
    X = feats.cpu().numpy()
    assert X.shape == (n, 2 * K)
    y = (0.6 + 1.2 * rng.random(n)).astype(np.float32)       # roughness-like targets in [0.6, 1.8]
    print("ridge paper-sized fit", flush=True)
    _check(X, y, 1.0)


def test_argument_errors():
    import torch
    X = torch.zeros(4, 3, device="cuda")
    y = torch.zeros(4, device="cuda")
    for alpha in (0.0, -1.0, float("nan")):
        with pytest.raises(rocket.RocketError):
            rocket.rocket_ridge_fit(X, y, alpha)
    with pytest.raises(rocket.RocketError):
        rocket.rocket_ridge_fit(torch.zeros(5000, 2, device="cuda"), torch.zeros(5000, device="cuda"), 1.0)
    with pytest.raises(rocket.RocketError):
        rocket.rocket_ridge_fit(X, y, 1.0, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))
