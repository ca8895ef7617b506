"""GPU parity of rocket_ridge_fit / rocket_ridge_predict against the oracle's ridge
regressor (needs an MI355X).  Both sides work in fp64 on the same fp32 features, so the
results agree to rounding-order level."""
import numpy as np
import pytest

import oracle
import synth
from paper_2301_08527_amd import rocket

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
                                       (257, 1000, 10.0), (100, 65, 1e-3), (32, 17, 1.0), (31, 16, 1.0), (65, 2003, 0.5),
                                       (300, 1003, 1.0), (1500, 300, 1.0), (4500, 64, 3.0)])
def test_small_systems(n, p, alpha):
    """sizes around the 32-column panels and 64-row tiles of the factorisation, feature counts that are no
    multiple of 4 or 16, more examples than features, and more examples than one workgroup's LDS could hold"""
    print("ridge", n, p, alpha, flush=True)
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
        rocket.rocket_ridge_fit(torch.zeros(32769, 2, device="cuda"), torch.zeros(32769, device="cuda"), 1.0)
    with pytest.raises(rocket.RocketError):
        rocket.rocket_ridge_fit(X, y, 1.0, workspace=torch.empty(256, dtype=torch.uint8, device="cuda"))


def _oracle_features(z, kr, mask):
    """(B, F*K) fp64 feature matrix in the library's plane order, and its per-entry parity tolerance"""
    o = oracle.transform(z, kr)
    n = o["n_out"][None, :].astype(np.float64)
    cols, tols = [], []
    if mask & 1:
        cols.append(o["max"]); tols.append(1e-4 * np.abs(o["max"]) + 1e-5)
    if mask & 2:
        cols.append(o["count"] / n); tols.append(o["ambiguous"] / n)
    if mask & 4:
        cols.append(o["softppv"]); tols.append(1e-4 * np.abs(o["softppv"]) + 1e-5)
    return np.concatenate(cols, axis=1), np.concatenate(tols, axis=1)


@pytest.mark.parametrize("mask", [3, 7])
def test_infer_from_bytes_to_prediction(mask):
    """The whole model in one call: raw 8-bit examples -> features -> ridge prediction, against
    the oracle pipeline (z-normalise, transform, fit, predict) with the oracle's coefficients."""
    import torch
    rng = np.random.default_rng(123)
    n_train, n_test, C, L, K = 48, 9, 4, 801, 300
    raw = rng.integers(0, 256, size=(n_train + n_test, C, L)).astype(np.uint8)
    smooth = rng.random(n_train + n_test)                      # per-example roughness-like factor
    for i, s in enumerate(smooth):                              # smoother examples have a lower target
        w = 1 + int(12 * (1 - s))
        raw[i] = np.clip(np.apply_along_axis(lambda r: np.convolve(r, np.ones(w) / w, "same"), -1,
                                             raw[i].astype(np.float64)), 0, 255).astype(np.uint8)
    y = (0.6 + 1.2 * smooth).astype(np.float32)
    h = rocket.rocket_make_kernels(55, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    z = oracle.znormalize_u8(raw)
    F_ref, F_tol = _oracle_features(z, kr, mask)
    w_ref, b_ref = oracle.ridge_fit(F_ref[:n_train].astype(np.float32), y[:n_train], 1.0)
    pred_ref = oracle.ridge_predict(F_ref[n_train:].astype(np.float32), w_ref, b_ref)

    coef = torch.from_numpy(w_ref).cuda()
    icpt = torch.tensor([b_ref], dtype=torch.float64, device="cuda")
    x_test = torch.from_numpy(raw[n_train:]).cuda()
    print("infer u8", mask, flush=True)
    pred, feats = rocket.rocket_infer(h, x_test, mask, coef, icpt)
    torch.cuda.synchronize()
    # composition: the same bits as the two separate calls
    feats2 = rocket.rocket_transform_u8(h, x_test, mask)
    pred2 = rocket.rocket_ridge_predict(feats2, coef, icpt)
    torch.cuda.synchronize()
    assert torch.equal(feats, feats2) and torch.equal(pred, pred2)
    # parity with the oracle pipeline: the feature tolerances propagated through the linear model
    bound = (np.abs(w_ref)[None, :] * (F_tol[n_train:] + 1e-7 * np.abs(F_ref[n_train:]))).sum(axis=1) + 1e-8
    err = np.abs(pred.cpu().numpy() - pred_ref)
    assert np.all(err <= bound), (err, bound)
    # the model is a model: it ranks the held-out examples by the planted roughness factor
    assert np.corrcoef(pred_ref, y[n_train:])[0, 1] > 0.8
    # float32 input through the same entry point
    pred_f, _ = rocket.rocket_infer(h, torch.from_numpy(z[n_train:]).cuda(), mask, coef, icpt)
    torch.cuda.synchronize()
    assert np.all(np.abs(pred_f.cpu().numpy() - pred_ref) <= bound)
