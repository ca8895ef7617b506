"""Pins the oracle's training step (softPPV's gradient flow, paper section 3.2; training the
weights, section 6) without a GPU: central finite differences of the whole loss, the descent
property, closed forms of the update, and the vanishing gradient of a saturated sigmoid."""
import numpy as np
import pytest

import oracle


def _setup(mask, seed=3, B=3, C=3, L=120, K=24):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    kr = oracle.sample_kernels(seed + 100, K, C, L)
    planes = bin(mask).count("1")
    coef = rng.standard_normal(planes * K) * 0.3
    y = rng.standard_normal(B)
    return x, kr, coef, 0.25, y


def _with(kr, **changes):
    out = dict(kr)
    out.update(changes)
    return out


@pytest.mark.parametrize("mask", [4, 5, 7])
def test_gradient_matches_finite_differences_of_the_loss(mask):
    lam = 4.0
    x, kr, coef, icpt, y = _setup(mask)
    st = oracle.train_step(x, kr, mask, y, coef, icpt, lr=0.0, lam=lam)
    stable = oracle.transform(x, kr, lam=lam)["gap"].min(axis=0) > 1e-2 if mask & 1 else np.ones(len(kr["length"]), bool)
    h = 2.0 ** -9
    rng = np.random.default_rng(0)
    checked = 0
    for k in rng.permutation(len(kr["length"])):
        if not stable[k]:
            continue
        lo, hi = int(kr["w_off"][k]), int(kr["w_off"][k + 1])
        for idx in (lo, hi - 1, None):                      # first and last weight, then the bias
            name = "bias" if idx is None else "weights"
            i = k if idx is None else idx
            up, dn = np.array(kr[name], np.float32), np.array(kr[name], np.float32)
            up[i] += h
            dn[i] -= h
            fd = (oracle.loss_of(x, _with(kr, **{name: up}), mask, y, coef, icpt, lam=lam)
                  - oracle.loss_of(x, _with(kr, **{name: dn}), mask, y, coef, icpt, lam=lam)) / (float(up[i]) - float(dn[i]))
            an = st["grad_b"][k] if idx is None else st["grad_w"][idx]
            scale = max(np.abs(st["grad_w"][lo:hi]).max(), abs(st["grad_b"][k]))
            assert abs(fd - an) <= 2e-3 * scale + 1e-9, (k, name, fd, an)
        checked += 1
        if checked == 6:
            break
    assert checked == 6


def test_a_small_step_descends_by_lr_times_squared_gradient():
    mask, lam = 5, 4.0
    x, kr, coef, icpt, y = _setup(mask, seed=8)
    lr = 2.0 ** -10
    st = oracle.train_step(x, kr, mask, y, coef, icpt, lr=lr, lam=lam)
    after = oracle.loss_of(x, _with(kr, weights=st["weights"], bias=st["bias"]), mask, y, coef, icpt, lam=lam)
    drop = st["loss"] - after
    first_order = lr * (np.sum(st["grad_w"] ** 2) + np.sum(st["grad_b"] ** 2))
    assert drop > 0
    assert abs(drop - first_order) <= 0.1 * first_order
    # loss reported is the one before the update
    assert st["loss"] == pytest.approx(oracle.loss_of(x, kr, mask, y, coef, icpt, lam=lam), rel=1e-12)


def test_update_closed_forms():
    x, kr, coef, icpt, y = _setup(4)
    nw, K = len(kr["weights"]), len(kr["length"])
    rng = np.random.default_rng(1)
    gw, gb = rng.standard_normal(nw), rng.standard_normal(K)
    w0, b0 = oracle.sgd_update(kr, gw, gb, 0.0)
    assert np.array_equal(w0, kr["weights"]) and np.array_equal(b0, kr["bias"])
    w1, b1 = oracle.sgd_update(kr, gw, gb, 0.5)
    np.testing.assert_allclose(w1, np.asarray(kr["weights"], np.float64) - 0.5 * gw, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(b1, np.asarray(kr["bias"], np.float64) - 0.5 * gb, rtol=1e-6, atol=1e-7)
    # re-centring: rows sum to zero, the bias is untouched, and only the row means of the step are removed
    w2, b2 = oracle.sgd_update(kr, gw, gb, 0.5, recentre=True)
    assert np.array_equal(b2, b1)
    for k in range(K):
        ln, lo = int(kr["length"][k]), int(kr["w_off"][k])
        for c in range(int(kr["n_ch"][k])):
            sl = slice(lo + c * ln, lo + (c + 1) * ln)
            assert abs(w2[sl].astype(np.float64).sum()) < 1e-5
            np.testing.assert_allclose(w2[sl], w1[sl].astype(np.float64) - w1[sl].astype(np.float64).mean(), atol=1e-6)


def test_mse_gradient_closed_form():
    F = np.array([[1.0, 2.0], [0.5, -1.0]])
    coef, icpt, y = np.array([2.0, -1.0]), 0.5, np.array([1.0, 0.0])
    loss, G = oracle.mse_loss_grad(F, y, coef, icpt)
    # predictions 0.5 and 2.5 -> residuals -0.5 and 2.5
    assert loss == pytest.approx((0.25 + 6.25) / 2)
    np.testing.assert_allclose(G, [[-1.0, 0.5], [5.0, -2.5]])


def test_saturated_sigmoid_passes_almost_no_gradient():
    """large |lambda*y + shift| everywhere: s(1-s) <= exp(-|z|), so the update vanishes (section 3.2)"""
    mask, lam = 4, 10.0
    x, kr, coef, icpt, y = _setup(mask, seed=5)
    plain = oracle.train_step(x, kr, mask, y, coef, icpt, lr=0.0, lam=lam)
    assert np.abs(plain["grad_b"]).max() > 1e-3
    # every output pushed far into the positive tail of the sigmoid
    far = _with(kr, bias=(np.asarray(kr["bias"]) + 200.0).astype(np.float32))
    sat = oracle.train_step(x, far, mask, y, coef, icpt, lr=0.0, lam=lam)
    assert np.abs(sat["grad_b"]).max() < 1e-100 and np.abs(sat["grad_w"]).max() < 1e-100
    # moderately saturated (inputs scaled by 5): per kernel
    # |grad_b| <= sum_b |G_bk| * lam * mean_t exp(-|lam*y_t + shift|), and the sum shrinks
    xs = 5.0 * x
    mid = oracle.train_step(xs, kr, mask, y, coef, icpt, lr=0.0, lam=lam)
    o = oracle.transform(xs, kr, lam=lam)
    _, G = oracle.mse_loss_grad(oracle.feature_matrix(o, mask), y, coef, icpt)
    for k in range(len(kr["length"])):
        bound = 0.0
        for b in range(x.shape[0]):
            z = lam * oracle.conv_output(xs[b], kr, k) - 3.0
            bound += abs(G[b, k]) * lam * np.mean(np.exp(-np.abs(z)))
        assert abs(mid["grad_b"][k]) <= bound * (1 + 1e-9) + 1e-300
