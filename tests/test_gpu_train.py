"""GPU parity of the training step through softPPV (rocket_mse_grad, rocket_sgd_update,
rocket_train_step) and of kernel pruning (rocket_kernels_subset) against the CPU oracle.
Needs an MI355X."""
import numpy as np
import pytest

import oracle
from paper_2301_08527_amd import rocket
from parity import G_RTOL, check_forward, grad_scale_tol

pytestmark = pytest.mark.gpu


def _gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def test_mse_grad_matches_closed_form():
    import torch
    rng = np.random.default_rng(2)
    for B, p in ((1, 1), (3, 700), (64, 20000)):
        pred, y, coef = rng.standard_normal(B), rng.standard_normal(B).astype(np.float32), rng.standard_normal(p)
        g, loss = rocket.rocket_mse_grad(_gpu(pred), _gpu(y), _gpu(coef))
        torch.cuda.synchronize()
        # the head is linear: with F = pred as a single feature of weight 1 the oracle gives the residuals
        ref_loss, _ = oracle.mse_loss_grad(pred[:, None], y, np.ones(1), 0.0)
        r = pred - y.astype(np.float64)
        ref = (2.0 / B) * r[:, None] * coef[None, :]
        assert abs(float(loss.cpu()[0]) - ref_loss) <= 1e-12 * max(1.0, ref_loss)
        np.testing.assert_allclose(g.cpu().numpy(), ref, rtol=1e-6, atol=1e-30)


@pytest.mark.parametrize("recentre", [False, True])
def test_sgd_update_and_download(recentre):
    import torch
    rng = np.random.default_rng(4)
    B, C, L, K = 3, 4, 500, 200
    h = rocket.rocket_make_kernels(12, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    kr = {k: np.array(v) for k, v in kr.items()}           # detach from the handle's memory
    gw = rng.standard_normal(len(kr["weights"])).astype(np.float32)
    gb = rng.standard_normal(K).astype(np.float32)
    lr = 0.125
    print("sgd update", recentre, flush=True)
    rocket.rocket_sgd_update(h, _gpu(gw), _gpu(gb), lr, recentre)
    new = rocket.rocket_kernels_view_get(h)                # waits for the update and downloads
    w_ref, b_ref = oracle.sgd_update(kr, gw, gb, lr, recentre)
    np.testing.assert_allclose(new["weights"], w_ref, rtol=1e-6, atol=1e-6 if recentre else 1e-7)
    np.testing.assert_allclose(new["bias"], b_ref, rtol=1e-6, atol=1e-7)
    for name in ("length", "dilation", "padding", "n_ch", "channels"):
        assert np.array_equal(new[name], kr[name])
    # later transforms use the updated parameters
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    out = rocket.rocket_transform(h, _gpu(x), 7)
    torch.cuda.synchronize()
    check_forward(x, {k: np.array(v) for k, v in new.items()}, out.cpu().numpy(), 7)
    # host-side parameters set afterwards win again
    rocket.rocket_kernels_set_params(h, kr["weights"], kr["bias"])
    back = rocket.rocket_kernels_view_get(h)
    assert np.array_equal(back["weights"], kr["weights"]) and np.array_equal(back["bias"], kr["bias"])


def _unit_gradients(x, kr, mask, coef, lam):
    """per-series gradients for a unit residual: gw = sum_b r_b * U_b (the head is linear)"""
    B, K = x.shape[0], len(kr["length"])
    planes = bin(mask).count("1")
    g_soft = (2.0 / B) * coef[(planes - 1) * K:][None, :]
    g_max = (2.0 / B) * coef[:K][None, :] if mask & 1 else None
    return [oracle.backward(x[b:b + 1], kr, g_soft, g_max, lam=lam) for b in range(B)]


@pytest.mark.parametrize("mask,from_u8,recentre", [(4, False, False), (5, False, True), (7, True, False)])
def test_train_step_matches_the_oracle(mask, from_u8, recentre):
    import torch
    rng = np.random.default_rng(10 + mask)
    B, C, L, K = 4, 3, 700, 96
    lam, lr = 4.0, 0.25
    if from_u8:
        raw = rng.integers(0, 256, size=(B, C, L)).astype(np.uint8)
        x, x_in = oracle.znormalize_u8(raw), raw
    else:
        x = rng.standard_normal((B, C, L)).astype(np.float32)
        x_in = x
    h = rocket.rocket_make_kernels(21, K, C, L)
    kr = {k: np.array(v) for k, v in rocket.rocket_kernels_view_get(h).items()}
    planes = bin(mask).count("1")
    coef = rng.standard_normal(planes * K) * 0.2
    icpt, y = 0.3, rng.standard_normal(B).astype(np.float32)
    print("train step", mask, from_u8, recentre, flush=True)
    loss = rocket.rocket_train_step(h, _gpu(x_in), mask, _gpu(coef), _gpu(np.array([icpt])), _gpu(y), lr,
                                    lam=lam, recentre=recentre)
    new = rocket.rocket_kernels_view_get(h)
    loss = float(loss.cpu()[0])
    ref = oracle.train_step(x, kr, mask, y, coef, icpt, lr, lam=lam, recentre=recentre)

    # tolerance of the predictions: the feature tolerances through the linear head
    o = oracle.transform(x, kr, lam=lam)
    n = o["n_out"][None, :].astype(np.float64)
    tol = []
    if mask & 1:
        tol.append(1e-4 * np.abs(o["max"]) + 1e-5)
    if mask & 2:
        tol.append(o["ambiguous"] / n)
    tol.append(1e-4 * np.abs(o["softppv"]) + 1e-5)
    dpred = (np.abs(coef)[None, :] * np.concatenate(tol, axis=1)).sum(axis=1) + 1e-9
    F = oracle.feature_matrix(o, mask)
    r = F @ coef + icpt - y
    assert abs(loss - ref["loss"]) <= np.mean(2 * np.abs(r) * dpred + dpred ** 2) + 1e-12

    # tolerance of the gradients: the backward rule plus the residual error times the unit gradients
    U = _unit_gradients(x, kr, mask, coef, lam)
    gw_lin = sum(r[b] * U[b][0] for b in range(B))
    np.testing.assert_allclose(gw_lin, ref["grad_w"], rtol=1e-9, atol=1e-12)     # the decomposition itself
    slack_w = sum(dpred[b] * np.abs(U[b][0]) for b in range(B))
    slack_b = sum(dpred[b] * np.abs(U[b][1]) for b in range(B))
    stable = o["gap"].min(axis=0) > 1e-3 if mask & 1 else np.ones(K, bool)
    assert stable.sum() > K // 2
    centre_tol = 1e-6 if recentre else 0.0
    for k in np.nonzero(stable)[0]:
        lo, hi = int(kr["w_off"][k]), int(kr["w_off"][k + 1])
        scale = max(np.abs(ref["grad_w"][lo:hi]).max(), abs(ref["grad_b"][k]))
        gtol = G_RTOL * np.abs(ref["grad_w"][lo:hi]) + grad_scale_tol(lam) * scale + slack_w[lo:hi]
        if recentre:
            gtol = gtol + gtol.max()        # the removed row mean carries every element's error
        err = np.abs(new["weights"][lo:hi].astype(np.float64) - ref["weights"][lo:hi])
        assert np.all(err <= lr * gtol + 1e-6 * np.abs(ref["weights"][lo:hi]) + 1e-7 + centre_tol), (k, err.max())
        btol = G_RTOL * abs(ref["grad_b"][k]) + grad_scale_tol(lam) * scale + slack_b[k]
        assert abs(float(new["bias"][k]) - float(ref["bias"][k])) <= lr * btol + 1e-6 * abs(ref["bias"][k]) + 1e-7


def test_training_reduces_the_loss():
    """a few steps on a fixed batch: the loss before each update goes down"""
    import torch
    rng = np.random.default_rng(99)
    B, C, L, K, mask = 16, 3, 400, 128, 5
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(33, K, C, L)
    xd = _gpu(x)
    feats = rocket.rocket_transform(h, xd, mask, 4.0)
    y = _gpu((0.6 + 1.2 * rng.random(B)).astype(np.float32))
    coef, icpt = rocket.rocket_ridge_fit(feats, y, 10.0)
    losses = []
    for step in range(8):
        print("training step", step, flush=True)
        losses.append(rocket.rocket_train_step(h, xd, mask, coef, icpt, y, 0.05, lam=4.0, recentre=True))
    torch.cuda.synchronize()
    losses = [float(v.cpu()[0]) for v in losses]
    assert all(b < a for a, b in zip(losses, losses[1:])), losses
    # re-centred rows still sum to zero
    new = rocket.rocket_kernels_view_get(h)
    for k in range(K):
        ln, lo = int(new["length"][k]), int(new["w_off"][k])
        for c in range(int(new["n_ch"][k])):
            assert abs(float(new["weights"][lo + c * ln: lo + (c + 1) * ln].astype(np.float64).sum())) < 1e-5


def test_pruned_handle_gives_the_same_columns():
    import torch
    rng = np.random.default_rng(5)
    B, C, L, K = 3, 5, 3000, 400
    x = _gpu(rng.standard_normal((B, C, L)).astype(np.float32))
    h = rocket.rocket_make_kernels(8, K, C, L)
    keep = np.sort(rng.choice(K, size=150, replace=False)).astype(np.int32)
    hs = rocket.rocket_kernels_subset(h, keep)
    full = rocket.rocket_transform(h, x, 7)
    part = rocket.rocket_transform(hs, x, 7)
    torch.cuda.synchronize()
    full, part = full.cpu().numpy().reshape(B, 3, K), part.cpu().numpy().reshape(B, 3, len(keep))
    assert np.array_equal(full[:, :, keep], part)
