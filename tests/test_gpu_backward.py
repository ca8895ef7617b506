"""GPU parity of rocket_soft_ppv_backward against the CPU oracle (needs an MI355X)."""
import numpy as np
import pytest

import oracle
from paper_2301_08527_amd import rocket, synth
from parity import check_backward

pytestmark = pytest.mark.gpu


def _gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _backward(h, x, mask, grad_out, lam, shift, include_max):
    import torch
    gw, gb = rocket.rocket_soft_ppv_backward(h, _gpu(x), mask, _gpu(grad_out), lam, shift, include_max)
    torch.cuda.synchronize()
    return gw.cpu().numpy(), gb.cpu().numpy()


def _split(grad_out, mask, K):
    """(g_soft, g_max) planes of an upstream gradient laid out like the forward output."""
    F = rocket.rocket_num_features(mask)
    g_soft = grad_out[:, (F - 1) * K:F * K]
    g_max = grad_out[:, :K] if mask & 1 else None
    return g_soft, g_max


def _stable_argmax(x, kr, sel=None):
    """kernels whose maximum is separated from the runner-up, so fp32 and fp64 agree on where it is"""
    o = oracle.transform(x, kr, sel=sel)
    return o["gap"].min(axis=0) > 1e-3


@pytest.mark.parametrize("mask,include_max", [(4, False), (5, False), (5, True), (7, True), (6, False)])
def test_small_all_kernels(mask, include_max):
    rng = np.random.default_rng(31)
    B, C, L, K = 4, 6, 1500, 160
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(41, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    F = rocket.rocket_num_features(mask)
    grad_out = rng.standard_normal((B, F * K)).astype(np.float32)
    lam, shift = 4.0, -3.0
    print("backward small", mask, include_max, flush=True)
    gw, gb = _backward(h, x, mask, grad_out, lam, shift, include_max)
    g_soft, g_max = _split(grad_out, mask, K)
    sel = None
    if include_max:
        sel = np.nonzero(_stable_argmax(x, kr))[0].astype(np.int32)
        assert len(sel) > K // 2
    rep = {}
    check_backward(x, kr, gw, gb, g_soft, g_max if include_max else None, lam, shift, sel=sel, report=rep)
    print("worst error / bound:", rep["worst_ratio"], flush=True)


@pytest.mark.parametrize("lam,shift", [(0.0, -3.0), (1.0, -3.0), (10.0, -3.0), (100.0, -3.0), (10.0, 3.0)])
def test_lambda_sweep(lam, shift):
    rng = np.random.default_rng(32)
    B, C, L, K = 3, 3, 700, 90
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(42, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    grad_out = rng.standard_normal((B, K)).astype(np.float32)
    gw, gb = _backward(h, x, 4, grad_out, lam, shift, False)
    check_backward(x, kr, gw, gb, grad_out, None, lam, shift)
    if lam == 0.0:
        assert np.all(gw == 0) and np.all(gb == 0)


def test_shortest_series_and_single_positions():
    rng = np.random.default_rng(33)
    for (B, C, L, K) in ((2, 1, 11, 30), (1, 9, 61, 60), (3, 2, 130, 60)):
        x = rng.standard_normal((B, C, L)).astype(np.float32)
        h = rocket.rocket_make_kernels(43, K, C, L)
        kr = rocket.rocket_kernels_view_get(h)
        grad_out = rng.standard_normal((B, K)).astype(np.float32)
        gw, gb = _backward(h, x, 4, grad_out, 3.0, -3.0, False)
        check_backward(x, kr, gw, gb, grad_out, None, 3.0, -3.0)


def test_config3_full_size_sample():
    """B=60 x 20 x 50,000, K=10,000: forward max+softPPV then backward with the max
    sub-gradient, in the launch shape the benchmark times; the oracle checks a
    dilation-stratified sample of kernels summed over the whole batch."""
    import torch
    cfg = synth.CONFIGS[3]
    B, K, mask = cfg["B"], cfg["K"], cfg["features"]
    x = synth.make_input(3)
    h = rocket.rocket_make_kernels(synth.seed_k(3), K, cfg["C"], cfg["L"])
    kr = rocket.rocket_kernels_view_get(h)
    grad_out = synth.make_upstream_grad(3, B, 2 * K)
    print("config3 backward run", flush=True)
    xd = _gpu(x)
    gw, gb = rocket.rocket_soft_ppv_backward(h, xd, mask, _gpu(grad_out), 10.0, -3.0, True)
    torch.cuda.synchronize()
    gw, gb = gw.cpu().numpy(), gb.cpu().numpy()
    sel = synth.pick_kernels(kr, 48, seed=3)
    stable = _stable_argmax(x, kr, sel=sel)
    sel = sel[stable]
    assert len(sel) >= 24
    g_soft, g_max = _split(grad_out, mask, K)
    rep = {}
    check_backward(x, kr, gw, gb, g_soft, g_max, 10.0, -3.0, sel=sel, report=rep)
    print("config3 worst error / bound:", rep["worst_ratio"], flush=True)
    # without the max plane
    gw2, gb2 = rocket.rocket_soft_ppv_backward(h, xd, mask, _gpu(grad_out), 10.0, -3.0, False)
    torch.cuda.synchronize()
    check_backward(x, kr, gw2.cpu().numpy(), gb2.cpu().numpy(), g_soft, None, 10.0, -3.0, sel=sel[:16])


def test_backward_is_repeatable_and_overwrites():
    import torch
    rng = np.random.default_rng(34)
    B, C, L, K = 2, 4, 900, 64
    x = _gpu(rng.standard_normal((B, C, L)).astype(np.float32))
    h = rocket.rocket_make_kernels(44, K, C, L)
    v = rocket.rocket_kernels_view_get(h)
    g = _gpu(rng.standard_normal((B, K)).astype(np.float32))
    gw = torch.full((len(v["weights"]),), float("nan"), device="cuda")
    gb = torch.full((K,), float("nan"), device="cuda")
    rocket.rocket_soft_ppv_backward(h, x, 4, g, grad_w=gw, grad_b=gb)
    torch.cuda.synchronize()
    a, b = gw.cpu().numpy().copy(), gb.cpu().numpy().copy()
    assert np.all(np.isfinite(a)) and np.all(np.isfinite(b))
    rocket.rocket_soft_ppv_backward(h, x, 4, g, grad_w=gw, grad_b=gb)
    torch.cuda.synchronize()
    # every sum is taken in a fixed order without atomics: the bits repeat
    assert np.array_equal(gw.cpu().numpy(), a)
    assert np.array_equal(gb.cpu().numpy(), b)


def test_batch_that_uses_the_per_xcd_mapping():
    """8 series of more than 8,192 samples: the launch maps series to XCDs; all planes, max included"""
    rng = np.random.default_rng(77)
    B, C, L, K = 8, 2, 9001, 48
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    h = rocket.rocket_make_kernels(3, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    grad_out = rng.standard_normal((B, 3 * K)).astype(np.float32)
    print("backward, per-XCD mapping", flush=True)
    gw, gb = _backward(h, x, 7, grad_out, 10.0, -3.0, True)
    g_soft, g_max = _split(grad_out, 7, K)
    sel = np.nonzero(_stable_argmax(x, kr))[0].astype(np.int32)
    assert len(sel) > K // 2
    check_backward(x, kr, gw, gb, g_soft, g_max, 10.0, -3.0, sel=sel)
