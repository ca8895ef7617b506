"""GPU parity of the fused 8-bit input prologue (rocket_transform_u8,
rocket_soft_ppv_backward_u8) against the CPU oracle: the oracle z-normalises the bytes
(paper sections 4.1 and 4.3) and then transforms the result.  Needs an MI355X."""
import numpy as np
import pytest

import oracle
import synth
from paper_2301_08527_amd import rocket
from parity import check_backward, check_forward

pytestmark = pytest.mark.gpu


def _gpu(x):
    import torch
    return torch.from_numpy(x).cuda()


def _run_u8(h, x_u8, mask, lam=10.0, shift=-3.0):
    import torch
    out = rocket.rocket_transform_u8(h, _gpu(x_u8), mask, lam, shift)
    torch.cuda.synchronize()
    return out.cpu().numpy()


def test_small_ragged_with_dead_and_saturated_channels():
    """L not a multiple of 4, a constant channel, a channel clipped at both ends of the range"""
    rng = np.random.default_rng(5)
    B, C, L, K = 5, 4, 1003, 300
    x = rng.integers(0, 256, size=(B, C, L)).astype(np.uint8)
    x[:, 1, :] = 17                                           # dead sensor: zero variance
    x[2, 2, :] = np.where(rng.random(L) < 0.5, 0, 255)        # saturating sensor
    x[3, 3, :] = 200
    x[3, 3, 500] = 201                                        # almost constant: tiny variance
    h = rocket.rocket_make_kernels(77, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    print("u8 small", flush=True)
    out = _run_u8(h, x, 7)
    z = oracle.znormalize_u8(x)
    assert np.all(z[:, 1] == 0)
    check_forward(z, kr, out, 7)


def test_matches_float_entry_point_on_normalised_input():
    """same kernels, the oracle's normalised fp32 batch through rocket_transform"""
    import torch
    cfg = synth.CONFIGS[1]
    x = synth.make_input_u8(1, B=32)
    h = rocket.rocket_make_kernels(synth.seed_k(1), 2000, cfg["C"], cfg["L"])
    print("u8 vs f32 entry", flush=True)
    a = _run_u8(h, x, 5)
    b = rocket.rocket_transform(h, _gpu(oracle.znormalize_u8(x)), 5)
    torch.cuda.synchronize()
    np.testing.assert_allclose(a, b.cpu().numpy(), rtol=1e-5, atol=1e-6)


def test_config2_shape_u8():
    """20 channels x 50,000 bytes per example, K = 10,000, kernel sample checked by the oracle"""
    cfg = synth.CONFIGS[2]
    B = 8
    x = synth.make_input_u8(2, B=B)
    h = rocket.rocket_make_kernels(synth.seed_k(2), cfg["K"], cfg["C"], cfg["L"])
    kr = rocket.rocket_kernels_view_get(h)
    print("u8 config2 run", flush=True)
    out = _run_u8(h, x, cfg["features"])
    sel = synth.pick_kernels(kr, 128, seed=12)
    check_forward(oracle.znormalize_u8(x), kr, out, cfg["features"], sel=sel)


def test_backward_u8():
    import torch
    rng = np.random.default_rng(9)
    B, C, L, K = 3, 5, 2001, 120
    x = rng.integers(0, 256, size=(B, C, L)).astype(np.uint8)
    x[1, 0, :] = 3
    h = rocket.rocket_make_kernels(91, K, C, L)
    kr = rocket.rocket_kernels_view_get(h)
    g = rng.standard_normal((B, K)).astype(np.float32)
    print("u8 backward", flush=True)
    gw, gb = rocket.rocket_soft_ppv_backward_u8(h, _gpu(x), 4, _gpu(g), 4.0, -3.0)
    torch.cuda.synchronize()
    check_backward(oracle.znormalize_u8(x), kr, gw.cpu().numpy(), gb.cpu().numpy(), g, None, 4.0, -3.0)


def test_dtype_is_checked():
    import torch
    h = rocket.rocket_make_kernels(1, 10, 1, 100)
    with pytest.raises(rocket.RocketError):
        rocket.rocket_transform_u8(h, torch.zeros((1, 1, 100), device="cuda"), 1)
    with pytest.raises(rocket.RocketError):
        rocket.rocket_transform(h, torch.zeros((1, 1, 100), dtype=torch.uint8, device="cuda"), 1)
