"""Pins the oracle's input prologue (8-bit intensities -> per-channel z-scores, paper
sections 4.1 and 4.3) without a GPU: scipy's zscore as the library opinion, invariants,
and the degenerate constant channel."""
import numpy as np
from scipy.stats import zscore

import oracle
import synth


def test_matches_scipy_zscore():
    x = synth.make_input_u8(2, B=2)[:, :5, :4000]
    z = oracle.znormalize_u8(x)
    ref = zscore(x.astype(np.float64), axis=-1, ddof=0)
    assert z.dtype == np.float32 and z.shape == x.shape
    np.testing.assert_allclose(z, ref.astype(np.float32), rtol=0, atol=1e-6)
    assert np.abs(z.astype(np.float64).mean(axis=-1)).max() < 1e-6
    assert np.abs(z.astype(np.float64).std(axis=-1) - 1.0).max() < 1e-6


def test_affine_invariance_and_constant_channel():
    rng = np.random.default_rng(0)
    x = rng.integers(0, 100, size=(3, 50)).astype(np.uint8)
    z = oracle.znormalize_u8(x)
    # a brighter, higher-gain copy of the same signal normalises to the same z-scores
    z2 = oracle.znormalize_u8((2 * x + 30).astype(np.uint8))
    np.testing.assert_allclose(z2, z, rtol=0, atol=1e-6)
    # hand-checked row: values 1, 3 -> mean 2, population std 1
    assert oracle.znormalize_u8(np.array([[1, 3]], np.uint8)).tolist() == [[-1.0, 1.0]]
    # a dead sensor (constant row) gives zeros, not NaN
    assert np.all(oracle.znormalize_u8(np.full((1, 20), 7, np.uint8)) == 0.0)


def test_u8_workload_uses_the_sensor_range():
    x = synth.make_input_u8(2, B=1)
    assert x.dtype == np.uint8 and x.shape == (1, 20, 50000)
    assert x.min() >= 0 and x.max() <= 255 and x.std(axis=-1).min() > 5
