"""GPU parity of the MINIROCKET-style variant (paper section 2) against the CPU oracle: the predetermined
kernel set bit for bit, the biases fitted to data within the feature tolerance, and the PPV features.
Needs an MI355X.  (Parity with the original MINIROCKET model is not claimed: see oracle/minirocket.py.)"""
import numpy as np
import pytest

import oracle
import synth
from kernels_of import INT_FIELDS
from paper_2301_08527_amd import rocket
from parity import ATOL, RTOL, check_forward

pytestmark = pytest.mark.gpu


def _gpu(a):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def _same_set(h, kr):
    v = rocket.rocket_kernels_view_get(h)
    for name in INT_FIELDS:
        assert np.array_equal(v[name], kr[name]), name
    assert np.array_equal(v["weights"], kr["weights"])
    return v


@pytest.mark.parametrize("seed,groups,C,L", [(1, 3, 1, 9), (2, 5, 4, 700), (3, 40, 20, 50000), (2**64 - 2, 2, 12, 8193)])
def test_kernel_set_is_the_oracles(seed, groups, C, L):
    h = rocket.rocket_minirocket_kernels(seed, groups, C, L)
    v = _same_set(h, oracle.minirocket_kernels(seed, groups, C, L))
    assert np.all(v["bias"] == 0) and len(v["length"]) == 84 * groups


def _fit_and_check(seed, groups, x):
    import torch
    B, C, L = x.shape
    h = rocket.rocket_minirocket_kernels(seed, groups, C, L)
    kr0 = oracle.minirocket_kernels(seed, groups, C, L)
    print("minirocket fit", x.shape, groups, flush=True)
    rocket.rocket_minirocket_fit_bias(h, _gpu(x), seed + 100)
    torch.cuda.synchronize()
    got = rocket.rocket_kernels_view_get(h)["bias"].astype(np.float64)
    kr, ex, rank = oracle.minirocket_fit_bias(x, kr0, seed + 100)
    ref = kr["bias"].astype(np.float64)
    err = np.abs(got - ref)
    assert np.all(err <= RTOL * np.abs(ref) + ATOL), (int(np.argmax(err)), float(err.max()))
    return h, kr


def test_bias_fit_and_features_small():
    rng = np.random.default_rng(71)
    x = rng.standard_normal((5, 3, 1200)).astype(np.float32)
    h, kr = _fit_and_check(5, 4, x)
    import torch
    xt = rng.standard_normal((7, 3, 1200)).astype(np.float32)
    out = rocket.rocket_transform(h, _gpu(xt), 2)
    torch.cuda.synchronize()
    # the library's biases differ from the oracle's by rounding: compare the features through the oracle's kernels
    # with the library's biases, so that both sides pool the same thing
    kr_lib = dict(kr)
    kr_lib["bias"] = rocket.rocket_kernels_view_get(h)["bias"]
    check_forward(xt, kr_lib, out.cpu().numpy(), 2)
    # and on the training batch every kernel's PPV on its own example is what the rank says (up to near-ties)
    out_train = rocket.rocket_transform(h, _gpu(x), 2).cpu().numpy().astype(np.float64)
    ref = oracle.minirocket_transform(x, kr_lib)
    assert np.all(np.abs(np.rint(out_train * ref["n_out"][None, :]) - ref["count"]) <= ref["ambiguous"])


def test_bias_fit_with_ties_and_one_series():
    """8-bit-like samples (many equal outputs: the selected order statistic is still an element of the row) and a
    training batch of one series, shortest legal length included"""
    rng = np.random.default_rng(72)
    x = rng.integers(0, 4, size=(1, 2, 333)).astype(np.float32)
    _fit_and_check(6, 2, x)
    _fit_and_check(7, 1, rng.standard_normal((2, 1, 9)).astype(np.float32))
    _fit_and_check(8, 2, rng.standard_normal((3, 5, 64)).astype(np.float32))


def test_paper_shape_sample():
    """20 channels x 50,000 samples, 119 groups (9,996 kernels): fit on 4 series, features of 3 others, a
    stratified sample of kernels checked by the oracle"""
    import torch
    x = synth.make_input(2, B=7)
    groups = 119
    h = rocket.rocket_minirocket_kernels(31, groups, 20, 50000)
    kr0 = oracle.minirocket_kernels(31, groups, 20, 50000)
    _same_set(h, kr0)
    print("minirocket paper shape: fit", flush=True)
    rocket.rocket_minirocket_fit_bias(h, _gpu(x[:4]), 77)
    torch.cuda.synchronize()
    bias = rocket.rocket_kernels_view_get(h)["bias"]
    sel = synth.pick_kernels(kr0, 96, seed=5)
    ex, q = oracle.minirocket.bias_draws(77, kr0["K"], 4)
    for k in sel:
        y = oracle.conv_output(x[ex[k]], kr0, int(k))
        r = int(np.floor(q[k] * (len(y) - 1)))
        ref = -np.partition(y, r)[r]
        assert abs(float(bias[k]) - ref) <= RTOL * abs(ref) + ATOL, int(k)
    print("minirocket paper shape: transform", flush=True)
    out = rocket.rocket_transform(h, _gpu(x[4:]), 2)
    torch.cuda.synchronize()
    kr_lib = dict(kr0)
    kr_lib["bias"] = bias
    check_forward(x[4:], kr_lib, out.cpu().numpy(), 2, sel=sel)
