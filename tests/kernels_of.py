"""Kernels for the parity tests, drawn twice: by the library (the handle the GPU path uses) and
by the oracle's own sampler (the arrays the oracle computes with).  The two must agree bit for
bit (paper section 3.1 fixes the laws; the draw recipe is this build's), so a deviation of the
library's sampler on the machine that runs the GPU tests cannot hide behind kernels that the
oracle merely copied from the library."""
import numpy as np

import oracle
from paper_2301_08527_amd import rocket

INT_FIELDS = ("length", "dilation", "padding", "n_ch", "channels", "ch_off", "w_off")


def assert_same_kernels(view, kr):
    assert (view["K"], view["C"], view["L"]) == (kr["K"], kr["C"], kr["L"])
    for name in INT_FIELDS:
        assert np.array_equal(view[name], kr[name]), name
    assert np.array_equal(view["bias"].view(np.uint32), kr["bias"].view(np.uint32)), "bias bits"
    assert np.array_equal(view["weights"].view(np.uint32), kr["weights"].view(np.uint32)), "weight bits"


def sampled(seed, K, C, L):
    """(library handle, oracle-sampled kernel arrays) of the same (seed, K, C, L), checked equal."""
    h = rocket.rocket_make_kernels(seed, K, C, L)
    kr = oracle.sample_kernels(seed, K, C, L)
    assert_same_kernels(rocket.rocket_kernels_view_get(h), kr)
    return h, kr
