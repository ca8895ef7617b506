"""Pins of the oracle's MINIROCKET-style variant (paper section 2: two-valued predetermined weights,
convolution by additions, biases from the data, PPV only).  No GPU needed.  The original MINIROCKET
is not available here: these pins fix this build's definition, not parity with that model."""
import itertools

import numpy as np

import oracle
from oracle import minirocket as mr


def _kernels(seed=3, groups=2, C=4, L=300):
    return mr.minirocket_kernels(seed, groups, C, L)


def test_predetermined_weight_set():
    """84 kernels per group: three 2s and six -1s (zero sum), all distinct, lexicographic, the same
    row on every channel; a group shares dilation, padding and channels"""
    kr = _kernels(groups=3, C=12)
    K = kr["K"]
    assert K == 3 * 84 and mr.SET_SIZE == 84
    rows = set()
    for k in range(K):
        w = kr["weights"][kr["w_off"][k]:kr["w_off"][k + 1]].reshape(kr["n_ch"][k], 9)
        assert np.all(w == w[0])
        assert sorted(w[0].tolist()) == [-1.0] * 6 + [2.0] * 3 and w[0].sum() == 0.0
        if k < 84:
            rows.add(tuple(w[0].tolist()))
            assert tuple(np.nonzero(w[0] == 2.0)[0]) == list(itertools.combinations(range(9), 3))[k]
    assert len(rows) == 84
    for g in range(3):
        sl = slice(84 * g, 84 * (g + 1))
        for name in ("dilation", "padding", "n_ch"):
            assert len(set(kr[name][sl].tolist())) == 1
        ch = [tuple(kr["channels"][kr["ch_off"][k]:kr["ch_off"][k + 1]]) for k in range(84 * g, 84 * (g + 1))]
        assert len(set(ch)) == 1 and len(set(ch[0])) == len(ch[0])
    d = kr["dilation"]
    assert np.all(d >= 1) and np.all(d <= (300 - 1) // 8)
    assert np.all((kr["padding"] == 0) | (kr["padding"] == 4 * d))
    assert np.all(kr["bias"] == 0)


def test_group_parameters_follow_the_laws_of_section_3_1():
    kr = mr.minirocket_kernels(11, 1500, 20, 50000)
    d = kr["dilation"][::84].astype(np.float64)
    A = np.log2(49999 / 8)
    assert abs((np.log2(d + 0.5) / A).mean() - 0.5) < 0.04            # log2 d roughly uniform
    assert abs((kr["padding"][::84] != 0).mean() - 0.5) < 0.05         # fair padding coin
    assert abs(kr["n_ch"][::84].mean() - 3.44) < 0.25                   # channel-count law, mean 3.44


def test_additions_equal_the_convolution():
    """3 * (sum over the 2-taps) - (sum over all taps) is the kernel's output: the shifted-sum code
    against the oracle's conv routine (a different program) and against numpy.correlate"""
    rng = np.random.default_rng(5)
    kr = _kernels(seed=9, groups=4, C=5, L=400)
    x = rng.standard_normal((5, 400)).astype(np.float32)
    for k in (0, 17, 83, 84, 200, 335):
        a = mr.output_by_additions(x, kr, k)
        b = oracle.conv_output(x, kr, k)
        assert a.shape == b.shape and np.allclose(a, b, rtol=0, atol=1e-12)
        d, p = int(kr["dilation"][k]), int(kr["padding"][k])
        ch = kr["channels"][kr["ch_off"][k]:kr["ch_off"][k + 1]]
        w = kr["weights"][kr["w_off"][k]:kr["w_off"][k] + 9].astype(np.float64)
        stuffed = np.zeros(8 * d + 1)
        stuffed[::d] = w
        series = np.pad(x[ch].astype(np.float64).sum(axis=0), p)
        assert np.allclose(a, np.correlate(series, stuffed, "valid"), atol=1e-12)


def test_bias_is_the_stated_order_statistic():
    """brute force: sort the bias-free output of the drawn example and take the drawn rank; and the
    consequence for the strict PPV on that example: (n - 1 - rank) / n"""
    rng = np.random.default_rng(6)
    kr0 = _kernels(seed=4, groups=2, C=3, L=257)
    x = rng.standard_normal((6, 3, 257)).astype(np.float32)
    kr, ex, rank = mr.minirocket_fit_bias(x, kr0, seed=21)
    assert ex.min() >= 0 and ex.max() < 6 and len(set(ex.tolist())) > 1
    for k in range(0, kr["K"], 7):
        y = np.sort(oracle.conv_output(x[ex[k]], kr0, k))
        assert 0 <= rank[k] <= len(y) - 1
        assert kr["bias"][k] == np.float32(-y[rank[k]])
    o = mr.minirocket_transform(x, kr)
    assert np.all((o["ppv"] >= 0) & (o["ppv"] <= 1))
    checked = 0
    for k in range(kr["K"]):
        n = int(o["n_out"][k])
        y = oracle.conv_output(x[ex[k]], kr0, k)
        # the float32 rounding of the bias can move the outputs next to it across zero: the count may be off
        # by the number of outputs within 1e-6 of zero (the order statistic itself is one of them)
        shifted = np.abs(y + np.float64(kr["bias"][k]))
        if np.sort(shifted)[1] > 1e-4:                 # nothing but the order statistic near zero: a clear case
            assert abs(int(o["count"][ex[k], k]) - (n - 1 - int(rank[k]))) <= np.sum(shifted < 1e-6)
            checked += 1
    assert checked > kr["K"] // 2


def test_rank_never_reaches_the_largest_output():
    """rank = floor(q (n - 1)) with q < 1 is at most n - 2: with two outputs the bias is always minus the
    smaller one, with one output minus that one; and over many kernels the relative rank is uniform"""
    rng = np.random.default_rng(9)
    kr0 = mr.minirocket_kernels(3, 3, 1, 10)
    kr0["padding"][:] = 0
    kr0["dilation"][:] = 1                       # n = 10 - 8 = 2
    x = rng.standard_normal((4, 1, 10)).astype(np.float32)
    kr, ex, rank = mr.minirocket_fit_bias(x, kr0, seed=2)
    assert np.all(rank == 0)
    for k in range(kr["K"]):
        y = oracle.conv_output(x[ex[k]], kr0, k)
        assert len(y) == 2 and kr["bias"][k] == np.float32(-y.min())
    one = mr.minirocket_kernels(3, 1, 1, 9)
    one["padding"][:] = 0
    kr1, ex1, rank1 = mr.minirocket_fit_bias(x[:, :, :9], one, seed=2)
    assert np.all(rank1 == 0)
    big = mr.minirocket_kernels(5, 6, 2, 400)
    _, _, rank_big = mr.minirocket_fit_bias(rng.standard_normal((3, 2, 400)).astype(np.float32), big, seed=3)
    n = 400 + 2 * big["padding"].astype(np.int64) - 8 * big["dilation"].astype(np.int64)
    rel = rank_big / np.maximum(n - 1, 1)
    assert np.all(rank_big <= np.maximum(n - 2, 0)) and abs(rel.mean() - 0.5) < 0.07 and rel.min() < 0.05 and rel.max() > 0.95


def test_ramp_closed_form():
    """a linear ramp through a zero-sum kernel without padding gives the constant sum_j w_j * j * d * slope:
    every order statistic equals it, the bias is its negative, and the strict PPV of the ramp is 0"""
    L = 200
    kr0 = mr.minirocket_kernels(2, 1, 1, L)
    kr0["padding"][:] = 0
    x = (0.5 * np.arange(L, dtype=np.float32))[None, None, :]
    kr, ex, rank = mr.minirocket_fit_bias(x, kr0, seed=8)
    d = int(kr0["dilation"][0])
    for k in (0, 40, 83):
        w = kr0["weights"][kr0["w_off"][k]:kr0["w_off"][k] + 9].astype(np.float64)
        const = 0.5 * d * np.dot(w, np.arange(9))
        assert abs(float(kr["bias"][k]) + const) < 1e-9
    assert np.all(mr.minirocket_transform(x, kr)["count"] == 0)


def test_draws_are_seeded_and_in_range():
    ex1, q1 = mr.bias_draws(5, 200, 7)
    ex2, q2 = mr.bias_draws(5, 200, 7)
    ex3, _ = mr.bias_draws(6, 200, 7)
    assert np.array_equal(ex1, ex2) and np.array_equal(q1, q2) and not np.array_equal(ex1, ex3)
    assert ex1.min() >= 0 and ex1.max() < 7 and q1.min() >= 0 and q1.max() < 1
    assert abs(q1.mean() - 0.5) < 0.1
