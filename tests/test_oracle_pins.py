"""Pins the CPU oracle to things other than itself (no GPU needed).

Each test states what a plausible mistake in the oracle would break.  The
independent opinions are numpy.correlate with a zero-stuffed kernel, torch's
CPU conv1d, scipy's logistic function, closed forms that follow from the
paper's section 3.1 / 3.2, brute force in pure Python, and central finite
differences.
"""
import math
import os

import numpy as np
import pytest
from scipy.special import expit

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def make_kernels(specs, C, L):
    """specs: list of dict(length, dilation, padded, bias, channels, weights[n_ch][length])."""
    K = len(specs)
    kr = {"K": K, "C": C, "L": L}
    kr["length"] = np.array([s["length"] for s in specs], np.int32)
    kr["dilation"] = np.array([s["dilation"] for s in specs], np.int32)
    kr["padding"] = np.array([(s["length"] - 1) * s["dilation"] // 2 if s["padded"] else 0
                              for s in specs], np.int32)
    kr["bias"] = np.array([s["bias"] for s in specs], np.float32)
    kr["n_ch"] = np.array([len(s["channels"]) for s in specs], np.int32)
    kr["ch_off"] = np.concatenate([[0], np.cumsum(kr["n_ch"])]).astype(np.int64)
    kr["w_off"] = np.concatenate([[0], np.cumsum(kr["n_ch"] * kr["length"])]).astype(np.int64)
    kr["channels"] = np.concatenate([np.asarray(s["channels"], np.int32) for s in specs])
    kr["weights"] = np.concatenate([np.asarray(s["weights"], np.float32).reshape(-1) for s in specs])
    return kr


def random_specs(rng, K, C, L, centred=True):
    specs = []
    for _ in range(K):
        ln = int(rng.choice([7, 9, 11]))
        d = int(rng.integers(1, (L - 1) // (ln - 1) + 1))
        nch = int(rng.integers(1, min(C, 9) + 1))
        ch = rng.permutation(C)[:nch]
        w = rng.standard_normal((nch, ln))
        if centred:
            w -= w.mean(axis=1, keepdims=True)
        specs.append(dict(length=ln, dilation=d, padded=bool(rng.integers(0, 2)),
                          bias=float(rng.uniform(-1, 1)), channels=ch, weights=w))
    return specs


def numpy_conv(x, spec):
    """Independent definition: correlate the zero-padded series with the kernel
    stretched to (len-1)*d+1 taps (zeros between the weights)."""
    ln, d = spec["length"], spec["dilation"]
    p = (ln - 1) * d // 2 if spec["padded"] else 0
    w32 = np.asarray(spec["weights"], np.float32).astype(np.float64)
    y = None
    for c, ch in enumerate(spec["channels"]):
        stuffed = np.zeros((ln - 1) * d + 1)
        stuffed[::d] = w32[c]
        xp = np.concatenate([np.zeros(p), x[ch].astype(np.float64), np.zeros(p)])
        yc = np.correlate(xp, stuffed, mode="valid")
        y = yc if y is None else y + yc
    return y + float(np.float32(spec["bias"]))


# ---------------------------------------------------------------- conv geometry

def test_conv_matches_numpy_correlate():
    """wrong tap index, dilation stride, padding offset, channel gather or a
    flipped kernel all fail here."""
    rng = np.random.default_rng(1)
    C, L = 5, 97
    x = rng.standard_normal((C, L)).astype(np.float32)
    specs = random_specs(rng, 40, C, L, centred=False)
    kr = make_kernels(specs, C, L)
    for k, s in enumerate(specs):
        y = oracle.conv_output(x, kr, k)
        ref = numpy_conv(x, s)
        assert y.shape == ref.shape
        np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


def test_conv_matches_torch_conv1d():
    """third opinion: torch's CPU conv1d with dilation= and padding=."""
    import torch
    rng = np.random.default_rng(2)
    C, L = 4, 80
    x = rng.standard_normal((C, L)).astype(np.float32)
    specs = random_specs(rng, 20, C, L, centred=False)
    kr = make_kernels(specs, C, L)
    for k, s in enumerate(specs):
        xin = torch.from_numpy(x[np.asarray(s["channels"])].astype(np.float64))[None]
        w = torch.from_numpy(np.asarray(s["weights"], np.float32).astype(np.float64))[None]
        p = int(kr["padding"][k])
        ref = torch.nn.functional.conv1d(xin, w, bias=torch.tensor([float(np.float32(s["bias"]))], dtype=torch.float64),
                                         dilation=s["dilation"], padding=p)[0, 0].numpy()
        y = oracle.conv_output(x, kr, k)
        np.testing.assert_allclose(y, ref, rtol=0, atol=1e-12)


def test_conv_brute_force_tiny():
    """hand-enumerable case written as the bare double sum of the definition."""
    L = 16
    x = np.arange(1, L + 1, dtype=np.float32)[None, :] ** 2
    w = np.array([[1, -2, 3, 0.5, -1, 2, -3.5]], np.float32)
    for padded in (False, True):
        s = dict(length=7, dilation=2, padded=padded, bias=0.25, channels=[0], weights=w)
        kr = make_kernels([s], 1, L)
        p = 6 if padded else 0
        n = L + 2 * p - 12
        want = []
        for t in range(n):
            acc = 0.25
            for j in range(7):
                idx = t + 2 * j - p
                if 0 <= idx < L:
                    acc += float(w[0, j]) * float(x[0, idx])
            want.append(acc)
        y = oracle.conv_output(x, kr, 0)
        assert len(y) == n == (L if padded else L - 12)
        np.testing.assert_allclose(y, want, rtol=0, atol=1e-12)


def test_output_length_formula():
    """'same' padding keeps the input length; no padding loses (len-1)*d."""
    rng = np.random.default_rng(3)
    C, L = 2, 211
    x = rng.standard_normal((C, L)).astype(np.float32)
    specs = random_specs(rng, 30, C, L)
    kr = make_kernels(specs, C, L)
    out = oracle.transform(x[None], kr)
    for k, s in enumerate(specs):
        want = L if s["padded"] else L - (s["length"] - 1) * s["dilation"]
        assert out["n_out"][k] == want == len(oracle.conv_output(x, kr, k))


def test_unit_impulse_reads_back_weights():
    """an impulse at t0 makes y[t] - bias = w[j] exactly where t + j*d - p = t0;
    pins dilation and padding geometry and the unflipped orientation."""
    L, t0 = 101, 50
    x = np.zeros((1, L), np.float32)
    x[0, t0] = 1.0
    rng = np.random.default_rng(4)
    for ln in (7, 9, 11):
        for d in (1, 3, 10):
            for padded in (False, True):
                w = rng.standard_normal((1, ln)).astype(np.float32)
                s = dict(length=ln, dilation=d, padded=padded, bias=0.5, channels=[0], weights=w)
                kr = make_kernels([s], 1, L)
                p = int(kr["padding"][0])
                y = oracle.conv_output(x, kr, 0)
                want = np.full(len(y), 0.5)
                for j in range(ln):
                    t = t0 - j * d + p
                    if 0 <= t < len(y):
                        want[t] += float(w[0, j])
                np.testing.assert_allclose(y, want, rtol=0, atol=1e-15)


def test_constant_series_gives_bias():
    """mean-centred weights (section 3.1): a constant series through an unpadded
    kernel yields the bias at every position, whatever the per-channel constants;
    with 'same' padding this holds at interior positions."""
    C, L = 6, 300
    consts = np.array([0.0, 1.0, -2.5, 3.25, 7.0, -0.125], np.float32)
    x = np.repeat(consts[:, None], L, axis=1)
    kr = oracle.sample_kernels(11, 200, C, L)
    out = oracle.transform(x[None], kr, lam=10.0, shift=-3.0)
    for k in range(200):
        y = oracle.conv_output(x, kr, k)
        b = float(kr["bias"][k])
        p, d, ln = int(kr["padding"][k]), int(kr["dilation"][k]), int(kr["length"][k])
        interior = y[p: len(y) - p] if p else y
        # weights are rounded to fp32 after centring, so sum_j w is ~1e-7, not 0
        np.testing.assert_allclose(interior, b, rtol=0, atol=3e-5)
        if p == 0:
            assert abs(out["max"][0, k] - b) < 3e-5
            if abs(b) > 1e-4:
                assert out["ppv"][0, k] == (1.0 if b > 0 else 0.0)
            assert abs(out["softppv"][0, k] - expit(10.0 * b - 3.0)) < 1e-4
    # channel 0 is identically zero: kernels that only see it give the bias exactly
    only0 = [k for k in range(200) if kr["n_ch"][k] == 1 and kr["channels"][kr["ch_off"][k]] == 0]
    for k in only0:
        assert np.all(oracle.conv_output(x, kr, k) == float(kr["bias"][k]))


# ------------------------------------------------------------------- pooling

def test_pooling_matches_numpy_and_scipy():
    """max, Heaviside mean (Eq. 1-2) and sigmoid mean (Eq. 3-4) recomputed with
    numpy/scipy from an independently computed conv output."""
    rng = np.random.default_rng(5)
    B, C, L = 3, 4, 150
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    specs = random_specs(rng, 25, C, L)
    kr = make_kernels(specs, C, L)
    for lam, shift in ((10.0, -3.0), (2.0, -3.0), (1.0, 3.0), (0.0, -3.0)):
        out = oracle.transform(x, kr, lam=lam, shift=shift)
        for b in range(B):
            for k, s in enumerate(specs):
                y = numpy_conv(x[b], s)
                assert abs(out["max"][b, k] - y.max()) < 1e-12
                assert out["argmax"][b, k] == int(np.argmax(y))
                assert out["count"][b, k] == int((y > 0).sum())
                assert abs(out["ppv"][b, k] - (y > 0).mean()) < 1e-15
                assert abs(out["softppv"][b, k] - expit(lam * y + shift).mean()) < 1e-13
                assert out["ambiguous"][b, k] == int((np.abs(y) < 1e-5).sum())


def test_heaviside_is_strict_at_zero():
    """Eq. 1: H(0) = 0.  An all-zero series with zero bias gives y == 0."""
    L = 64
    x = np.zeros((1, 1, L), np.float32)
    w = np.ones((1, 7), np.float32)
    kr = make_kernels([dict(length=7, dilation=1, padded=False, bias=0.0, channels=[0], weights=w)], 1, L)
    out = oracle.transform(x, kr)
    assert out["count"][0, 0] == 0 and out["ppv"][0, 0] == 0.0
    assert out["ambiguous"][0, 0] == out["n_out"][0]


def test_soft_heaviside_golden_values():
    """Eq. 3 with the shift of the prose, at the lambdas of Fig. 1: a constant
    output y == x0 (zero weights, bias x0) pools to the soft step at x0."""
    rows = [l.split() for l in open(os.path.join(GOLDEN, "soft_heaviside.txt"))
            if l.strip() and not l.startswith("#")]
    L = 40
    x = np.ones((1, 1, L), np.float32)
    for lam, x0, _, want in rows:
        lam, x0, want = float(lam), float(x0), float(want)
        kr = make_kernels([dict(length=9, dilation=2, padded=False, bias=x0, channels=[0],
                                weights=np.zeros((1, 9), np.float32))], 1, L)
        b32 = float(np.float32(x0))
        got = oracle.transform(x, kr, lam=lam, shift=-3.0)["softppv"][0, 0]
        # the bias is stored in fp32: allow its rounding through the slope lam/4
        assert abs(got - want) <= lam * abs(b32 - x0) / 4 + 1e-15
        # the printed form of Eq. 3 is the same function with shift = +3
        got_printed = oracle.transform(x, kr, lam=lam, shift=3.0)["softppv"][0, 0]
        assert abs(got_printed - 1.0 / (1.0 + math.exp(-lam * b32 - 3.0))) < 1e-15


def test_soft_ppv_limits():
    """lambda = 0 gives sigma(shift) for every kernel; lambda -> infinity gives
    PPV (section 3.2).  With z = lam*y - 3, |sigma(z) - 1[z > 0]| <= exp(-|z|),
    and 1[z > 0] differs from H(y) only for 0 < y <= 3/lam."""
    rng = np.random.default_rng(6)
    B, C, L = 2, 3, 200
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    kr = oracle.sample_kernels(7, 60, C, L)
    o0 = oracle.transform(x, kr, lam=0.0, shift=-3.0)
    np.testing.assert_allclose(o0["softppv"], expit(-3.0), rtol=0, atol=1e-15)
    prev = None
    for lam in (10.0, 1e2, 1e4, 1e7):
        o = oracle.transform(x, kr, lam=lam, shift=-3.0)
        assert np.all((o["softppv"] > 0) & (o["softppv"] < 1) | (lam >= 1e4))
        err = np.abs(o["softppv"] - o["ppv"])
        for b in range(B):
            for k in range(60):
                y = oracle.conv_output(x[b], kr, k)
                bound = (np.exp(-np.abs(lam * y - 3.0)) + ((y > 0) & (y <= 3.0 / lam))).mean()
                assert err[b, k] <= bound + 1e-15
        if prev is not None:
            assert err.max() <= prev
        prev = err.max()
    assert prev < 1e-5


def test_max_and_ppv_invariants():
    """max >= every output and is attained; scaling (x, bias) by a > 0 scales
    the max and leaves PPV unchanged; negating weights and bias maps the count
    to n - count - #{y == 0}; PPV in [0, 1]; softPPV increases with the bias."""
    rng = np.random.default_rng(8)
    B, C, L = 2, 3, 128
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    specs = random_specs(rng, 30, C, L)
    kr = make_kernels(specs, C, L)
    o = oracle.transform(x, kr)
    assert np.all((o["ppv"] >= 0) & (o["ppv"] <= 1))
    assert np.all((o["count"] >= 0) & (o["count"] <= o["n_out"][None, :]))
    for b in range(B):
        for k in range(30):
            y = oracle.conv_output(x[b], kr, k)
            assert o["max"][b, k] >= y.max() and o["max"][b, k] in y
            assert abs(o["gap"][b, k] - (np.sort(y)[-1] - np.sort(y)[-2])) < 1e-12
    # scaling by a power of two is exact in fp32
    kr2 = dict(kr)
    kr2["bias"] = kr["bias"] * np.float32(4.0)
    o2 = oracle.transform(x * np.float32(4.0), kr2)
    np.testing.assert_allclose(o2["max"], 4.0 * o["max"], rtol=1e-14)
    assert np.array_equal(o2["count"], o["count"])
    krn = dict(kr)
    krn["bias"] = -kr["bias"]
    krn["weights"] = -kr["weights"]
    on = oracle.transform(x, krn)
    assert np.array_equal(on["count"], o["n_out"][None, :] - o["count"])  # no exact zeros here
    krb = dict(kr)
    krb["bias"] = kr["bias"] + np.float32(0.5)
    ob = oracle.transform(x, krb)
    assert np.all(ob["softppv"] > o["softppv"]) and np.all(ob["count"] >= o["count"])


# ------------------------------------------------------------------ backward

def _objective(x, kr, gs, gm, lam, shift):
    o = oracle.transform(x, kr, lam=lam, shift=shift)
    v = (gs * o["softppv"]).sum()
    if gm is not None:
        v += (gm * o["max"]).sum()
    return v


@pytest.mark.parametrize("with_max", [False, True])
def test_backward_matches_finite_differences(with_max):
    """a wrong factor (lambda/n, s(1-s)), a wrong tap index in the weight
    gradient, or a missing batch sum fails here."""
    rng = np.random.default_rng(9)
    B, C, L = 3, 3, 60
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    specs = random_specs(rng, 6, C, L)
    for s in specs:   # keep finite differences well conditioned
        s["dilation"] = min(s["dilation"], 4)
    kr = make_kernels(specs, C, L)
    lam, shift = 2.0, -3.0
    gs = rng.standard_normal((B, 6))
    gm = rng.standard_normal((B, 6)) if with_max else None
    gw, gb = oracle.backward(x, kr, gs, gm, lam=lam, shift=shift)
    assert oracle.transform(x, kr)["gap"].min() > 1e-3   # argmax is stable under the steps below
    h = 2.0 ** -10
    for name, grad in (("weights", gw), ("bias", gb)):
        base = kr[name].copy()
        for i in range(len(base)):
            hi, lo = base.copy(), base.copy()
            hi[i] = np.float32(base[i] + h)
            lo[i] = np.float32(base[i] - h)
            step = float(hi[i]) - float(lo[i])
            k_hi, k_lo = dict(kr), dict(kr)
            k_hi[name], k_lo[name] = hi, lo
            fd = (_objective(x, k_hi, gs, gm, lam, shift) - _objective(x, k_lo, gs, gm, lam, shift)) / step
            assert abs(fd - grad[i]) <= 2e-5 * max(1.0, abs(grad[i])), (name, i, fd, grad[i])


def test_backward_bias_identity_and_selection():
    """grad_b[k] = sum_b g * (lambda/n) * sum_t s(1-s), recomputed with numpy;
    kernels that are not selected get zero gradients."""
    rng = np.random.default_rng(10)
    B, C, L = 2, 2, 90
    x = rng.standard_normal((B, C, L)).astype(np.float32)
    specs = random_specs(rng, 8, C, L)
    kr = make_kernels(specs, C, L)
    sel = np.array([1, 4, 6], np.int32)
    gs = rng.standard_normal((B, 3))
    lam = 5.0
    gw, gb = oracle.backward(x, kr, gs, None, lam=lam, shift=-3.0, sel=sel)
    for k in range(8):
        lo, hi = kr["w_off"][k], kr["w_off"][k + 1]
        if k not in sel:
            assert gb[k] == 0 and np.all(gw[lo:hi] == 0)
            continue
        s_i = list(sel).index(k)
        want_b, want_w = 0.0, np.zeros(hi - lo)
        ln, d, p = specs[k]["length"], specs[k]["dilation"], int(kr["padding"][k])
        for b in range(B):
            y = numpy_conv(x[b], specs[k])
            sg = expit(lam * y - 3.0)
            q = gs[b, s_i] * lam / len(y) * sg * (1 - sg)
            want_b += q.sum()
            for c, ch in enumerate(specs[k]["channels"]):
                xp = np.concatenate([np.zeros(p), x[b, ch].astype(np.float64), np.zeros(p)])
                for j in range(ln):
                    want_w[c * ln + j] += (q * xp[j * d: j * d + len(y)]).sum()
        assert abs(gb[k] - want_b) < 1e-13
        np.testing.assert_allclose(gw[lo:hi], want_w, rtol=0, atol=1e-13)
