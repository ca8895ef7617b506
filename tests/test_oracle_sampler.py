"""Pins the oracle's kernel sampler to the laws of the paper's section 3.1
(no GPU needed): supports, frequencies, moments, a Kolmogorov-Smirnov test of
the normal draws, the published SplitMix64 test vector, and stored
known-answer kernels (tests/golden/sampler_kat.json, written by
tests/golden/make_sampler_kat.py from the oracle alone)."""
import json
import math
import os

import numpy as np
from scipy import stats

import oracle
from oracle import sampler

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_splitmix64_published_vector():
    """the first outputs for seed 1234567 as published with the generator"""
    want = [6457827717110365317, 3203168211198807973, 9817491932198370423,
            4593380528125082431, 16408922859458223821]
    s, got = 1234567, []
    for _ in range(5):
        s = (s + sampler.GAMMA) & sampler.MASK
        got.append(sampler.mix64(s))
    assert got == want


def test_uniform_conversions():
    st = sampler.Stream(3, 0)
    u = np.array([st.u01() for _ in range(20000)])
    assert u.min() >= 0.0 and u.max() < 1.0
    assert stats.kstest(u, "uniform").pvalue > 1e-3
    v = np.array([st.u_open() for _ in range(20000)])
    assert v.min() > 0.0 and v.max() <= 1.0
    assert abs(sampler.ROU_C - math.sqrt(2.0 / math.e)) < 1e-16


def test_series_logarithm_and_power_against_the_math_library():
    """the sampler's own ln / log2 / 2^y (series of basic operations, so that its decisions do
    not depend on a math library's last bit) agree with the library functions to a few ulp, hit
    the exact values, and are monotone across the range-reduction seams"""
    rng = np.random.default_rng(8)
    xs = np.concatenate([rng.random(20000), 10.0 ** rng.uniform(-12, 8, 20000), [1.0, 0.5, 2.0, 2.0 ** -53, 8333.0]])
    for x in xs:
        x = float(x)
        if x <= 0.0:
            continue
        want = math.log(x)
        assert abs(sampler.ln_series(x) - want) <= 4e-16 * max(1.0, abs(want))
        assert abs(sampler.log2_series(x) - math.log2(x)) <= 6e-16 * max(1.0, abs(math.log2(x)))
    for y in np.concatenate([rng.uniform(0, 16, 20000), [0.0, 1.0, 3.0, 13.0, 15.999999999]]):
        y = float(y)
        assert abs(sampler.exp2_series(y) - 2.0 ** y) <= 4e-16 * 2.0 ** y
    assert sampler.ln_series(1.0) == 0.0 and sampler.exp2_series(0.0) == 1.0 and sampler.exp2_series(5.0) == 32.0
    assert abs(sampler.LN2 - math.log(2.0)) < 1e-16 and abs(sampler.SQRT_HALF - math.sqrt(0.5)) < 1e-16
    seam = [sampler.ln_series(sampler.SQRT_HALF * (1.0 + i * 1e-16)) for i in range(-40, 41)]
    assert all(b >= a - 2e-16 for a, b in zip(seam, seam[1:]))
    ints = [sampler.exp2_series(4.0 + i * 2.0 ** -50) for i in range(-8, 9)]
    assert all(b >= a for a, b in zip(ints, ints[1:]))


def test_normal_draws_are_standard_normal():
    """a wrong box width or acceptance test skews the law: KS against N(0,1)"""
    st = sampler.Stream(5, 1)
    g = np.array([st.normal() for _ in range(40000)])
    assert stats.kstest(g, "norm").pvalue > 1e-3
    assert abs(g.mean()) < 0.02 and abs(g.std() - 1.0) < 0.02
    assert abs(stats.kurtosis(g)) < 0.1


def test_kernel_laws_multivariate():
    C, L, K = 20, 50000, 6000
    kr = oracle.sample_kernels(2002, K, C, L)
    ln, d, p, b, nch = kr["length"], kr["dilation"], kr["padding"], kr["bias"], kr["n_ch"]
    # length: uniform on {7, 9, 11}
    assert set(np.unique(ln)) == {7, 9, 11}
    for v in (7, 9, 11):
        assert abs((ln == v).mean() - 1 / 3) < 0.03
    # bias: U[-1, 1)
    assert b.dtype == np.float32 and b.min() >= -1.0 and b.max() < 1.0
    assert abs(b.mean()) < 0.03 and abs(b.var() - 1 / 3) < 0.02
    # dilation: 1 <= d <= floor((L-1)/(len-1)) and log2 d roughly uniform
    dmax = (L - 1) // (ln - 1)
    assert np.all(d >= 1) and np.all(d <= dmax)
    A = np.log2((L - 1) / (ln - 1))
    frac = np.log2(d + 0.5) / A          # centre of [log2 d, log2(d+1))
    assert abs(frac.mean() - 0.5) < 0.03
    assert abs((d == 1).mean() - np.mean(1.0 / A)) < 0.02          # P(d=1) = 1/A
    # padding: a fair coin between 0 and (len-1)*d/2
    padded = p != 0
    assert np.all(p[padded] == ((ln - 1) * d // 2)[padded])
    assert abs(padded.mean() - 0.5) < 0.03
    # output length is >= 1 for every kernel
    assert np.all(L + 2 * p - (ln - 1) * d >= 1)
    # channel count: P(m) = log(1 + 1/m) / log(10) on 1..9, mean 3.44
    assert nch.min() >= 1 and nch.max() <= 9
    for m in range(1, 10):
        assert abs((nch == m).mean() - math.log10(1 + 1 / m)) < 0.025
    assert abs(nch.mean() - 3.44) < 0.1
    # channels: distinct, in range, every channel used about equally
    use = np.zeros(C)
    for k in range(K):
        ch = kr["channels"][kr["ch_off"][k]: kr["ch_off"][k + 1]]
        assert len(set(ch.tolist())) == len(ch) == nch[k]
        assert ch.min() >= 0 and ch.max() < C
        use[ch] += 1
    assert np.all(np.abs(use / use.sum() - 1 / C) < 0.01)
    # weights: every (kernel, channel) row is centred; fp32; variance (len-1)/len
    assert kr["weights"].dtype == np.float32
    assert kr["w_off"][K] == (nch * ln).sum() == len(kr["weights"])
    rows9 = []
    for k in range(K):
        w = kr["weights"][kr["w_off"][k]: kr["w_off"][k + 1]].reshape(nch[k], ln[k])
        assert np.all(np.abs(w.astype(np.float64).sum(axis=1)) < 2e-6)
        if ln[k] == 9:
            rows9.append(w)
    rows9 = np.concatenate(rows9)
    assert abs(rows9.var() - 8 / 9) < 0.03


def test_kernel_laws_univariate():
    kr = oracle.sample_kernels(2000, 500, 1, 512)
    assert np.all(kr["n_ch"] == 1) and np.all(kr["channels"] == 0)
    assert kr["dilation"].max() <= 511 // 6
    assert np.all(512 + 2 * kr["padding"] - (kr["length"] - 1) * kr["dilation"] >= 1)


def test_streams_are_per_kernel_and_seeded():
    """kernel k depends only on (seed, k, C, L): any kernel can be drawn alone"""
    kr = oracle.sample_kernels(77, 30, 5, 400)
    ln, d, p, b, ch, w = oracle.sample_kernel(77, 17, 5, 400)
    assert (ln, d, p) == (kr["length"][17], kr["dilation"][17], kr["padding"][17])
    assert b == kr["bias"][17]
    assert ch == kr["channels"][kr["ch_off"][17]: kr["ch_off"][18]].tolist()
    assert np.array_equal(w.reshape(-1), kr["weights"][kr["w_off"][17]: kr["w_off"][18]])
    other = oracle.sample_kernels(78, 30, 5, 400)
    assert not np.array_equal(other["bias"], kr["bias"])


def test_known_answer_kernels():
    """stored kernels (bit patterns) guard against silent changes of the spec"""
    kat = json.load(open(os.path.join(GOLDEN, "sampler_kat.json")))
    for case in kat["cases"]:
        kr = oracle.sample_kernels(case["seed"], case["K"], case["C"], case["L"])
        for name in ("length", "dilation", "padding", "n_ch", "channels"):
            assert kr[name].tolist() == case[name], name
        assert kr["bias"].view(np.uint32).tolist() == case["bias_bits"]
        assert kr["weights"].view(np.uint32).tolist() == case["weight_bits"]
