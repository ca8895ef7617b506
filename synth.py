"""Seeded synthetic workloads with the shapes of the paper's data.

The paper's examples are 20 sensor channels x 50,000 timesteps of integer
intensities, z-normalised per channel (sections 4.1 and 4.3); that data set is
proprietary, so these generators stand in for it.  This module holds input
generation only -- none of the transform's arithmetic -- and is the one module
both the CPU oracle's tests and the GPU tests draw their inputs from.

Every example b of workload i is generated from its own stream
(seed_x(i), b), so a sub-batch is a prefix of the full batch.
"""
import numpy as np
from scipy.signal import lfilter

F_MAX, F_PPV, F_SOFTPPV = 1, 2, 4

# B, C, L, K and the pooled features of the five workloads
CONFIGS = {
    0: dict(name="univariate-tiny", B=16, C=1, L=512, K=500, features=F_MAX | F_PPV),
    1: dict(name="univariate-standard", B=256, C=1, L=1000, K=10000,
            features=F_MAX | F_PPV | F_SOFTPPV),
    2: dict(name="multivariate-20x50k", B=64, C=20, L=50000, K=10000, features=F_MAX | F_PPV),
    3: dict(name="multivariate-20x50k-grad", B=60, C=20, L=50000, K=10000,
            features=F_MAX | F_SOFTPPV),
    4: dict(name="long-20x200k", B=8, C=20, L=200000, K=20000,
            features=F_MAX | F_PPV | F_SOFTPPV),
}


def seed_x(i):
    return 1000 + i


def seed_k(i):
    return 2000 + i


def seed_g(i):
    return 3000 + i


def _znorm(a):
    """Mean-centre each row (last axis) and divide by its population std."""
    a = a - a.mean(axis=-1, keepdims=True)
    return a / a.std(axis=-1, keepdims=True)


def _ar1_channels(rng, C, L):
    """C independent AR(1) rows, phi = 0.95, unit innovations, started from the
    stationary law, with a gain in U(0.5, 2) and an offset in U(-1, 1)."""
    phi = 0.95
    e = rng.standard_normal((C, L))
    e[:, 0] /= np.sqrt(1.0 - phi * phi)
    a = lfilter([1.0], [1.0, -phi], e, axis=-1)
    gain = rng.uniform(0.5, 2.0, size=(C, 1))
    offset = rng.uniform(-1.0, 1.0, size=(C, 1))
    return gain * a + offset


def _example(i, b):
    cfg = CONFIGS[i]
    C, L = cfg["C"], cfg["L"]
    rng = np.random.Generator(np.random.PCG64([seed_x(i), b]))
    if i == 0:
        return rng.standard_normal((C, L))
    if i == 1:
        t = np.arange(L, dtype=np.float64)
        f = rng.uniform(1.0, 50.0, size=3) / L
        ph = rng.uniform(0.0, 2.0 * np.pi, size=3)
        s = np.sin(2.0 * np.pi * f[:, None] * t[None, :] + ph[:, None]).sum(axis=0)
        s = s + 0.3 * rng.standard_normal(L)
        return _znorm(s[None, :])
    a = _znorm(_ar1_channels(rng, C, L))
    if i == 4:
        mask = rng.random((C, L)) < 0.01
        spikes = 10.0 * rng.standard_normal((C, L))
        a = np.where(mask, spikes, a)
    return a


def make_input(i, B=None):
    """float32 array (B, C, L) of workload i; B defaults to the workload's."""
    cfg = CONFIGS[i]
    B = cfg["B"] if B is None else B
    out = np.empty((B, cfg["C"], cfg["L"]), np.float32)
    for b in range(B):
        out[b] = _example(i, b).astype(np.float32)
    return out


def make_input_u8(i, B=None):
    """uint8 array (B, C, L): workload i before normalisation, as 8-bit sensor intensities
    (the paper's raw data are integers 0..255): each channel gets its own gain and offset,
    is clipped to the sensor range and rounded."""
    cfg = CONFIGS[i]
    B = cfg["B"] if B is None else B
    out = np.empty((B, cfg["C"], cfg["L"]), np.uint8)
    for b in range(B):
        a = _example(i, b)
        rng = np.random.Generator(np.random.PCG64([seed_x(i), b, 8]))
        gain = rng.uniform(15.0, 45.0, size=(cfg["C"], 1))
        offset = rng.uniform(90.0, 160.0, size=(cfg["C"], 1))
        out[b] = np.clip(np.rint(a * gain + offset), 0, 255).astype(np.uint8)
    return out


def make_upstream_grad(i, B, n_features):
    """N(0,1) upstream gradient (B, n_features) float32 for the backward workloads."""
    rng = np.random.Generator(np.random.PCG64(seed_g(i)))
    return rng.standard_normal((B, n_features)).astype(np.float32)


def pick_kernels(kernels, count, seed=0):
    """Indices of a parity sub-sample of kernels: the largest dilation, the
    shortest output, then kernels spread evenly over the dilation-sorted order."""
    K = len(kernels["length"])
    if count >= K:
        return np.arange(K, dtype=np.int32)
    d = np.asarray(kernels["dilation"]).astype(np.int64)
    ln = np.asarray(kernels["length"]).astype(np.int64)
    p = np.asarray(kernels["padding"]).astype(np.int64)
    n_out = 2 * p - (ln - 1) * d  # + L, the same for all
    chosen = {int(np.argmax(d)), int(np.argmin(n_out)), int(np.argmin(d))}
    order = np.argsort(d, kind="stable")
    rng = np.random.Generator(np.random.PCG64(seed))
    step = K / float(count)
    for q in range(count):
        lo = int(q * step)
        hi = max(lo + 1, int((q + 1) * step))
        chosen.add(int(order[rng.integers(lo, hi)]))
        if len(chosen) >= count:
            break
    return np.array(sorted(chosen), dtype=np.int32)
