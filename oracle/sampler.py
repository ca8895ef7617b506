"""Random kernel initialisation of the ROCKET transform -- oracle side.

TEST INFRASTRUCTURE ONLY: this module belongs to the CPU oracle.  It shares no
code with the HIP library; only tests, the smoke check and the benchmark's
cpu_baseline leg may import it.

Paper section 3.1 lists what every kernel draws:
  * a length chosen uniformly from {7, 9, 11};
  * weights from a normal distribution, then mean centred;
  * a bias from a uniform distribution on (-1, 1);
  * a coin flip between "same" padding and no padding;
  * a dilation drawn on an exponential scale up to the input length;
  * a random choice of the channels that are convolved.

The paper leaves the generator, the order of the draws and the multivariate
details open.  The readings used here (and, separately written, in the
library) are:

  generator   one SplitMix64 stream per kernel index, so any kernel can be
              sampled alone.  Every draw consumes exactly one 64-bit output.
  length      7 + 2*floor(3*u32 / 2^32)
  channels    count = floor(2^(u * log2(min(C,9)+1))) clamped to [1, min(C,9)],
              then a uniform subset without replacement (partial Fisher-Yates),
              weights attach to channels in the order they were drawn
  weights     N(0,1) by the Kinderman-Monahan ratio of uniforms, in fp64;
              each channel row is centred on its own mean (sum in index
              order, divided by the length) and then rounded once to fp32
  bias        (u32 >> 8) * 2^-23 - 1, exact in fp32, in [-1, 1)
  dilation    floor(2^(u * log2((L-1)/(len-1)))), clamped to
              [1, floor((L-1)/(len-1))]
  padding     low bit of a u32:  (len-1)*dilation/2 zeros on each side, or 0
  logarithm   the accept test of the normal draws and the two floors above must
  and power   fall the same way wherever the sampler runs, so ln, log2 and 2^y
              are not taken from a math library: they are the short series
              below (ln_series, exp2_series), built from IEEE additions,
              multiplications and divisions only, every one in a stated order
"""
import math

import numpy as np

MASK = (1 << 64) - 1
GAMMA = 0x9E3779B97F4A7C15
MUL1 = 0xBF58476D1CE4E5B9
MUL2 = 0x94D049BB133111EB
ROU_C = 0.8577638849607068  # sqrt(2/e), half-width of the ratio-of-uniforms box
TWO_M53 = 2.0 ** -53
TWO_M23 = 2.0 ** -23
LN2 = 0.6931471805599453        # ln 2, nearest double
SQRT_HALF = 0.7071067811865476  # sqrt(1/2), nearest double
LN_TERMS = 12                   # odd powers z, z^3, ... z^25 of the atanh series
EXP_TERMS = 19                  # Taylor terms of exp on [0, ln 2)


def ln_series(x):
    """Natural logarithm of a positive finite double.  x = m * 2^e with m in
    [sqrt(1/2), sqrt(2)); ln m = 2 atanh(z), z = (m-1)/(m+1), |z| < 0.172, by
    its series sum_i z^(2i+1)/(2i+1), i = 0..LN_TERMS, summed from the smallest
    term (Horner in z^2).  Truncation error below 1e-19; every operation is an
    IEEE double operation in the order written."""
    m, e = math.frexp(x)            # exact: m in [0.5, 1)
    if m < SQRT_HALF:
        m = m * 2.0                 # exact
        e -= 1
    z = (m - 1.0) / (m + 1.0)
    z2 = z * z
    s = 1.0 / (2 * LN_TERMS + 1)
    for i in range(LN_TERMS - 1, -1, -1):
        s = s * z2 + 1.0 / (2 * i + 1)
    return e * LN2 + (2.0 * z) * s


def log2_series(x):
    return ln_series(x) / LN2


def exp2_series(y):
    """2^y for 0 <= y < 1000: 2^floor(y) * exp(t), t = (y - floor(y)) * ln 2 in
    [0, ln 2), exp by its Taylor polynomial of degree EXP_TERMS in nested form
    (truncation error below 1e-19), scaled by the exact power of two."""
    n = math.floor(y)
    t = (y - n) * LN2
    s = 1.0
    for i in range(EXP_TERMS, 0, -1):
        s = 1.0 + (s * t) / i
    return math.ldexp(s, int(n))


def mix64(z):
    z &= MASK
    z = ((z ^ (z >> 30)) * MUL1) & MASK
    z = ((z ^ (z >> 27)) * MUL2) & MASK
    return z ^ (z >> 31)


class Stream:
    """SplitMix64 stream of kernel `k` under `seed`."""

    def __init__(self, seed, k):
        s = mix64((seed + GAMMA) & MASK)
        self.s = mix64((s + (k + 1) * GAMMA) & MASK)

    def next64(self):
        self.s = (self.s + GAMMA) & MASK
        return mix64(self.s)

    def u32(self):
        return self.next64() >> 32

    def u01(self):          # [0, 1)
        return (self.next64() >> 11) * TWO_M53

    def u_open(self):       # (0, 1]
        return ((self.next64() >> 11) + 1) * TWO_M53

    def normal(self):
        """Standard normal by the ratio of uniforms: (u, v) uniform on
        (0,1] x [-c, c), candidate x = v/u, accepted iff x^2 <= -4 ln u."""
        while True:
            u = self.u_open()
            v = ROU_C * (2.0 * self.u01() - 1.0)
            x = v / u
            if x * x <= -4.0 * ln_series(u):
                return x


def sample_kernel(seed, k, C, L):
    """Returns (length, dilation, padding, bias, channels, weights[n_ch][length])."""
    st = Stream(seed, k)
    length = 7 + 2 * ((st.u32() * 3) >> 32)

    m = min(C, 9)
    n_ch = int(math.floor(exp2_series(st.u01() * log2_series(float(m + 1)))))
    n_ch = max(1, min(n_ch, m))

    idx = list(range(C))
    for i in range(n_ch):
        j = i + ((st.u32() * (C - i)) >> 32)
        idx[i], idx[j] = idx[j], idx[i]
    channels = idx[:n_ch]

    weights = np.empty((n_ch, length), dtype=np.float32)
    for c in range(n_ch):
        g = [st.normal() for _ in range(length)]
        total = 0.0
        for v in g:
            total += v
        mean = total / length
        for j in range(length):
            weights[c, j] = np.float32(g[j] - mean)

    bias = np.float32((st.u32() >> 8) * TWO_M23 - 1.0)

    ratio = (L - 1) / (length - 1)
    dilation = int(math.floor(exp2_series(st.u01() * log2_series(ratio))))
    dilation = max(1, min(dilation, (L - 1) // (length - 1)))

    padding = ((length - 1) * dilation) // 2 if (st.u32() & 1) else 0
    return length, dilation, padding, bias, channels, weights


def sample_kernels(seed, K, C, L):
    """Flat arrays for K kernels, in the layout the transform functions take:
    length, dilation, padding (int32[K]), bias (float32[K]), n_ch (int32[K]),
    ch_off, w_off (int64[K+1]), channels (int32[sum n_ch]),
    weights (float32[sum n_ch*length], channel-major per kernel)."""
    if K < 1 or C < 1 or L < 11:
        raise ValueError("need K >= 1, C >= 1, L >= 11")
    length = np.empty(K, np.int32)
    dilation = np.empty(K, np.int32)
    padding = np.empty(K, np.int32)
    bias = np.empty(K, np.float32)
    n_ch = np.empty(K, np.int32)
    ch_off = np.zeros(K + 1, np.int64)
    w_off = np.zeros(K + 1, np.int64)
    chans, wts = [], []
    for k in range(K):
        ln, d, p, b, ch, w = sample_kernel(seed, k, C, L)
        length[k], dilation[k], padding[k], bias[k], n_ch[k] = ln, d, p, b, len(ch)
        ch_off[k + 1] = ch_off[k] + len(ch)
        w_off[k + 1] = w_off[k] + w.size
        chans.append(np.asarray(ch, np.int32))
        wts.append(w.reshape(-1))
    return {
        "K": K, "C": C, "L": L,
        "length": length, "dilation": dilation, "padding": padding,
        "bias": bias, "n_ch": n_ch, "ch_off": ch_off, "w_off": w_off,
        "channels": np.concatenate(chans), "weights": np.concatenate(wts),
    }
