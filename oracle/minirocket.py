"""MINIROCKET-style variant of the transform -- oracle side.

TEST INFRASTRUCTURE ONLY: part of the CPU oracle; shares nothing with the HIP library.

The paper describes MINIROCKET only in its related-work section (section 2) and names it as the
extension to build next (section 6).  What that paragraph fixes:
  * the kernels are "binary": two weight values, so that the convolution can be done by additions;
  * the weights come from a predetermined set instead of being drawn at random;
  * the biases are sampled from the input data;
  * there is no max pooling, only PPV: one feature per kernel.
Everything else is this build's reading (the original MINIROCKET publication is not available here:
PARITY UNPINNED against the original model; what is pinned is this definition):
  * length 9 (the middle one of the lengths of section 3.1) and the weight values -1 and 2; a kernel
    has three weights of 2 and six of -1, so its weights sum to zero as the mean-centred weights of
    section 3.1 do.  The predetermined set is all C(9,3) = 84 such kernels, in lexicographic order of
    the positions of the 2s.  The same weights apply to every channel the kernel uses.
  * kernels come in groups of 84 (the whole set) that share dilation, padding and channel subset;
    those three are drawn per group by the laws of section 3.1 (exponential dilation, fair padding
    coin, channel count floor(2^(u log2(min(C,9)+1))) and a uniform subset), from the SplitMix64
    stream of (seed, group) -- in that order: channel count, channels, dilation, padding.
  * convolution by additions: with S the positions of the 2s,
        sum_j w_j x[t + j d] = 3 * sum_{j in S} x[t + j d] - sum_{all j} x[t + j d];
    this module computes it that way (shifted sums), independently of the oracle's conv routine.
  * bias from the data: kernel k draws a training example b* and a level q in [0,1) from the stream
    of (seed + 1, k); its bias is minus the order statistic of rank floor(q (n-1)) (0-based, ascending)
    of its own bias-free output on that example, so that on that example
    PPV = (n - 1 - rank) / n exactly when the outputs are distinct (Eq. 1 is strict).
  * feature: PPV (Eq. 1-2) of output + bias, one per kernel, kernels in (group, set) order.
"""
import itertools
import math

import numpy as np

from . import sampler
from .rocket_oracle import transform

LENGTH = 9
LOW, HIGH = -1.0, 2.0
SET = list(itertools.combinations(range(LENGTH), 3))      # 84 position triples, lexicographic
SET_SIZE = len(SET)


def minirocket_kernels(seed, groups, C, L):
    """Kernel arrays (the layout of sample_kernels, bias = 0) of `groups` groups of 84 kernels for
    series of C channels and L samples, plus 'group' (int32[K])."""
    if groups < 1 or C < 1 or L < LENGTH:
        raise ValueError("need groups >= 1, C >= 1, L >= 9")
    K = groups * SET_SIZE
    m = min(C, 9)
    length = np.full(K, LENGTH, np.int32)
    dilation = np.empty(K, np.int32)
    padding = np.empty(K, np.int32)
    n_ch = np.empty(K, np.int32)
    chans, wts = [], []
    for g in range(groups):
        st = sampler.Stream(seed, g)
        count = int(math.floor(sampler.exp2_series(st.u01() * sampler.log2_series(float(m + 1)))))
        count = max(1, min(count, m))
        idx = list(range(C))
        for i in range(count):
            j = i + ((st.u32() * (C - i)) >> 32)
            idx[i], idx[j] = idx[j], idx[i]
        ch = idx[:count]
        ratio = (L - 1) / (LENGTH - 1)
        d = int(math.floor(sampler.exp2_series(st.u01() * sampler.log2_series(ratio))))
        d = max(1, min(d, (L - 1) // (LENGTH - 1)))
        p = ((LENGTH - 1) * d) // 2 if (st.u32() & 1) else 0
        for s, triple in enumerate(SET):
            k = g * SET_SIZE + s
            dilation[k], padding[k], n_ch[k] = d, p, count
            row = np.full(LENGTH, LOW, np.float32)
            row[list(triple)] = HIGH
            chans.append(np.asarray(ch, np.int32))
            wts.append(np.tile(row, count))
    ch_off = np.concatenate([[0], np.cumsum(n_ch)]).astype(np.int64)
    w_off = np.concatenate([[0], np.cumsum(n_ch.astype(np.int64) * LENGTH)]).astype(np.int64)
    return {
        "K": K, "C": C, "L": L, "length": length, "dilation": dilation, "padding": padding,
        "bias": np.zeros(K, np.float32), "n_ch": n_ch, "ch_off": ch_off, "w_off": w_off,
        "channels": np.concatenate(chans), "weights": np.concatenate(wts),
        "group": np.repeat(np.arange(groups, dtype=np.int32), SET_SIZE),
    }


def output_by_additions(x_series, kr, k):
    """Bias-free output of kernel k over one series (C x L), by shifted sums only:
    3 * (sum over the taps that carry a 2) - (sum over all taps), on the channel-summed,
    zero-padded series.  fp64."""
    x = np.asarray(x_series, np.float64)
    L = x.shape[1]
    d, p = int(kr["dilation"][k]), int(kr["padding"][k])
    ch = kr["channels"][int(kr["ch_off"][k]):int(kr["ch_off"][k + 1])]
    total = np.zeros(L + 2 * p, np.float64)
    total[p:p + L] = x[ch].sum(axis=0)
    n = L + 2 * p - (LENGTH - 1) * d
    taps = [total[j * d:j * d + n] for j in range(LENGTH)]
    w = kr["weights"][int(kr["w_off"][k]):int(kr["w_off"][k]) + LENGTH]
    high = sum(taps[j] for j in range(LENGTH) if w[j] == HIGH)
    return 3.0 * high - sum(taps)


def bias_draws(seed, K, n_train):
    """(example, level) of every kernel: example uniform on [0, n_train), level uniform on [0, 1)."""
    ex = np.empty(K, np.int64)
    q = np.empty(K, np.float64)
    for k in range(K):
        st = sampler.Stream(seed + 1, k)
        ex[k] = (st.u32() * n_train) >> 32
        q[k] = st.u01()
    return ex, q


def minirocket_fit_bias(x_train, kr, seed):
    """Returns a copy of kr whose biases are drawn from the training batch x_train (B x C x L):
    bias_k = -(order statistic of rank floor(q_k (n_k - 1)) of kernel k's output on example b*_k),
    rounded to float32; also returns the examples and ranks used."""
    x_train = np.asarray(x_train, np.float32)
    K = len(kr["length"])
    ex, q = bias_draws(seed, K, x_train.shape[0])
    bias = np.empty(K, np.float32)
    rank = np.empty(K, np.int64)
    for k in range(K):
        y = output_by_additions(x_train[ex[k]], kr, k)
        rank[k] = int(math.floor(q[k] * (len(y) - 1)))
        bias[k] = np.float32(-np.partition(y, rank[k])[rank[k]])
    out = dict(kr)
    out["bias"] = bias
    return out, ex, rank


def minirocket_transform(x, kr, sel=None):
    """PPV features (B x nsel, fp64) with the integer counts, ambiguity counts and output lengths."""
    o = transform(x, kr, sel=sel)
    return {"ppv": o["ppv"], "count": o["count"], "ambiguous": o["ambiguous"], "n_out": o["n_out"]}
