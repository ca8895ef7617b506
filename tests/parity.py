"""Shared comparison rules of the GPU-vs-oracle parity tests.

Tolerances (fp32 path against the fp64 oracle):
  max, softPPV   |gpu - oracle| <= 1e-4 * |oracle| + 1e-5
  hard PPV       integer counts; |count_gpu - count_oracle| <= number of
                 positions where the oracle's conv output has |y| < 1e-5
"""
import numpy as np

import oracle

RTOL, ATOL = 1e-4, 1e-5


def planes(out, mask, K):
    """Splits a (B, F*K) feature matrix into a dict of (B, K) planes."""
    res, f = {}, 0
    for bit, name in ((1, "max"), (2, "ppv"), (4, "softppv")):
        if mask & bit:
            res[name] = out[:, f * K:(f + 1) * K]
            f += 1
    assert out.shape[1] == f * K
    return res


def check_forward(x, kr, out_gpu, mask, lam=10.0, shift=-3.0, sel=None, rows=None):
    """Compares the GPU features of series `rows` (default all) and kernels
    `sel` (default all) with the oracle.  Returns the oracle result."""
    K = len(kr["length"])
    out_gpu = np.asarray(out_gpu, dtype=np.float64)
    rows = np.arange(x.shape[0]) if rows is None else np.asarray(rows)
    sel = np.arange(K, dtype=np.int32) if sel is None else np.asarray(sel, np.int32)
    ref = oracle.transform(x[rows], kr, lam=lam, shift=shift, sel=sel)
    got = planes(out_gpu[rows], mask, K)
    assert np.all(np.isfinite(out_gpu[rows]))
    if "max" in got:
        err = np.abs(got["max"][:, sel] - ref["max"])
        bad = err > RTOL * np.abs(ref["max"]) + ATOL
        assert not bad.any(), ("max", np.argwhere(bad)[:5], err.max())
    if "softppv" in got:
        err = np.abs(got["softppv"][:, sel] - ref["softppv"])
        bad = err > RTOL * np.abs(ref["softppv"]) + ATOL
        assert not bad.any(), ("softppv", np.argwhere(bad)[:5], err.max())
    if "ppv" in got:
        n = ref["n_out"][None, :].astype(np.float64)
        cnt = np.rint(got["ppv"][:, sel] * n)
        assert np.all(np.abs(cnt / n - got["ppv"][:, sel]) < 1e-6)
        diff = np.abs(cnt - ref["count"])
        bad = diff > ref["ambiguous"]
        assert not bad.any(), ("ppv", np.argwhere(bad)[:5], diff.max())
    return ref
