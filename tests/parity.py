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


# Gradients are sums of up to B*n (millions of) signed fp32 terms q_t*x_t, so an
# element's error is bounded relative to the magnitude of the terms, not of the
# (possibly cancelling) sum.  The scale used here is the largest |gradient| of
# the same kernel: |gpu - oracle| <= G_RTOL*|oracle| + G_STOL*max_k|oracle|.
# Measured errors sit near 1e-6 of that scale at lambda = 10.  The fp32 error of a conv
# output (about 1e-6) enters q = g*(lambda/n)*s(1-s) through its slope lambda*(1-2s)*q,
# so the scale term grows with lambda beyond 10.
G_RTOL, G_STOL = 1e-4, 1e-5


def grad_scale_tol(lam):
    return G_STOL * max(1.0, abs(lam) / 10.0)


def check_backward(x, kr, gw_gpu, gb_gpu, g_soft, g_max, lam, shift, sel=None, report=None):
    """Compares GPU gradients with the oracle for the kernels in sel (default all)."""
    K = len(kr["length"])
    sel = np.arange(K, dtype=np.int32) if sel is None else np.asarray(sel, np.int32)
    gs = np.asarray(g_soft, np.float64)[:, sel]
    gm = None if g_max is None else np.asarray(g_max, np.float64)[:, sel]
    gw_ref, gb_ref = oracle.backward(x, kr, gs, gm, lam=lam, shift=shift, sel=sel)
    gw_gpu = np.asarray(gw_gpu, np.float64)
    gb_gpu = np.asarray(gb_gpu, np.float64)
    assert np.all(np.isfinite(gw_gpu)) and np.all(np.isfinite(gb_gpu))
    worst = 0.0
    for k in sel:
        lo, hi = int(kr["w_off"][k]), int(kr["w_off"][k + 1])
        ref = np.concatenate([gw_ref[lo:hi], [gb_ref[k]]])
        got = np.concatenate([gw_gpu[lo:hi], [gb_gpu[k]]])
        scale = np.abs(ref).max()
        err = np.abs(got - ref)
        bound = G_RTOL * np.abs(ref) + grad_scale_tol(lam) * scale + 1e-12
        worst = max(worst, float((err / bound).max()))
        assert np.all(err <= bound), (int(k), float(err.max()), float(scale))
    if report is not None:
        report["worst_ratio"] = worst
    return gw_ref, gb_ref
