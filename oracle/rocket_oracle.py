"""ctypes front end of the C oracle (rocket_oracle.c).

TEST INFRASTRUCTURE ONLY: part of the CPU oracle; shares nothing with the HIP
library.  Argument marshalling only -- every number is computed in the C file.
"""
import ctypes as C
import os

import numpy as np

from . import build as _build

# |y| below this may legitimately change sign in a float32 evaluation; hard-PPV
# counts are compared up to the number of such positions.
AMBIGUOUS_EPS = 1e-5

_lib = None


def _load():
    global _lib
    if _lib is None:
        path = _build.LIB
        if not os.path.exists(path):
            _build.build()
        _lib = C.CDLL(path)
        _lib.rk_oracle_conv.restype = C.c_int
        _lib.rk_oracle_transform.restype = C.c_int
        _lib.rk_oracle_backward.restype = C.c_int
        _lib.rk_oracle_num_threads.restype = C.c_int
    return _lib


def _p(a, t):
    return a.ctypes.data_as(C.POINTER(t))


def _arr(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def num_threads():
    return int(_load().rk_oracle_num_threads())


def set_threads(n):
    _load().rk_oracle_set_threads(C.c_int(int(n)))


def _kernel_args(kr):
    ks = {
        "length": _arr(kr["length"], np.int32), "dilation": _arr(kr["dilation"], np.int32),
        "padding": _arr(kr["padding"], np.int32), "bias": _arr(kr["bias"], np.float32),
        "n_ch": _arr(kr["n_ch"], np.int32), "ch_off": _arr(kr["ch_off"], np.int64),
        "channels": _arr(kr["channels"], np.int32), "w_off": _arr(kr["w_off"], np.int64),
        "weights": _arr(kr["weights"], np.float32),
    }
    args = [_p(ks["length"], C.c_int), _p(ks["dilation"], C.c_int), _p(ks["padding"], C.c_int),
            _p(ks["bias"], C.c_float), _p(ks["n_ch"], C.c_int),
            _p(ks["ch_off"], C.c_longlong), _p(ks["channels"], C.c_int),
            _p(ks["w_off"], C.c_longlong), _p(ks["weights"], C.c_float)]
    return ks, args


def conv_output(x_series, kr, k):
    """fp64 conv output y[0..n) of kernel k over one series (C x L float32)."""
    x = _arr(x_series, np.float32)
    Cn, L = x.shape
    lo, hi = int(kr["ch_off"][k]), int(kr["ch_off"][k + 1])
    wlo, whi = int(kr["w_off"][k]), int(kr["w_off"][k + 1])
    ch = _arr(kr["channels"][lo:hi], np.int32)
    w = _arr(kr["weights"][wlo:whi], np.float32)
    ln, d, p = int(kr["length"][k]), int(kr["dilation"][k]), int(kr["padding"][k])
    n = L + 2 * p - (ln - 1) * d
    y = np.empty(max(n, 1), np.float64)
    r = _load().rk_oracle_conv(_p(x, C.c_float), Cn, L, ln, d, p, C.c_double(float(kr["bias"][k])),
                               hi - lo, _p(ch, C.c_int), _p(w, C.c_float), _p(y, C.c_double))
    if r < 1:
        raise ValueError("kernel does not fit the series")
    return y[:r]


def transform(x, kr, lam=10.0, shift=-3.0, sel=None, amb_eps=AMBIGUOUS_EPS):
    """Pooled features of x (B x C x L float32) for the kernels in `sel`
    (default: all).  Returns a dict of B x nsel arrays: max, count, ambiguous,
    ppv, softppv (fp64 / int64), argmax, gap, and n_out (nsel)."""
    x = _arr(x, np.float32)
    B, Cn, L = x.shape
    K = len(kr["length"])
    sel = np.arange(K, dtype=np.int32) if sel is None else _arr(sel, np.int32)
    ns = len(sel)
    ks, kargs = _kernel_args(kr)
    omax = np.empty((B, ns), np.float64)
    osoft = np.empty((B, ns), np.float64)
    ogap = np.empty((B, ns), np.float64)
    ocnt = np.empty((B, ns), np.int64)
    oamb = np.empty((B, ns), np.int64)
    oarg = np.empty((B, ns), np.int64)
    on = np.empty(ns, np.int32)
    r = _load().rk_oracle_transform(
        _p(x, C.c_float), B, Cn, L, *kargs, ns, _p(sel, C.c_int),
        C.c_double(lam), C.c_double(shift), C.c_double(amb_eps),
        _p(omax, C.c_double), _p(ocnt, C.c_longlong), _p(oamb, C.c_longlong),
        _p(osoft, C.c_double), _p(on, C.c_int), _p(oarg, C.c_longlong), _p(ogap, C.c_double))
    if r != 0:
        raise ValueError("a kernel does not fit the series")
    return {"max": omax, "count": ocnt, "ambiguous": oamb, "softppv": osoft,
            "ppv": ocnt / on[None, :].astype(np.float64), "n_out": on,
            "argmax": oarg, "gap": ogap, "sel": sel}


def backward(x, kr, g_soft, g_max=None, lam=10.0, shift=-3.0, sel=None):
    """Gradients of sum(g_soft*softPPV) [+ sum(g_max*max)] with respect to the
    stored weights and biases, summed over the batch.  g_* are B x nsel.
    Returns (grad_w [like weights], grad_b [K]) in fp64."""
    x = _arr(x, np.float32)
    B, Cn, L = x.shape
    K = len(kr["length"])
    sel = np.arange(K, dtype=np.int32) if sel is None else _arr(sel, np.int32)
    ns = len(sel)
    ks, kargs = _kernel_args(kr)
    gs = _arr(g_soft, np.float64).reshape(B, ns)
    gm = None if g_max is None else _arr(g_max, np.float64).reshape(B, ns)
    gw = np.empty(int(kr["w_off"][K]), np.float64)
    gb = np.empty(K, np.float64)
    r = _load().rk_oracle_backward(
        _p(x, C.c_float), B, Cn, L, K, *kargs, ns, _p(sel, C.c_int),
        C.c_double(lam), C.c_double(shift), _p(gs, C.c_double),
        None if gm is None else _p(gm, C.c_double), _p(gw, C.c_double), _p(gb, C.c_double))
    if r != 0:
        raise ValueError("a kernel does not fit the series")
    return gw, gb
