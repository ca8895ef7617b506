"""Python binding of librocket_mi355x.so (include/rocket.h), same names as the C ABI.

Argument marshalling only: every step of the transform runs in the HIP
library.  torch supplies device memory and the current stream.  There is no
CPU fallback: importing works without a GPU (kernel sampling is host code),
but the compute calls need the library and a device and fail loudly otherwise.
"""
import ctypes as C
import os

import numpy as np

ROCKET_F_MAX, ROCKET_F_PPV, ROCKET_F_SOFTPPV = 1, 2, 4
ROCKET_OK, ROCKET_EINVAL, ROCKET_ENOMEM, ROCKET_EHIP, ROCKET_ESHAPE, ROCKET_EWORKSPACE = 0, -1, -2, -3, -4, -5

_HERE = os.path.dirname(os.path.abspath(__file__))
# the in-tree library; the environment variable ROCKET_LIB names another build of it
LIB_PATH = os.environ.get("ROCKET_LIB") or os.path.join(_HERE, "librocket_mi355x.so")

EXPORTS = [
    "rocket_make_kernels", "rocket_kernels_import", "rocket_kernels_view_get",
    "rocket_kernels_set_params", "rocket_num_features", "rocket_workspace_bytes",
    "rocket_transform", "rocket_transform_noalloc", "rocket_soft_ppv_backward", "rocket_transform_u8", "rocket_soft_ppv_backward_u8",
    "rocket_work_per_series", "rocket_jobs_view_get",
    "rocket_profile_enable", "rocket_profile_read", "rocket_calibrate_fma", "rocket_calibrate_units",
    "rocket_ridge_workspace_bytes", "rocket_ridge_fit", "rocket_ridge_predict", "rocket_infer",
    "rocket_mse_grad", "rocket_sgd_update", "rocket_train_workspace_bytes", "rocket_train_step",
    "rocket_kernels_subset",
    "rocket_minirocket_kernels", "rocket_minirocket_fit_workspace_bytes", "rocket_minirocket_fit_bias",
    "rocket_minirocket_workspace_bytes", "rocket_minirocket_transform", "rocket_minirocket_transform_u8",
    "rocket_minirocket_jobs_view_get",
    "rocket_free_kernels", "rocket_last_error",
]


class RocketError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("rocket error %d: %s" % (code, message))
        self.code = code


class _View(C.Structure):
    _fields_ = [
        ("K", C.c_int32), ("C", C.c_int32), ("L", C.c_int32),
        ("total_channels", C.c_int64), ("total_weights", C.c_int64),
        ("length", C.POINTER(C.c_int32)), ("dilation", C.POINTER(C.c_int32)),
        ("padding", C.POINTER(C.c_int32)), ("n_ch", C.POINTER(C.c_int32)),
        ("bias", C.POINTER(C.c_float)),
        ("ch_off", C.POINTER(C.c_int64)), ("w_off", C.POINTER(C.c_int64)),
        ("channels", C.POINTER(C.c_int32)), ("weights", C.POINTER(C.c_float)),
    ]


_lib = None


def load_library():
    """Loads the in-tree library; builds it first only if it is absent."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from . import build as _build
        _build.build()
    lib = C.CDLL(LIB_PATH)
    vp, i32, u32, u64, f32 = C.c_void_p, C.c_int32, C.c_uint32, C.c_uint64, C.c_float
    lib.rocket_make_kernels.argtypes = [u64, i32, i32, i32, C.POINTER(vp)]
    lib.rocket_kernels_import.argtypes = [i32, i32, i32, vp, vp, vp, vp, vp, vp, vp, C.POINTER(vp)]
    lib.rocket_kernels_view_get.argtypes = [vp, C.POINTER(_View)]
    lib.rocket_kernels_set_params.argtypes = [vp, vp, vp]
    lib.rocket_num_features.argtypes = [u32]
    lib.rocket_num_features.restype = i32
    lib.rocket_workspace_bytes.argtypes = [vp, i32, u32, C.c_int]
    lib.rocket_workspace_bytes.restype = C.c_size_t
    lib.rocket_transform.argtypes = [vp, vp, i32, u32, f32, f32, vp, vp, C.c_size_t, vp]
    lib.rocket_transform_noalloc.argtypes = [vp, vp, i32, u32, f32, f32, vp, vp]
    lib.rocket_soft_ppv_backward.argtypes = [vp, vp, i32, u32, vp, f32, f32, C.c_int, vp, vp, vp, C.c_size_t, vp]
    lib.rocket_transform_u8.argtypes = lib.rocket_transform.argtypes
    lib.rocket_soft_ppv_backward_u8.argtypes = lib.rocket_soft_ppv_backward.argtypes
    lib.rocket_jobs_view_get.argtypes = [vp, C.POINTER(i32)] + [C.POINTER(C.POINTER(i32))] * 4 + [C.POINTER(i32)]
    lib.rocket_work_per_series.argtypes = [vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.rocket_profile_enable.argtypes = [vp, C.c_int]
    lib.rocket_profile_read.argtypes = [vp, C.POINTER(i32), C.POINTER(C.c_double)]
    lib.rocket_calibrate_fma.argtypes = [C.POINTER(C.c_double), vp]
    lib.rocket_calibrate_units.argtypes = [C.POINTER(C.c_double), i32, vp]
    lib.rocket_ridge_workspace_bytes.argtypes = [i32, i32]
    lib.rocket_ridge_workspace_bytes.restype = C.c_size_t
    lib.rocket_ridge_fit.argtypes = [vp, vp, i32, i32, C.c_double, vp, vp, vp, C.c_size_t, vp]
    lib.rocket_ridge_predict.argtypes = [vp, i32, i32, vp, vp, vp, vp]
    lib.rocket_infer.argtypes = [vp, vp, C.c_int, i32, u32, f32, f32, vp, vp, vp, vp, vp, C.c_size_t, vp]
    lib.rocket_mse_grad.argtypes = [vp, vp, vp, i32, i32, vp, vp, vp]
    lib.rocket_sgd_update.argtypes = [vp, vp, vp, f32, C.c_int, vp]
    lib.rocket_train_workspace_bytes.argtypes = [vp, i32, u32]
    lib.rocket_train_workspace_bytes.restype = C.c_size_t
    lib.rocket_train_step.argtypes = [vp, vp, C.c_int, i32, u32, f32, f32, vp, vp, vp, f32, C.c_int, vp, vp,
                                      C.c_size_t, vp]
    lib.rocket_kernels_subset.argtypes = [vp, vp, i32, C.POINTER(vp)]
    lib.rocket_minirocket_kernels.argtypes = [u64, i32, i32, i32, C.POINTER(vp)]
    lib.rocket_minirocket_fit_workspace_bytes.argtypes = [vp, i32]
    lib.rocket_minirocket_fit_workspace_bytes.restype = C.c_size_t
    lib.rocket_minirocket_fit_bias.argtypes = [vp, vp, i32, u64, vp, C.c_size_t, vp]
    lib.rocket_minirocket_workspace_bytes.argtypes = [vp, i32]
    lib.rocket_minirocket_workspace_bytes.restype = C.c_size_t
    lib.rocket_minirocket_transform.argtypes = [vp, vp, i32, vp, vp, C.c_size_t, vp]
    lib.rocket_minirocket_transform_u8.argtypes = [vp, vp, i32, vp, vp, C.c_size_t, vp]
    lib.rocket_minirocket_jobs_view_get.argtypes = [vp, C.POINTER(i32), C.POINTER(C.POINTER(i32))]
    lib.rocket_free_kernels.argtypes = [vp]
    lib.rocket_free_kernels.restype = None
    lib.rocket_last_error.restype = C.c_char_p
    _lib = lib
    return lib


def rocket_last_error():
    return load_library().rocket_last_error().decode()


def _check(rc):
    if rc != ROCKET_OK:
        raise RocketError(rc, rocket_last_error())


def rocket_num_features(mask):
    return int(load_library().rocket_num_features(mask))


class Kernels:
    """Owns a rocket_kernels handle."""

    def __init__(self, handle):
        self._h = C.c_void_p(handle)
        # the sizes never change; keeping them here lets the compute wrappers check their
        # arguments without asking the library for a view (which, after a training update,
        # would wait for the device and download the parameters)
        v = _View()
        _check(load_library().rocket_kernels_view_get(self._h, C.byref(v)))
        self.K, self.C, self.L = int(v.K), int(v.C), int(v.L)
        self.total_channels, self.total_weights = int(v.total_channels), int(v.total_weights)

    @property
    def handle(self):
        if not self._h:
            raise RocketError(ROCKET_EINVAL, "kernels already freed")
        return self._h

    def free(self):
        if self._h:
            load_library().rocket_free_kernels(self._h)
            self._h = C.c_void_p(None)

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass


def rocket_make_kernels(seed, K, C_, L):
    out = C.c_void_p()
    _check(load_library().rocket_make_kernels(seed, K, C_, L, C.byref(out)))
    return Kernels(out.value)


def _np(a, dt):
    return np.ascontiguousarray(a, dtype=dt)


def rocket_kernels_import(K, C_, L, length, dilation, padding, bias, n_ch, channels, weights):
    arrs = [_np(length, np.int32), _np(dilation, np.int32), _np(padding, np.int32), _np(bias, np.float32),
            _np(n_ch, np.int32), _np(channels, np.int32), _np(weights, np.float32)]
    out = C.c_void_p()
    _check(load_library().rocket_kernels_import(K, C_, L, *[a.ctypes.data for a in arrs], C.byref(out)))
    return Kernels(out.value)


def rocket_kernels_view_get(kernels):
    """Copies of the handle's arrays, keyed like the C struct."""
    v = _View()
    _check(load_library().rocket_kernels_view_get(kernels.handle, C.byref(v)))
    K = v.K

    def arr(ptr, n, dt):
        return np.ctypeslib.as_array(ptr, shape=(n,)).astype(dt, copy=True) if n else np.zeros(0, dt)

    return {
        "K": K, "C": v.C, "L": v.L,
        "length": arr(v.length, K, np.int32), "dilation": arr(v.dilation, K, np.int32),
        "padding": arr(v.padding, K, np.int32), "n_ch": arr(v.n_ch, K, np.int32),
        "bias": arr(v.bias, K, np.float32),
        "ch_off": arr(v.ch_off, K + 1, np.int64), "w_off": arr(v.w_off, K + 1, np.int64),
        "channels": arr(v.channels, v.total_channels, np.int32),
        "weights": arr(v.weights, v.total_weights, np.float32),
    }


def rocket_kernels_set_params(kernels, weights=None, bias=None):
    w = None if weights is None else _np(weights, np.float32)
    b = None if bias is None else _np(bias, np.float32)
    _check(load_library().rocket_kernels_set_params(
        kernels.handle, None if w is None else w.ctypes.data, None if b is None else b.ctypes.data))


def rocket_workspace_bytes(kernels, B, feature_mask, backward=False):
    return int(load_library().rocket_workspace_bytes(kernels.handle, B, feature_mask, int(bool(backward))))


def rocket_jobs_view_get(kernels):
    """dict of int32 arrays (copies): kernel, row0, row1, flags of every job, in launch order."""
    n, stride = C.c_int32(), C.c_int32()
    ptrs = [C.POINTER(C.c_int32)() for _ in range(4)]
    _check(load_library().rocket_jobs_view_get(kernels.handle, C.byref(n), *[C.byref(p) for p in ptrs], C.byref(stride)))
    step = stride.value // 4
    out = {}
    for name, p in zip(("kernel", "row0", "row1", "flags"), ptrs):
        out[name] = np.ctypeslib.as_array(p, shape=(n.value * step,))[::step].copy()
    return out


def rocket_work_per_series(kernels):
    fma, outs = C.c_double(), C.c_double()
    _check(load_library().rocket_work_per_series(kernels.handle, C.byref(fma), C.byref(outs)))
    return fma.value, outs.value


def rocket_profile_enable(kernels, enable=True):
    _check(load_library().rocket_profile_enable(kernels.handle, int(bool(enable))))


def rocket_profile_read(kernels):
    """(launches, total milliseconds) of the dominant kernel since the last read."""
    n, ms = C.c_int32(), C.c_double()
    _check(load_library().rocket_profile_read(kernels.handle, C.byref(n), C.byref(ms)))
    return n.value, ms.value


def _torch():
    import torch
    if not torch.cuda.is_available():
        raise RocketError(ROCKET_EHIP, "no GPU visible: the transform has no CPU path")
    return torch


def _stream_ptr(torch, stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return C.c_void_p(s.cuda_stream)


def _workspace(torch, kernels, B, mask, backward, workspace, device):
    need = rocket_workspace_bytes(kernels, B, mask, backward)
    if workspace is None:
        workspace = torch.empty(need, dtype=torch.uint8, device=device)
    return workspace, need


def rocket_transform(kernels, x, feature_mask, lam=10.0, shift=-3.0, out=None, workspace=None, stream=None,
                     _dtype="float32", _entry="rocket_transform"):
    """x: float32 CUDA tensor (B, C, L), contiguous.  Returns out (B, F*K)."""
    torch = _torch()
    if not (x.is_cuda and x.dtype == getattr(torch, _dtype) and x.is_contiguous() and x.dim() == 3):
        raise RocketError(ROCKET_EINVAL, "x must be a contiguous %s CUDA tensor of shape (B, C, L)" % _dtype)
    v = kernels
    B = x.shape[0]
    if x.shape[1] != v.C or x.shape[2] != v.L:
        raise RocketError(ROCKET_ESHAPE, "x is (B, %d, %d) but the kernels were made for (%d, %d)"
                          % (x.shape[1], x.shape[2], v.C, v.L))
    F = rocket_num_features(feature_mask)
    if out is None:
        out = torch.empty((B, max(F, 1) * v.K), dtype=torch.float32, device=x.device)
    workspace, _ = _workspace(torch, kernels, B, feature_mask, False, workspace, x.device)
    _check(getattr(load_library(), _entry)(
        kernels.handle, x.data_ptr(), B, feature_mask, lam, shift, out.data_ptr(),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(torch, stream)))
    return out


def rocket_transform_noalloc(kernels, x, feature_mask, out, lam=10.0, shift=-3.0, stream=None):
    """rocket_transform into `out` (float32 CUDA, (B, F*K)) with the library's resident workspace:
    nothing is allocated, here or in the library."""
    torch = _torch()
    if not (x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 3):
        raise RocketError(ROCKET_EINVAL, "x must be a contiguous float32 CUDA tensor of shape (B, C, L)")
    B = x.shape[0]
    if x.shape[1] != kernels.C or x.shape[2] != kernels.L:
        raise RocketError(ROCKET_ESHAPE, "x does not match the kernels' (C, L)")
    F = rocket_num_features(feature_mask)
    if not (out.is_cuda and out.dtype == torch.float32 and out.is_contiguous() and tuple(out.shape) == (B, F * kernels.K)):
        raise RocketError(ROCKET_EINVAL, "out must be a contiguous float32 CUDA tensor of shape (B, F*K)")
    _check(load_library().rocket_transform_noalloc(kernels.handle, x.data_ptr(), B, feature_mask, lam, shift,
                                                   out.data_ptr(), _stream_ptr(torch, stream)))
    return out


def rocket_transform_u8(kernels, x_u8, feature_mask, lam=10.0, shift=-3.0, out=None, workspace=None, stream=None):
    """x_u8: uint8 CUDA tensor (B, C, L), contiguous; rows are z-normalised inside the call."""
    return rocket_transform(kernels, x_u8, feature_mask, lam, shift, out, workspace, stream,
                            _dtype="uint8", _entry="rocket_transform_u8")


def rocket_soft_ppv_backward(kernels, x, feature_mask, grad_out, lam=10.0, shift=-3.0, include_max=False,
                             grad_w=None, grad_b=None, workspace=None, stream=None,
                             _dtype="float32", _entry="rocket_soft_ppv_backward"):
    """Returns (grad_w [total_weights], grad_b [K]) as float32 CUDA tensors."""
    torch = _torch()
    for t, name, dt in ((x, "x", _dtype), (grad_out, "grad_out", "float32")):
        if not (t.is_cuda and t.dtype == getattr(torch, dt) and t.is_contiguous()):
            raise RocketError(ROCKET_EINVAL, "%s must be a contiguous %s CUDA tensor" % (name, dt))
    v = kernels
    B = x.shape[0]
    if x.dim() != 3 or x.shape[1] != v.C or x.shape[2] != v.L:
        raise RocketError(ROCKET_ESHAPE, "x does not match the kernels' (C, L)")
    F = rocket_num_features(feature_mask)
    if tuple(grad_out.shape) != (B, F * v.K):
        raise RocketError(ROCKET_ESHAPE, "grad_out must be (B, F*K)")
    if grad_w is None:
        grad_w = torch.empty(v.total_weights, dtype=torch.float32, device=x.device)
    if grad_b is None:
        grad_b = torch.empty(v.K, dtype=torch.float32, device=x.device)
    workspace, _ = _workspace(torch, kernels, B, feature_mask, True, workspace, x.device)
    _check(getattr(load_library(), _entry)(
        kernels.handle, x.data_ptr(), B, feature_mask, grad_out.data_ptr(), lam, shift, int(bool(include_max)),
        grad_w.data_ptr(), grad_b.data_ptr(), workspace.data_ptr(),
        workspace.numel() * workspace.element_size(), _stream_ptr(torch, stream)))
    return grad_w, grad_b


def rocket_soft_ppv_backward_u8(kernels, x_u8, feature_mask, grad_out, lam=10.0, shift=-3.0, include_max=False,
                                grad_w=None, grad_b=None, workspace=None, stream=None):
    """The backward pass on uint8 samples, z-normalised inside the call."""
    return rocket_soft_ppv_backward(kernels, x_u8, feature_mask, grad_out, lam, shift, include_max,
                                    grad_w, grad_b, workspace, stream,
                                    _dtype="uint8", _entry="rocket_soft_ppv_backward_u8")


def rocket_calibrate_fma(stream=None):
    """Measured plain-FMA rate of the current device in TFLOP/s."""
    torch = _torch()
    v = C.c_double()
    _check(load_library().rocket_calibrate_fma(C.byref(v), _stream_ptr(torch, stream)))
    return v.value


CAL_NAMES = ("load_b32_l1_GBps", "load_b32_l2_GBps", "load_b128_l1_GBps", "load_b128_l2_GBps",
             "load_b128_to_lds_GBps", "lds_read_b32_GBps", "mfma_f32_4x4x1_TFLOPs", "mfma_valu_serial_ratio",
             "conv_strip_valu_TFLOPs", "conv_strip_mfma_toeplitz_TFLOPs")


def rocket_calibrate_units(stream=None):
    """Measured rates of the load, LDS and matrix units of the current device, keyed by CAL_NAMES."""
    torch = _torch()
    v = (C.c_double * len(CAL_NAMES))()
    _check(load_library().rocket_calibrate_units(v, len(CAL_NAMES), _stream_ptr(torch, stream)))
    return dict(zip(CAL_NAMES, list(v)))


def rocket_ridge_workspace_bytes(n, p):
    return int(load_library().rocket_ridge_workspace_bytes(n, p))


def rocket_ridge_fit(features, targets, alpha, workspace=None, stream=None):
    """features: float32 CUDA (n, p); targets: float32 CUDA (n).  Returns (coef [p], intercept [1]) float64 CUDA."""
    torch = _torch()
    if not (features.is_cuda and features.dtype == torch.float32 and features.is_contiguous() and features.dim() == 2):
        raise RocketError(ROCKET_EINVAL, "features must be a contiguous float32 CUDA tensor (n, p)")
    n, p = features.shape
    if not (targets.is_cuda and targets.dtype == torch.float32 and targets.is_contiguous() and tuple(targets.shape) == (n,)):
        raise RocketError(ROCKET_EINVAL, "targets must be a contiguous float32 CUDA tensor (n,)")
    coef = torch.empty(p, dtype=torch.float64, device=features.device)
    intercept = torch.empty(1, dtype=torch.float64, device=features.device)
    if workspace is None:
        workspace = torch.empty(rocket_ridge_workspace_bytes(n, p), dtype=torch.uint8, device=features.device)
    _check(load_library().rocket_ridge_fit(features.data_ptr(), targets.data_ptr(), n, p, float(alpha), coef.data_ptr(),
                                           intercept.data_ptr(), workspace.data_ptr(),
                                           workspace.numel(), _stream_ptr(torch, stream)))
    return coef, intercept


def rocket_ridge_predict(features, coef, intercept, stream=None):
    """Returns float64 CUDA predictions (m,) for float32 CUDA features (m, p)."""
    torch = _torch()
    if not (features.is_cuda and features.dtype == torch.float32 and features.is_contiguous() and features.dim() == 2):
        raise RocketError(ROCKET_EINVAL, "features must be a contiguous float32 CUDA tensor (m, p)")
    m, p = features.shape
    if not (coef.is_cuda and coef.dtype == torch.float64 and coef.numel() == p and intercept.dtype == torch.float64):
        raise RocketError(ROCKET_EINVAL, "coef must be float64 CUDA of length p, intercept float64")
    pred = torch.empty(m, dtype=torch.float64, device=features.device)
    _check(load_library().rocket_ridge_predict(features.data_ptr(), m, p, coef.data_ptr(), intercept.data_ptr(),
                                               pred.data_ptr(), _stream_ptr(torch, stream)))
    return pred


def rocket_infer(kernels, x, feature_mask, coef, intercept, lam=10.0, shift=-3.0, features=None, workspace=None,
                 stream=None):
    """x: float32 or uint8 CUDA tensor (B, C, L).  Returns (pred float64 (B,), features float32 (B, F*K))."""
    torch = _torch()
    if not (x.is_cuda and x.dtype in (torch.float32, torch.uint8) and x.is_contiguous() and x.dim() == 3):
        raise RocketError(ROCKET_EINVAL, "x must be a contiguous float32 or uint8 CUDA tensor of shape (B, C, L)")
    v = kernels
    B = x.shape[0]
    if x.shape[1] != v.C or x.shape[2] != v.L:
        raise RocketError(ROCKET_ESHAPE, "x does not match the kernels' (C, L)")
    p = rocket_num_features(feature_mask) * v.K
    if not (coef.is_cuda and coef.dtype == torch.float64 and coef.numel() == p and coef.is_contiguous()
            and intercept.is_cuda and intercept.dtype == torch.float64 and intercept.numel() == 1):
        raise RocketError(ROCKET_EINVAL, "coef must be float64 CUDA of length F*K, intercept float64 CUDA of length 1")
    if features is None:
        features = torch.empty((B, max(p, 1)), dtype=torch.float32, device=x.device)
    pred = torch.empty(B, dtype=torch.float64, device=x.device)
    workspace, _ = _workspace(torch, kernels, B, feature_mask, False, workspace, x.device)
    _check(load_library().rocket_infer(
        kernels.handle, x.data_ptr(), int(x.dtype == torch.uint8), B, feature_mask, lam, shift,
        coef.data_ptr(), intercept.data_ptr(), features.data_ptr(), pred.data_ptr(),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(torch, stream)))
    return pred, features


def rocket_mse_grad(pred, targets, coef, grad_out=None, stream=None):
    """pred float64 (B,), targets float32 (B,), coef float64 (p,), all CUDA.
    Returns (grad_out float32 (B, p), loss float64 (1,))."""
    torch = _torch()
    B, p = pred.numel(), coef.numel()
    if not (pred.is_cuda and pred.dtype == torch.float64 and targets.is_cuda and targets.dtype == torch.float32
            and targets.numel() == B and coef.is_cuda and coef.dtype == torch.float64
            and pred.is_contiguous() and targets.is_contiguous() and coef.is_contiguous()):
        raise RocketError(ROCKET_EINVAL, "pred float64 (B,), targets float32 (B,), coef float64 (p,) CUDA tensors expected")
    if grad_out is None:
        grad_out = torch.empty((B, p), dtype=torch.float32, device=pred.device)
    loss = torch.empty(1, dtype=torch.float64, device=pred.device)
    _check(load_library().rocket_mse_grad(pred.data_ptr(), targets.data_ptr(), coef.data_ptr(), B, p,
                                          grad_out.data_ptr(), loss.data_ptr(), _stream_ptr(torch, stream)))
    return grad_out, loss


def rocket_sgd_update(kernels, grad_w, grad_b, lr, recentre=False, stream=None):
    torch = _torch()
    v = kernels
    for t, n, name in ((grad_w, v.total_weights, "grad_w"), (grad_b, v.K, "grad_b")):
        if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous() and t.numel() == n):
            raise RocketError(ROCKET_EINVAL, "%s must be a contiguous float32 CUDA tensor of %d elements" % (name, n))
    _check(load_library().rocket_sgd_update(kernels.handle, grad_w.data_ptr(), grad_b.data_ptr(), lr,
                                            int(bool(recentre)), _stream_ptr(torch, stream)))


def rocket_train_workspace_bytes(kernels, B, feature_mask):
    return int(load_library().rocket_train_workspace_bytes(kernels.handle, B, feature_mask))


def rocket_train_step(kernels, x, feature_mask, coef, intercept, targets, lr, lam=10.0, shift=-3.0, recentre=False,
                      workspace=None, stream=None):
    """One gradient-descent step on the kernels' weights and biases.  Returns the loss before
    the update as a float64 CUDA tensor of one element."""
    torch = _torch()
    if not (x.is_cuda and x.dtype in (torch.float32, torch.uint8) and x.is_contiguous() and x.dim() == 3):
        raise RocketError(ROCKET_EINVAL, "x must be a contiguous float32 or uint8 CUDA tensor of shape (B, C, L)")
    v = kernels
    B = x.shape[0]
    if x.shape[1] != v.C or x.shape[2] != v.L:
        raise RocketError(ROCKET_ESHAPE, "x does not match the kernels' (C, L)")
    p = rocket_num_features(feature_mask) * v.K
    if not (coef.is_cuda and coef.dtype == torch.float64 and coef.numel() == p and coef.is_contiguous()
            and intercept.is_cuda and intercept.dtype == torch.float64 and intercept.numel() == 1
            and targets.is_cuda and targets.dtype == torch.float32 and targets.numel() == B
            and targets.is_contiguous()):
        raise RocketError(ROCKET_EINVAL, "coef float64 (F*K,), intercept float64 (1,), targets float32 (B,) CUDA expected")
    if workspace is None:
        workspace = torch.empty(rocket_train_workspace_bytes(kernels, B, feature_mask), dtype=torch.uint8,
                                device=x.device)
    loss = torch.empty(1, dtype=torch.float64, device=x.device)
    _check(load_library().rocket_train_step(
        kernels.handle, x.data_ptr(), int(x.dtype == torch.uint8), B, feature_mask, lam, shift,
        coef.data_ptr(), intercept.data_ptr(), targets.data_ptr(), lr, int(bool(recentre)), loss.data_ptr(),
        workspace.data_ptr(), workspace.numel() * workspace.element_size(), _stream_ptr(torch, stream)))
    return loss


def rocket_kernels_subset(kernels, index):
    idx = np.ascontiguousarray(index, dtype=np.int32)
    out = C.c_void_p()
    _check(load_library().rocket_kernels_subset(kernels.handle, idx.ctypes.data_as(C.c_void_p), len(idx),
                                                C.byref(out)))
    return Kernels(out.value)


def rocket_minirocket_kernels(seed, groups, C_, L):
    out = C.c_void_p()
    _check(load_library().rocket_minirocket_kernels(seed, groups, C_, L, C.byref(out)))
    return Kernels(out.value)


def rocket_minirocket_fit_workspace_bytes(kernels, B):
    return int(load_library().rocket_minirocket_fit_workspace_bytes(kernels.handle, B))


def rocket_minirocket_fit_bias(kernels, x, seed, workspace=None, stream=None):
    """x: float32 CUDA tensor (B, C, L) of training series; sets the kernels' biases from it."""
    torch = _torch()
    if not (x.is_cuda and x.dtype == torch.float32 and x.is_contiguous() and x.dim() == 3):
        raise RocketError(ROCKET_EINVAL, "x must be a contiguous float32 CUDA tensor of shape (B, C, L)")
    if x.shape[1] != kernels.C or x.shape[2] != kernels.L:
        raise RocketError(ROCKET_ESHAPE, "x does not match the kernels' (C, L)")
    B = x.shape[0]
    if workspace is None:
        workspace = torch.empty(rocket_minirocket_fit_workspace_bytes(kernels, B), dtype=torch.uint8, device=x.device)
    _check(load_library().rocket_minirocket_fit_bias(kernels.handle, x.data_ptr(), B, seed, workspace.data_ptr(),
                                                     workspace.numel() * workspace.element_size(),
                                                     _stream_ptr(torch, stream)))


def rocket_minirocket_workspace_bytes(kernels, B):
    return int(load_library().rocket_minirocket_workspace_bytes(kernels.handle, B))


def rocket_minirocket_jobs_view_get(kernels):
    """(count, 8) int32 array (a copy): group, mode, first, count, col0, width, rows, 0 of every work item."""
    n = C.c_int32()
    p = C.POINTER(C.c_int32)()
    _check(load_library().rocket_minirocket_jobs_view_get(kernels.handle, C.byref(n), C.byref(p)))
    return np.ctypeslib.as_array(p, shape=(n.value, 8)).copy()


def rocket_minirocket_transform(kernels, x, out=None, workspace=None, stream=None, _dtype="float32",
                                _entry="rocket_minirocket_transform"):
    """x: float32 CUDA tensor (B, C, L); returns the (B, K) float32 PPV features of a MINIROCKET-style handle."""
    torch = _torch()
    if not (x.is_cuda and x.dtype == getattr(torch, _dtype) and x.is_contiguous() and x.dim() == 3):
        raise RocketError(ROCKET_EINVAL, "x must be a contiguous %s CUDA tensor of shape (B, C, L)" % _dtype)
    if x.shape[1] != kernels.C or x.shape[2] != kernels.L:
        raise RocketError(ROCKET_ESHAPE, "x does not match the kernels' (C, L)")
    B = x.shape[0]
    if out is None:
        out = torch.empty((B, kernels.K), dtype=torch.float32, device=x.device)
    if workspace is None:
        workspace = torch.empty(max(256, rocket_minirocket_workspace_bytes(kernels, B)), dtype=torch.uint8, device=x.device)
    _check(getattr(load_library(), _entry)(kernels.handle, x.data_ptr(), B, out.data_ptr(), workspace.data_ptr(),
                                           workspace.numel() * workspace.element_size(), _stream_ptr(torch, stream)))
    return out


def rocket_minirocket_transform_u8(kernels, x_u8, out=None, workspace=None, stream=None):
    """x_u8: uint8 CUDA tensor (B, C, L), contiguous; rows are z-normalised inside the call."""
    return rocket_minirocket_transform(kernels, x_u8, out, workspace, stream, _dtype="uint8",
                                       _entry="rocket_minirocket_transform_u8")


def rocket_free_kernels(kernels):
    kernels.free()
