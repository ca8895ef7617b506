"""Training step through softPPV -- oracle side.  The paper makes the pooling differentiable
(section 3.2, Eq. 3-4) so that the kernel weights can be trained, and names that training as
future work (section 6).  The step here is the plainest instance of it: the features feed a fixed
linear head (the ridge regressor of section 3.3), the loss is the mean squared error of its
predictions, and (weights, biases) move one gradient-descent step.

TEST INFRASTRUCTURE ONLY: part of the CPU oracle; shares no code with the library.

    F        = features(x; w, b)                       B x (planes*K), fp64
    pred_b   = intercept + sum_i F[b,i] coef[i]
    loss     = (1/B) sum_b (pred_b - y_b)^2
    G[b,i]   = dloss/dF[b,i] = (2/B) (pred_b - y_b) coef[i]
    (gw, gb) = backward(x, G)                          max plane at its first arg-max, PPV plane zero
    w <- w - lr*gw,  b <- b - lr*gb                    then, optionally, every (kernel, channel) row
                                                       of w is re-centred (the sampler's invariant)
Parameters are stored in float32: the update is computed in fp64 and rounded once.
"""
import numpy as np

from . import rocket_oracle as _ro


def feature_matrix(o, mask):
    """(B, planes*K) fp64 matrix from a transform() result over all kernels, planes in bit order."""
    cols = []
    if mask & 1:
        cols.append(o["max"])
    if mask & 2:
        cols.append(o["ppv"])
    if mask & 4:
        cols.append(o["softppv"])
    return np.concatenate(cols, axis=1)


def mse_loss_grad(F, y, coef, intercept):
    """loss and dloss/dF of the linear head's mean squared error."""
    F = np.asarray(F, np.float64)
    y = np.asarray(y, np.float64)
    coef = np.asarray(coef, np.float64)
    r = F @ coef + float(intercept) - y
    return float(np.mean(r * r)), (2.0 / len(y)) * r[:, None] * coef[None, :]


def sgd_update(kr, gw, gb, lr, recentre=False):
    """Returns (weights, bias) float32 after one descent step."""
    w = np.asarray(kr["weights"], np.float64) - float(lr) * np.asarray(gw, np.float64)
    b = np.asarray(kr["bias"], np.float64) - float(lr) * np.asarray(gb, np.float64)
    if recentre:
        for k in range(len(kr["length"])):
            ln, lo = int(kr["length"][k]), int(kr["w_off"][k])
            for c in range(int(kr["n_ch"][k])):
                row = w[lo + c * ln: lo + (c + 1) * ln]
                row -= row.mean()
    return w.astype(np.float32), b.astype(np.float32)


def loss_of(x, kr, mask, y, coef, intercept, lam=10.0, shift=-3.0):
    o = _ro.transform(x, kr, lam=lam, shift=shift)
    return mse_loss_grad(feature_matrix(o, mask), y, coef, intercept)[0]


def train_step(x, kr, mask, y, coef, intercept, lr, lam=10.0, shift=-3.0, recentre=False):
    """One step.  Returns dict(loss, grad_w, grad_b, weights, bias); loss is the one before the update."""
    if not mask & 4:
        raise ValueError("the feature mask must contain softPPV")
    K = len(kr["length"])
    o = _ro.transform(x, kr, lam=lam, shift=shift)
    loss, G = mse_loss_grad(feature_matrix(o, mask), y, coef, intercept)
    planes = G.shape[1] // K
    g_soft = G[:, (planes - 1) * K:]
    g_max = G[:, :K] if mask & 1 else None
    gw, gb = _ro.backward(x, kr, g_soft, g_max, lam=lam, shift=shift)
    w, b = sgd_update(kr, gw, gb, lr, recentre)
    return {"loss": loss, "grad_w": gw, "grad_b": gb, "weights": w, "bias": b}
