"""Input prologue of the paper's data path -- oracle side (sections 4.1 and 4.3): the raw
examples are 8-bit light intensities (integers 0..255); every sensor channel of every
example is mean-centred and divided by its standard deviation before the transform.

TEST INFRASTRUCTURE ONLY: part of the CPU oracle; shares no code with the library.

Readings: the standard deviation is the population one (divide by L); a channel with zero
variance (a dead or saturated sensor) becomes all zeros; the arithmetic is fp64 and the
result is rounded once to fp32, the transform's input type.
"""
import numpy as np


def znormalize_u8(x_u8):
    """x_u8: uint8 array (..., L).  Returns float32 of the same shape."""
    x = np.asarray(x_u8)
    if x.dtype != np.uint8:
        raise ValueError("expected uint8 intensities")
    v = x.astype(np.float64)
    mean = v.mean(axis=-1, keepdims=True)
    std = np.sqrt(((v - mean) ** 2).mean(axis=-1, keepdims=True))
    z = np.where(std > 0, (v - mean) / np.where(std > 0, std, 1.0), 0.0)
    return z.astype(np.float32)
