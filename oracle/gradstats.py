"""Gradient statistics for choosing a loss scale (oracle; test infrastructure only).

Paper Sec. 3.2: histograms of gradient magnitudes over the exponent axis show how much of the FP16 range is unused
and how many values fall below it (the figures bin log2 of the magnitude); a constant scale can be chosen from the
largest magnitude so that scale * max stays below 65504, the largest FP16 value.

Definitions, on the stored FP16 gradients:
  bin 0            : zeros (+0 and -0)
  bin 1 + (e + 24) : finite non-zero values with floor(log2 |g|) = e, e = -24 .. 15  (subnormals by their leading bit)
  bin 41           : Inf and NaN
  absmax           : the largest finite magnitude (0 if there is none)
  suggested scale  : the largest power of two 2^k with 2^k * absmax <= 65504
"""
import math

import numpy as np

from .fp16 import bits, to_f64

NBINS = 42
FP16_MAX = 65504.0


def exponent_histogram(g16):
    b = bits(np.asarray(g16)).astype(np.int64).reshape(-1)
    mag = b & 0x7FFF
    hist = np.zeros(NBINS, dtype=np.int64)
    special = mag >= 0x7C00
    zero = mag == 0
    hist[0] = int(zero.sum())
    hist[41] = int(special.sum())
    vals = to_f64(np.asarray(g16)).reshape(-1)[~special & ~zero]
    e = np.floor(np.log2(np.abs(vals))).astype(np.int64)      # exact: FP64 log2 of a power-of-two-bounded FP16 value
    assert e.size == 0 or (e.min() >= -24 and e.max() <= 15)
    np.add.at(hist, 1 + e + 24, 1)
    return hist


def absmax(g16):
    v = np.abs(to_f64(np.asarray(g16)).reshape(-1))
    v = v[np.isfinite(v)]
    return float(v.max()) if v.size else 0.0


def suggest_scale_log2(amax):
    """k such that 2^k is the largest power of two with 2^k * amax <= 65504; None when amax is 0."""
    if not (amax > 0.0):
        return None
    k = math.floor(math.log2(FP16_MAX / amax))
    while 2.0 ** k * amax > FP16_MAX:
        k -= 1
    while 2.0 ** (k + 1) * amax <= FP16_MAX:
        k += 1
    return k
