"""Batch normalisation over FP16 tensors with wide statistics (oracle; test
infrastructure only).

Paper Sec. 3.3: large reductions (batch-normalisation statistics, softmax) are
carried out in FP32 while the layer still reads and writes FP16 tensors and does
its arithmetic in FP32.  The paper gives no formulas; the standard training-mode
definition is taken, per channel c over the P rows of x[P, C] (P = all batch and
spatial positions of an NHWC tensor):

  mean_c = (1/P) sum_p x[p,c]            var_c = (1/P) sum_p (x[p,c] - mean_c)^2
  y[p,c] = rne16( gamma_c * (x[p,c] - mean_c) / sqrt(var_c + eps) + beta_c )

and its gradient for an upstream dy[P, C] (possibly loss-scaled; everything below
is linear in dy):

  dbeta_c  = sum_p dy[p,c]
  dgamma_c = sum_p dy[p,c] * xhat[p,c]          xhat = (x - mean_c) / sqrt(var_c + eps)
  dx[p,c]  = rne16( gamma_c / sqrt(var_c + eps) * ( dy - dbeta_c / P - xhat * dgamma_c / P ) )

Reductions are the plain definitions in FP64.  The pointwise parts are a fixed
sequence of individually rounded FP32 operations (no fused multiply-add), written
out below, so that an FP32 implementation fed the same statistics reproduces them
bit for bit.
"""
import numpy as np
from .fp16 import rne16, to_f64

F = np.float32


def bn_stats(x16):
    """FP64 per-channel mean and biased variance of x16[P, C]."""
    x = to_f64(x16)
    mean = x.mean(axis=0)
    var = ((x - mean) ** 2).mean(axis=0)
    return mean, var


def _invstd32(var32, eps):
    with np.errstate(divide="ignore"):
        return F(1.0) / np.sqrt(np.asarray(var32, dtype=F) + F(eps))


def bn_apply(x16, mean32, var32, gamma32, beta32, eps, relu=False):
    """FP32 op by op:  scale = gamma * (1 / sqrt(var + eps));  shift = beta - mean * scale;
    y = rne16(x * scale + shift), product and sum rounded separately; optional max(y, 0)."""
    x = to_f64(x16).astype(F)                       # exact
    scale = np.asarray(gamma32, dtype=F) * _invstd32(var32, eps)
    shift = np.asarray(beta32, dtype=F) - np.asarray(mean32, dtype=F) * scale
    y = x * scale + shift                           # numpy float32: two roundings
    if relu:
        y = np.where(y > 0, y, F(0.0))
    return rne16(y.astype(np.float64))


def bn_bwd_reduce(x16, dy16, mean32, var32, eps):
    """FP64 sums dgamma, dbeta, taking the FP32 mean and 1/sqrt(var + eps) as given."""
    x, dy = to_f64(x16), to_f64(dy16)
    invstd = _invstd32(var32, eps).astype(np.float64)
    xhat = (x - np.asarray(mean32, dtype=np.float64)) * invstd
    return (dy * xhat).sum(axis=0), dy.sum(axis=0)


def bn_bwd_apply(x16, dy16, mean32, var32, gamma32, eps, dgamma32, dbeta32):
    """FP32 op by op:  a = gamma * invstd;  b = dbeta / P;  g = dgamma / P;
    xhat = (x - mean) * invstd;  dx = rne16( a * ((dy - b) - xhat * g) )."""
    x = to_f64(x16).astype(F)
    dy = to_f64(dy16).astype(F)
    P = F(x.shape[0])
    invstd = _invstd32(var32, eps)
    a = np.asarray(gamma32, dtype=F) * invstd
    b = np.asarray(dbeta32, dtype=F) / P
    g = np.asarray(dgamma32, dtype=F) / P
    xhat = (x - np.asarray(mean32, dtype=F)) * invstd
    t = (dy - b) - xhat * g
    return rne16((a * t).astype(np.float64))
