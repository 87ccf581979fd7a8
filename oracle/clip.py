"""Gradient clipping by global norm on the unscaled gradient (oracle; test infrastructure only).

Paper Sec. 3.2: the weight gradients are unscaled before the weight update so that whatever acts on gradient
magnitudes afterwards (gradient clipping, weight decay) needs no retuning with the loss scale S.  The paper prints
no clipping rule; the customary clip-by-global-norm is taken:

    g_i    = float(grad_i) (*) inv_S                 one FP32 multiplication per element, as in the update
    sumsq  = sum over all buffers, all elements of g_i^2        exact squares, FP64 sum
    norm   = sqrt(sumsq)                                         FP64
    factor = 1                       if norm <= max_norm
             rne32(max_norm / norm)  otherwise                   FP64 division, rounded once to FP32
    the update then uses  g_i (*) factor  (one more FP32 multiplication) in place of g_i, before weight decay.

A gradient holding Inf or NaN makes the step a no-op anyway (Sec. 3.2), so sumsq and factor are then unspecified.
Parity unpinned against the paper (it gives no numbers); pinned by closed forms and torch's clip_grad_norm_.
"""
import numpy as np

from .update import _grad_f32

F = np.float32


def unscaled_sumsq(grads, inv_scale):
    """grads: a buffer or a list of buffers (FP16 or FP32 storage).  FP64 sum of the squares of the unscaled FP32
    gradients (each square is exact in FP64: an FP32 value has 24 significant bits)."""
    if isinstance(grads, np.ndarray):
        grads = [grads]
    total = np.float64(0.0)
    with np.errstate(all="ignore"):
        for g in grads:
            g32 = _grad_f32(g) * F(inv_scale)
            assert g32.dtype == np.float32
            g64 = g32.astype(np.float64).ravel()
            total = total + np.sum(g64 * g64, dtype=np.float64)
    return float(total)


def clip_factor(sumsq, max_norm):
    """Returns (factor as numpy float32, norm as float)."""
    norm = float(np.sqrt(np.float64(sumsq)))
    if not (norm > float(max_norm)):          # also the NaN case: leave the gradient alone, the step is skipped anyway
        return F(1.0), norm
    return F(np.float64(max_norm) / np.float64(norm)), norm


def clip_by_global_norm(grads, inv_scale, max_norm):
    """Returns (clipped unscaled FP32 gradients, factor, norm)."""
    if isinstance(grads, np.ndarray):
        grads = [grads]
    factor, norm = clip_factor(unscaled_sumsq(grads, inv_scale), max_norm)
    with np.errstate(all="ignore"):
        out = [(_grad_f32(g) * F(inv_scale)) * factor for g in grads]
    return out, factor, norm
