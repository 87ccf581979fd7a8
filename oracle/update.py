"""Loss-scaled gradient path into the FP32 master weights (oracle; test
infrastructure only).

Paper Sec. 3.2: weight gradients carry the loss-scale factor S and are unscaled
before the weight update; an overflow shows up as Inf/NaN in the weight
gradients and the update is then skipped.  Sec. 3.1: the FP32 master copy is
updated with the weight gradient and rounded to FP16 for the next iteration.

Readings taken (the paper prints no update formula and no optimizer-state
precision): heavy-ball SGD with an FP32 momentum buffer, no dampening, no
weight decay; overflow is tested on the stored gradient (exponent field all
ones), which is equivalent to testing the unscaled value for finite 1/S; a
skipped step leaves master, momentum and FP16 copy bit-identical (momentum is
not decayed).  Every arithmetic step is one individually rounded IEEE FP32
operation, never fused:
    g  = float(grad) (*) inv_S
    m' = (mu (*) m) (+) g         (momentum buffer present)
    w' = w (-) (lr (*) m')        (or lr (*) g without momentum)
    w16' = rne16(w')
"""
import numpy as np
from .fp16 import rne16, to_f64, bits, is_special_bits

F32 = np.float32


def _grad_f32(grad):
    grad = np.asarray(grad)
    if grad.dtype == np.float16:
        return to_f64(grad).astype(F32)          # exact widening
    assert grad.dtype == np.float32, grad.dtype
    return grad


def overflow_flag(grad):
    """1 if any stored gradient is Inf or NaN, else 0 (FP16 or FP32 storage)."""
    grad = np.asarray(grad)
    if grad.dtype == np.float16:
        return int(is_special_bits(bits(grad)).any())
    u = grad.astype(F32, copy=False).view(np.uint32)
    return int(((u & 0x7F800000) == 0x7F800000).any())


def unscale_check(grad, inv_scale):
    """Returns (g32, flag): g32 = float(grad) (*) inv_S in FP32; flag as above."""
    g = _grad_f32(grad)
    with np.errstate(all="ignore"):
        g32 = g * F32(inv_scale)
    assert g32.dtype == np.float32
    return g32, overflow_flag(grad)


def master_update(w32, m32, grad, inv_scale, lr, momentum, flag, w16=None):
    """One optimizer step.  Returns (w32', m32' or None, w16').

    flag != 0: skip; outputs are the inputs (w16 unchanged when given, else the
    rounding of the unchanged master).
    """
    w32 = np.asarray(w32, dtype=F32)
    if flag:
        keep16 = w16.copy() if w16 is not None else rne16(w32.astype(np.float64))
        return w32.copy(), (None if m32 is None else np.asarray(m32, F32).copy()), keep16
    with np.errstate(all="ignore"):
        g = _grad_f32(grad) * F32(inv_scale)
        if m32 is not None:
            t1 = F32(momentum) * np.asarray(m32, dtype=F32)
            m_new = t1 + g
            t2 = F32(lr) * m_new
        else:
            m_new = None
            t2 = F32(lr) * g
        w_new = w32 - t2
    assert w_new.dtype == np.float32 and t2.dtype == np.float32
    return w_new, m_new, rne16(w_new.astype(np.float64))


def master_update_fused(w32, m32, grad, inv_scale, lr, momentum):
    """The same step as one pass over the gradient (Sec. 3.2: the overflow test and the update are two uses of
    one read).  A skipped step must leave the state untouched, yet whether to skip is only known once every gradient
    has been seen; so the pass writes its results to a second set of buffers and reports the flag, and the caller adopts
    the second set only if the flag is clear.  Returns (flag, w32', m32' or None, w16'): the flag of overflow_flag on
    this gradient and the outputs of master_update computed as if the step were taken.  With the flag set the outputs
    are not to be used (they hold the arithmetic on Inf / NaN)."""
    w, m, h = master_update(w32, m32, grad, inv_scale, lr, momentum, 0)
    return overflow_flag(grad), w, m, h


def master_update_wide(w32, m32, grad, inv_scale, lr, momentum):
    """Information only: the same step with FP64 intermediates and one FP32
    rounding per stored value.  A per-step result of master_update lies within
    1 FP32 ulp of this, barring cancellation in w - lr*m'."""
    g = _grad_f32(grad).astype(np.float64) * float(F32(inv_scale))
    if m32 is not None:
        m_new = (float(F32(momentum)) * np.asarray(m32, F32).astype(np.float64) + g).astype(F32)
        step = float(F32(lr)) * m_new.astype(np.float64)
    else:
        m_new = None
        step = float(F32(lr)) * g
    w_new = (np.asarray(w32, F32).astype(np.float64) - step).astype(F32)
    return w_new, m_new


def fp16_only_update(w16, grad16, lr):
    """The thing Sec. 3.1 warns against: weights kept and updated in FP16, each
    operation rounded to FP16.  Used only to pin the two failure modes."""
    upd = rne16(to_f64(grad16) * float(lr))
    return rne16(to_f64(w16) - to_f64(upd))
