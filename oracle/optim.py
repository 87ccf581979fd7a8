"""Other master-weight optimizers in the same loss-scaled pass (oracle; test
infrastructure only).

Paper Sec. 4 trains with momentum SGD (classification, detection), Nesterov SGD
(speech), Adagrad (language model) and Adam (GAN); Sec. 3.1 keeps the weights,
and with them the optimizer state, in FP32 and rounds the updated master to
FP16 for the next iteration; Sec. 3.2 unscales the weight gradient before
anything else touches it (clipping, weight decay), so no hyper-parameter changes
with S, and skips the step on overflow.  The paper prints none of the update
rules; the customary forms are taken, each as a fixed sequence of individually
rounded FP32 operations (no fused multiply-add), (*) (+) (-) (/) sqrt below:

    g = float(grad) (*) inv_S                      [then, if clipping:  g = g (*) factor   (oracle/clip.py)]
                                                   [then, if weight_decay != 0:  g = g (+) (wd (*) w)]
  momentum:  m' = (mu (*) m) (+) g                 w' = w (-) (lr (*) m')
  nesterov:  m' = (mu (*) m) (+) g                 w' = w (-) (lr (*) (g (+) (mu (*) m')))
  adagrad:   h' = h (+) (g (*) g)                  w' = w (-) ((lr (*) g) (/) (sqrt(h') (+) eps))
  adam:      m' = (b1 (*) m) (+) (omb1 (*) g)      v' = (b2 (*) v) (+) (omb2 (*) (g (*) g))
             mh = m' (/) bc1     vh = v' (/) bc2    w' = w (-) ((lr (*) mh) (/) (sqrt(vh) (+) eps))
    w16' = rne16(w')

omb1, omb2 (1 - beta) and bc1, bc2 (1 - beta^t at this step) are inputs, rounded
to FP32 by the caller.  A skipped step (flag != 0) leaves every buffer
bit-identical: optimizer state does not advance.
"""
from dataclasses import dataclass

import numpy as np

from .fp16 import rne16
from .update import _grad_f32

F = np.float32
KINDS = ("momentum", "nesterov", "adagrad", "adam")


@dataclass
class OptParams:
    lr: float
    momentum: float = 0.0          # mu, or beta1 for adam
    beta2: float = 0.0
    eps: float = 0.0
    weight_decay: float = 0.0
    one_minus_beta1: float = 0.0
    one_minus_beta2: float = 0.0
    bias_corr1: float = 1.0
    bias_corr2: float = 1.0


def adam_params(lr, beta1, beta2, eps, step, weight_decay=0.0):
    """Adam's derived constants for 1-based step number `step`, formed in FP64 and rounded once."""
    return OptParams(lr=lr, momentum=beta1, beta2=beta2, eps=eps, weight_decay=weight_decay,
                     one_minus_beta1=float(F(1.0 - beta1)), one_minus_beta2=float(F(1.0 - beta2)),
                     bias_corr1=float(F(1.0 - beta1 ** step)), bias_corr2=float(F(1.0 - beta2 ** step)))


def optimizer_update(kind, w32, s1, s2, grad, inv_scale, p, flag, w16=None, clip=None):
    """One step.  s1: momentum / Adagrad sum / Adam first moment; s2: Adam second moment (else None).
    clip: None, or the FP32 factor of clip-by-global-norm (oracle/clip.py), applied to the unscaled gradient with
    one FP32 multiplication before weight decay.  Returns (w32', s1', s2', w16')."""
    assert kind in KINDS
    w = np.asarray(w32, dtype=F)
    a = np.asarray(s1, dtype=F)
    b = None if s2 is None else np.asarray(s2, dtype=F)
    if flag:
        keep16 = w16.copy() if w16 is not None else rne16(w.astype(np.float64))
        return w.copy(), a.copy(), (None if b is None else b.copy()), keep16
    lr, mu = F(p.lr), F(p.momentum)
    with np.errstate(all="ignore"):
        g = _grad_f32(grad) * F(inv_scale)
        if clip is not None:
            g = g * F(clip)
        if p.weight_decay != 0.0:
            g = g + F(p.weight_decay) * w
        if kind == "momentum":
            a2 = mu * a + g
            w2 = w - lr * a2
            b2 = b
        elif kind == "nesterov":
            a2 = mu * a + g
            w2 = w - lr * (g + mu * a2)
            b2 = b
        elif kind == "adagrad":
            a2 = a + g * g
            w2 = w - (lr * g) / (np.sqrt(a2) + F(p.eps))
            b2 = b
        else:
            a2 = mu * a + F(p.one_minus_beta1) * g
            b2 = F(p.beta2) * b + F(p.one_minus_beta2) * (g * g)
            mh = a2 / F(p.bias_corr1)
            vh = b2 / F(p.bias_corr2)
            w2 = w - (lr * mh) / (np.sqrt(vh) + F(p.eps))
    assert w2.dtype == np.float32 and a2.dtype == np.float32
    return w2, a2, b2, rne16(w2.astype(np.float64))


def optimizer_update_wide(kind, w32, s1, s2, grad, inv_scale, p):
    """Information only: the same formulas with FP64 intermediates, nothing rounded."""
    w = np.asarray(w32, dtype=np.float64)
    a = np.asarray(s1, dtype=np.float64)
    g = _grad_f32(grad).astype(np.float64) * float(F(inv_scale))
    if p.weight_decay != 0.0:
        g = g + float(F(p.weight_decay)) * w
    lr, mu = float(F(p.lr)), float(F(p.momentum))
    if kind == "momentum":
        a2 = mu * a + g
        return w - lr * a2, a2, None
    if kind == "nesterov":
        a2 = mu * a + g
        return w - lr * (g + mu * a2), a2, None
    if kind == "adagrad":
        a2 = a + g * g
        return w - lr * g / (np.sqrt(a2) + float(F(p.eps))), a2, None
    b = np.asarray(s2, dtype=np.float64)
    a2 = mu * a + float(F(p.one_minus_beta1)) * g
    b2 = float(F(p.beta2)) * b + float(F(p.one_minus_beta2)) * g * g
    mh, vh = a2 / float(F(p.bias_corr1)), b2 / float(F(p.bias_corr2))
    return w - lr * mh / (np.sqrt(vh) + float(F(p.eps))), a2, b2
