"""Pointwise and reduction glue of the small MLP step (oracle; test
infrastructure only).

Paper Sec. 3.3: large reductions such as softmax are carried out wide while
reading and writing FP16; pointwise non-linearities may use either precision.
Paper Sec. 3.2: the loss is multiplied by S before back-propagation; by
linearity that is the same as multiplying d(loss)/d(logits) by S, which is
where it is applied here (in wide arithmetic, before the FP16 store).
"""
import numpy as np
from .fp16 import rne16, to_f64


def relu_fwd(y16):
    y = to_f64(y16)
    return rne16(np.where(y > 0, y, 0.0))


def relu_bwd(dh16, y16):
    """dy = dh where the pre-activation was positive, else 0."""
    return rne16(np.where(to_f64(y16) > 0, to_f64(dh16), 0.0))


def softmax_xent_scaled(logits16, labels, scale):
    """Mean softmax cross-entropy over the batch and its scaled gradient.

    Returns (loss float64, dlogits16) with
      p = softmax(logits), loss = mean_b -log p[b, label_b],
      dlogits = rne16( scale * (p - onehot) / B ).
    """
    z = to_f64(logits16)
    B = z.shape[0]
    z = z - z.max(axis=1, keepdims=True)
    ez = np.exp(z)
    den = ez.sum(axis=1, keepdims=True)
    p = ez / den
    idx = np.arange(B)
    loss = float(np.mean(np.log(den[:, 0]) - z[idx, labels]))
    d = p.copy()
    d[idx, labels] -= 1.0
    d = d * (float(scale) / B)
    return loss, rne16(d)
