"""3x3 convolution, stride 1, zero pad 1, as the paper's dot-product category
(oracle; test infrastructure only).

Paper Sec. 3.3 / Sec. 4: convolutions are FP16 dot products accumulated wide and
rounded to FP16 on store, in forward, backward-activation and backward-weight.

Layouts: x[Nb,H,W,C] (NHWC), w[Kf,3,3,C] (KRSC), y and dy [Nb,H,W,Kf].
Cross-correlation (no filter flip):
  y [n,p,q,k] = rne16( sum_{r,s,c} x[n,p+r-1,q+s-1,c] * w[k,r,s,c] )
  dx[n,h,v,c] = rne16( sum_{r,s,k} dy[n,h-r+1,v-s+1,k] * w[k,r,s,c] )
  dw[k,r,s,c] = rne16( sum_{n,p,q} dy[n,p,q,k] * x[n,p+r-1,q+s-1,c] )
with out-of-image terms equal to zero.  Sums are taken in FP64, one rounding.
"""
import numpy as np
from .fp16 import rne16, to_f64


def _pad(a):
    return np.pad(a, ((0, 0), (1, 1), (1, 1), (0, 0)))


def conv3x3_fwd(x16, w16, full=False):
    x, w = to_f64(x16), to_f64(w16)
    Nb, H, W, C = x.shape
    Kf = w.shape[0]
    assert w.shape == (Kf, 3, 3, C)
    xp, ap = _pad(x), _pad(np.abs(x))
    y = np.zeros((Nb, H, W, Kf))
    sabs = np.zeros((Nb, H, W, Kf))
    for r in range(3):
        for s in range(3):
            y += xp[:, r:r + H, s:s + W, :] @ w[:, r, s, :].T
            sabs += ap[:, r:r + H, s:s + W, :] @ np.abs(w[:, r, s, :]).T
    return (rne16(y), sabs, y) if full else (rne16(y), sabs)


def conv3x3_dgrad(dy16, w16, full=False):
    dy, w = to_f64(dy16), to_f64(w16)
    Nb, H, W, Kf = dy.shape
    C = w.shape[3]
    assert w.shape == (Kf, 3, 3, C)
    dp, ap = _pad(dy), _pad(np.abs(dy))
    dx = np.zeros((Nb, H, W, C))
    sabs = np.zeros((Nb, H, W, C))
    for r in range(3):
        for s in range(3):
            # dy index h-r+1 in padded coordinates is h + (2-r)
            dx += dp[:, 2 - r:2 - r + H, 2 - s:2 - s + W, :] @ w[:, r, s, :]
            sabs += ap[:, 2 - r:2 - r + H, 2 - s:2 - s + W, :] @ np.abs(w[:, r, s, :])
    return (rne16(dx), sabs, dx) if full else (rne16(dx), sabs)


def conv3x3_wgrad(x16, dy16, full=False):
    x, dy = to_f64(x16), to_f64(dy16)
    Nb, H, W, C = x.shape
    Kf = dy.shape[3]
    assert dy.shape == (Nb, H, W, Kf)
    xp, ap = _pad(x), _pad(np.abs(x))
    dw = np.zeros((Kf, 3, 3, C))
    sabs = np.zeros((Kf, 3, 3, C))
    d2, a2 = dy.reshape(-1, Kf), np.abs(dy).reshape(-1, Kf)
    for r in range(3):
        for s in range(3):
            dw[:, r, s, :] = d2.T @ xp[:, r:r + H, s:s + W, :].reshape(-1, C)
            sabs[:, r, s, :] = a2.T @ ap[:, r:r + H, s:s + W, :].reshape(-1, C)
    return (rne16(dw), sabs, dw) if full else (rne16(dw), sabs)


# ---- explicit-loop definitions (tiny inputs only) ----

def conv3x3_fwd_loops(x16, w16):
    x, w = to_f64(x16), to_f64(w16)
    Nb, H, W, C = x.shape
    Kf = w.shape[0]
    y = np.zeros((Nb, H, W, Kf))
    for n in range(Nb):
        for p in range(H):
            for q in range(W):
                for k in range(Kf):
                    acc = 0.0
                    for r in range(3):
                        for s in range(3):
                            hh, ww = p + r - 1, q + s - 1
                            if 0 <= hh < H and 0 <= ww < W:
                                for c in range(C):
                                    acc += x[n, hh, ww, c] * w[k, r, s, c]
                    y[n, p, q, k] = acc
    return rne16(y)


def conv3x3_dgrad_loops(dy16, w16):
    dy, w = to_f64(dy16), to_f64(w16)
    Nb, H, W, Kf = dy.shape
    C = w.shape[3]
    dx = np.zeros((Nb, H, W, C))
    for n in range(Nb):
        for h in range(H):
            for v in range(W):
                for c in range(C):
                    acc = 0.0
                    for r in range(3):
                        for s in range(3):
                            p, q = h - r + 1, v - s + 1
                            if 0 <= p < H and 0 <= q < W:
                                for k in range(Kf):
                                    acc += dy[n, p, q, k] * w[k, r, s, c]
                    dx[n, h, v, c] = acc
    return rne16(dx)


def conv3x3_wgrad_loops(x16, dy16):
    x, dy = to_f64(x16), to_f64(dy16)
    Nb, H, W, C = x.shape
    Kf = dy.shape[3]
    dw = np.zeros((Kf, 3, 3, C))
    for k in range(Kf):
        for r in range(3):
            for s in range(3):
                for c in range(C):
                    acc = 0.0
                    for n in range(Nb):
                        for p in range(H):
                            for q in range(W):
                                hh, ww = p + r - 1, q + s - 1
                                if 0 <= hh < H and 0 <= ww < W:
                                    acc += dy[n, p, q, k] * x[n, hh, ww, c]
                    dw[k, r, s, c] = acc
    return rne16(dw)
