"""LSTM cell with projection, FP16 tensors and wide pointwise math (oracle; test infrastructure only).

Paper Sec. 4 (language model, speech, translation) trains recurrent layers whose matrix products follow Sec. 3.3's
dot-product rule (the GEMM oracle) and whose gate non-linearities are the "point-wise" category: either precision
is allowed there; FP32 math on FP16-stored tensors is taken.  The paper prints no cell equations; the customary
LSTM with a linear projection of the hidden state is used, gate order (i, f, g, o) along the 4H axis:

  a   = gx + gr (+ bias)                      gx = x_t W_x (time-batched), gr = r_{t-1} W_r, both stored FP16
  i, f, o = sigmoid(a_i), sigmoid(a_f), sigmoid(a_o);   g = tanh(a_g)
  c_t = f * c_{t-1} + i * g;   h_t = o * tanh(c_t)     (tanh of the unrounded c_t)
  stores: act = rne16(i, f, g, o), c16 = rne16(c_t), h16 = rne16(h_t);   r_t = rne16(h16 W_p) by the GEMM rule

Backward, from the stored FP16 act, c16, c_prev16 and the incoming dh (of h_t) and dc_next (carried from t+1):
  tc = tanh(c16);  dc = dh * o * (1 - tc^2) + dc_next
  da_i = dc * g * i(1-i);  da_f = dc * c_prev * f(1-f);  da_g = dc * i * (1-g^2);  da_o = dh * tc * o(1-o)
  dc_prev = dc * f;        stores: da = rne16(...), dc_prev16 = rne16(dc_prev)
All of it evaluated in FP64 here, rounded once per stored value.
"""
import numpy as np

from .fp16 import rne16, to_f64
from . import gemm


def _sigmoid(a):
    with np.errstate(over="ignore"):
        return 1.0 / (1.0 + np.exp(-a))


def lstm_cell_fwd(gx16, gr16, bias32, c_prev16):
    """gx16, gr16: [B, 4H]; bias32: [4H] or None; c_prev16: [B, H].  Returns (act16 [B,4H], c16, h16)."""
    a = to_f64(gx16) + to_f64(gr16)
    if bias32 is not None:
        a = a + np.asarray(bias32, dtype=np.float32).astype(np.float64)
    H = a.shape[1] // 4
    i, f, o = _sigmoid(a[:, :H]), _sigmoid(a[:, H:2 * H]), _sigmoid(a[:, 3 * H:])
    g = np.tanh(a[:, 2 * H:3 * H])
    c = f * to_f64(c_prev16) + i * g
    h = o * np.tanh(c)
    return rne16(np.concatenate([i, f, g, o], axis=1)), rne16(c), rne16(h)


def lstm_cell_bwd(dh16, dc_next16, act16, c16, c_prev16):
    """Returns (da16 [B,4H], dc_prev16 [B,H])."""
    act = to_f64(act16)
    H = act.shape[1] // 4
    i, f, g, o = act[:, :H], act[:, H:2 * H], act[:, 2 * H:3 * H], act[:, 3 * H:]
    dh = to_f64(dh16)
    tc = np.tanh(to_f64(c16))
    dc = dh * o * (1.0 - tc * tc) + to_f64(dc_next16)
    da = np.concatenate([dc * g * i * (1.0 - i), dc * to_f64(c_prev16) * f * (1.0 - f), dc * i * (1.0 - g * g),
                         dh * tc * o * (1.0 - o)], axis=1)
    return rne16(da), rne16(dc * f)


def lstmp_layer_fwd(x16, Wx16, Wr16, Wp16, bias32, r0_16, c0_16):
    """Free-running layer over T steps.  x16: [T, B, I].  Returns lists per step of (gx, gr, act, c, h, r)."""
    T, B, I = x16.shape
    gx_all, _ = gemm.gemm_fwd(x16.reshape(T * B, I), Wx16)           # time-batched input contraction
    gx_all = gx_all.reshape(T, B, -1)
    r, c = r0_16, c0_16
    out = []
    for t in range(T):
        gr, _ = gemm.gemm_fwd(r, Wr16)
        act, c, h = lstm_cell_fwd(gx_all[t], gr, bias32, c)
        r, _ = gemm.gemm_fwd(h, Wp16)
        out.append(dict(gx=gx_all[t], gr=gr, act=act, c=c, h=h, r=r))
    return out
