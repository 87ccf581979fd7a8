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


def lstmp_layer_bwd(x16, Wx16, Wr16, Wp16, r0_16, c0_16, fwd, dr_ext16, dc_last16=None):
    """Backward pass through time of the free-running layer (the reverse of lstmp_layer_fwd, same stored tensors).

    fwd: the list lstmp_layer_fwd returned.  dr_ext16: [T, B, P], the gradient of the (scaled) loss with respect to
    each projected output r_t as it arrives from the layers above.  dc_last16: gradient with respect to the last
    cell state (None = 0).  Per step, last to first, every stored tensor FP16, every contraction by the GEMM rule:
        dr_t   = rne16(dr_ext_t + dr_rec)            dr_rec: what step t+1 sent back through W_r (0 at the last step)
        dh_t   = dr_t W_p^T                           (activation gradient of the projection)
        da_t, dc_prev = cell backward(dh_t, dc_next, act_t, c_t, c_{t-1})
        dr_rec = da_t W_r^T                           (activation gradient of the recurrent product)
    and over all steps at once (reduction length T*B, one FP16 store each, Sec. 3.3):
        dx = dA W_x^T;   dW_x = x^T dA;   dW_r = r_prev^T dA;   dW_p = h^T dR;   dbias = sum over rows of dA (FP32)
    Returns a dict; "da", "dh", "dr" are lists per step."""
    T, B, I = x16.shape
    P = Wp16.shape[1]
    dr_rec = np.zeros((B, P), dtype=np.float16)
    dc_next = np.zeros_like(c0_16) if dc_last16 is None else dc_last16
    da_l, dh_l, dr_l = [None] * T, [None] * T, [None] * T
    for t in range(T - 1, -1, -1):
        dr = rne16(to_f64(dr_ext16[t]) + to_f64(dr_rec))
        dh, _ = gemm.gemm_dgrad(dr, Wp16)
        c_prev = fwd[t - 1]["c"] if t > 0 else c0_16
        da, dc_next = lstm_cell_bwd(dh, dc_next, fwd[t]["act"], fwd[t]["c"], c_prev)
        dr_rec, _ = gemm.gemm_dgrad(da, Wr16)
        da_l[t], dh_l[t], dr_l[t] = da, dh, dr
    dA = np.concatenate(da_l, axis=0)
    dR = np.concatenate(dr_l, axis=0)
    h_all = np.concatenate([f["h"] for f in fwd], axis=0)
    r_prev = np.concatenate([r0_16] + [f["r"] for f in fwd[:-1]], axis=0)
    dx, _ = gemm.gemm_dgrad(dA, Wx16)
    dWx, _ = gemm.gemm_wgrad(x16.reshape(T * B, I), dA)
    dWr, _ = gemm.gemm_wgrad(r_prev, dA)
    dWp, _ = gemm.gemm_wgrad(h_all, dR)
    dbias = to_f64(dA).sum(axis=0).astype(np.float32)
    return dict(da=da_l, dh=dh_l, dr=dr_l, dx=dx.reshape(T, B, I), dWx=dWx, dWr=dWr, dWp=dWp, dbias=dbias,
                dr0=dr_rec, dc0=dc_next)
