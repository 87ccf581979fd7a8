"""ctypes binding for libmpt.so: argument marshalling only.

Each function has the name of the C entry point it calls (include/mpt.h) and
takes torch CUDA tensors purely as carriers of device pointers; torch's current
stream is passed as the hipStream_t.  Every step of the method runs in the
library's kernels.  A missing library is an error, never a fallback.
"""
import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmpt.so")

OP_FWD, OP_DGRAD, OP_WGRAD = 0, 1, 2

c_i64, c_sz, c_f, c_i, c_vp = ctypes.c_int64, ctypes.c_size_t, ctypes.c_float, ctypes.c_int, ctypes.c_void_p


class MptError(RuntimeError):
    def __init__(self, fn, status, text):
        super().__init__("%s failed: %d (%s)" % (fn, status, text))
        self.status = status


class mpt_scaler(ctypes.Structure):
    _fields_ = [("scale", c_f), ("inv_scale", c_f), ("good_steps", ctypes.c_int32),
                ("growth_interval", ctypes.c_int32), ("growth", c_f), ("backoff", c_f),
                ("min_scale", c_f), ("max_scale", c_f)]


class mpt_opt_params(ctypes.Structure):
    _fields_ = [("lr", c_f), ("momentum", c_f), ("beta2", c_f), ("eps", c_f), ("weight_decay", c_f),
                ("one_minus_beta1", c_f), ("one_minus_beta2", c_f), ("bias_corr1", c_f), ("bias_corr2", c_f),
                ("clip_factor_dev", c_vp)]


class mpt_update_item(ctypes.Structure):
    _fields_ = [("w32_dev", c_vp), ("m32_dev", c_vp), ("grad_dev", c_vp), ("w16_dev", c_vp), ("n", c_sz)]


OPT_KINDS = {"momentum": 0, "nesterov": 1, "adagrad": 2, "adam": 3}

_GEMM = [c_vp, c_i64, c_i64, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_sz]
_CONV = [c_vp, c_i64, c_i64, c_i64, c_i64, c_i64, c_vp, c_vp, c_vp, c_vp, c_sz]
SIGNATURES = {
    "mpt_status_string": (ctypes.c_char_p, [c_i]),
    "mpt_version": (c_i, []),
    "mpt_gemm_workspace_bytes": (c_sz, [c_i, c_i64, c_i64, c_i64]),
    "mpt_gemm_fwd": (c_i, _GEMM),
    "mpt_gemm_dgrad": (c_i, _GEMM),
    "mpt_gemm_fwd_relu": (c_i, _GEMM),
    "mpt_gemm_dgrad_relu": (c_i, [c_vp, c_i64, c_i64, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_sz]),
    "mpt_gemm_wgrad": (c_i, [c_vp, c_i64, c_i64, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_i, c_i, c_vp, c_vp, c_sz]),
    "mpt_gemm_wgrad_static": (c_i, [c_vp, c_i64, c_i64, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_i, c_i, c_vp]),
    "mpt_conv3x3_workspace_bytes": (c_sz, [c_i, c_i64, c_i64, c_i64, c_i64, c_i64]),
    "mpt_conv3x3_fwd": (c_i, _CONV),
    "mpt_conv3x3_dgrad": (c_i, _CONV),
    "mpt_conv3x3_wgrad": (c_i, [c_vp, c_i64, c_i64, c_i64, c_i64, c_i64, c_vp, c_vp, c_vp, c_vp, c_vp, c_sz]),
    "mpt_scaler_init": (c_i, [ctypes.POINTER(mpt_scaler), c_f, ctypes.c_int32]),
    "mpt_loss_scale_update": (c_i, [ctypes.POINTER(mpt_scaler), c_i]),
    "mpt_loss_scale_update_dev": (c_i, [c_vp, c_vp, c_vp]),
    "mpt_unscale_check": (c_i, [c_vp, c_vp, c_i, c_sz, c_f, c_vp, c_vp]),
    "mpt_master_update": (c_i, [c_vp, c_sz, c_vp, c_vp, c_vp, c_i, c_vp, c_f, c_vp, c_f, c_f, c_vp]),
    "mpt_probe_mfma": (c_i, [c_vp, c_i, c_i, c_vp]),
    "mpt_master_update_fused": (c_i, [c_vp, c_sz, c_vp, c_vp, c_vp, c_i, c_vp, c_vp, c_vp, c_f, c_vp, c_f, c_f, c_vp]),
    "mpt_master_update_multi": (c_i, [c_vp, c_i, c_vp, c_i, c_f, c_vp, c_f, c_f, c_vp]),
    "mpt_add_fp16": (c_i, [c_vp, c_sz, c_vp, c_vp, c_vp]),
    "mpt_relu_fwd": (c_i, [c_vp, c_sz, c_vp, c_vp]),
    "mpt_relu_bwd": (c_i, [c_vp, c_sz, c_vp, c_vp, c_vp]),
    "mpt_softmax_xent_scaled": (c_i, [c_vp, c_i64, c_i64, c_vp, c_i64, c_vp, c_f, c_vp, c_vp, c_vp, c_i64]),
    "mpt_optimizer_update": (c_i, [c_vp, c_sz, c_i, c_vp, c_vp, c_vp, c_vp, c_vp, c_i, c_vp, c_f, c_vp, c_vp]),
    "mpt_grad_norm_workspace_bytes": (c_sz, []),
    "mpt_grad_sumsq": (c_i, [c_vp, c_vp, c_i, c_sz, c_f, c_vp, c_i, c_vp, c_vp, c_vp, c_sz]),
    "mpt_clip_factor": (c_i, [c_vp, c_vp, c_f, c_vp, c_vp]),
    "mpt_grad_stats": (c_i, [c_vp, c_vp, c_sz, c_i, c_vp, c_vp]),
    "mpt_suggest_loss_scale_log2": (c_i, [ctypes.c_uint32, c_i]),
    "mpt_lstm_cell_fwd": (c_i, [c_vp, c_i64, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64]),
    "mpt_lstm_cell_bwd": (c_i, [c_vp, c_i64, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_i64]),
    "mpt_bn_workspace_bytes": (c_sz, [c_i64, c_i64]),
    "mpt_bn_stats": (c_i, [c_vp, c_i64, c_i64, c_vp, c_i64, c_vp, c_vp, c_vp, c_sz]),
    "mpt_bn_apply": (c_i, [c_vp, c_i64, c_i64, c_vp, c_i64, c_vp, c_vp, c_vp, c_vp, c_f, c_i, c_vp, c_i64]),
    "mpt_bn_bwd_reduce": (c_i, [c_vp, c_i64, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_vp, c_f, c_vp, c_vp, c_vp, c_sz]),
    "mpt_bn_bwd_apply": (c_i, [c_vp, c_i64, c_i64, c_vp, c_i64, c_vp, c_i64, c_vp, c_vp, c_vp, c_f, c_vp, c_vp, c_vp, c_i64]),
}

_lib = None


def lib():
    """Load libmpt.so (once).  Raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError("libmpt.so is not built (%s); run `python -m paper_1710_03740_amd.build`. "
                               "There is no fallback path." % LIB_PATH)
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in SIGNATURES.items():
            f = getattr(L, name)
            f.restype, f.argtypes = res, args
        _lib = L
    return _lib


def _check(fn, st):
    if st != 0:
        raise MptError(fn, st, lib().mpt_status_string(st).decode())


def _stream():
    return c_vp(torch.cuda.current_stream().cuda_stream)


def _p(t):
    return c_vp(0) if t is None else c_vp(t.data_ptr())


def _dev(*ts):
    for t in ts:
        if t is not None and not t.is_cuda:
            raise ValueError("mpt binding takes device tensors only")


# The C ABI sees pointers and sizes only, so a tensor of the wrong dtype, a transposed view or a buffer shorter than
# its neighbours would be read or written out of bounds on the device.  Every wrapper checks its tensors against each
# other here, before the library is touched; a mismatch raises ValueError.
_F16, _F32, _I32, _I64, _U8 = torch.float16, torch.float32, torch.int32, torch.int64, torch.uint8


def _want(name, t, dtypes, shape=None, numel=None, optional=False):
    """t: tensor (or None when optional); dtypes: one dtype or a tuple; shape: exact shape; numel: exact element count."""
    if t is None:
        if optional:
            return
        raise ValueError("%s: a tensor is required" % name)
    if not isinstance(dtypes, tuple):
        dtypes = (dtypes,)
    if t.dtype not in dtypes:
        raise ValueError("%s: dtype %s, expected %s" % (name, t.dtype, " or ".join(str(d) for d in dtypes)))
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError("%s: shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))
    if numel is not None and t.numel() != numel:
        raise ValueError("%s: %d elements, expected %d" % (name, t.numel(), numel))


def _rows(name, t):
    """A row-major matrix view: unit stride along the last axis and a row stride that covers a row."""
    if t.dim() != 2:
        raise ValueError("%s: expected a matrix, got %d dimensions" % (name, t.dim()))
    if t.shape[1] > 1 and t.stride(1) != 1:
        raise ValueError("%s: last-axis stride %d, expected 1 (transposed views are not accepted)" % (name, t.stride(1)))
    if t.shape[0] > 1 and t.stride(0) < t.shape[1]:
        raise ValueError("%s: row stride %d is smaller than the row length %d" % (name, t.stride(0), t.shape[1]))


def _flat(name, t, optional=False):
    """A dense buffer (elements in memory order, no gaps)."""
    if t is None and optional:
        return
    if not t.is_contiguous():
        raise ValueError("%s: expected a contiguous buffer" % name)


def _mat(name, t, dtypes, shape, optional=False):
    _want(name, t, dtypes, optional=optional)
    if t is None:
        return
    _rows(name, t)
    if tuple(t.shape) != tuple(shape):
        raise ValueError("%s: shape %s, expected %s" % (name, tuple(t.shape), tuple(shape)))


def _dim2(name, t):
    if t is None or t.dim() != 2:
        raise ValueError("%s: expected a matrix" % name)
    return t.shape


def _ws_ok(ws):
    if ws is not None:
        _flat("ws", ws)


def mpt_version():
    return lib().mpt_version()


def mpt_status_string(st):
    return lib().mpt_status_string(st).decode()


# ---------------------------------------------------------------- GEMMs
def mpt_gemm_workspace_bytes(op, M, N, K):
    return lib().mpt_gemm_workspace_bytes(op, M, N, K)


def _ws(ws):
    return (_p(ws), c_sz(0 if ws is None else ws.numel() * ws.element_size()))


def _fwd_shapes(X, W, Y, yname):
    M, K = _dim2("X", X)
    N = _dim2("W", W)[1]
    _mat("X", X, _F16, (M, K)); _mat("W", W, _F16, (K, N)); _mat(yname, Y, _F16, (M, N))
    return M, N, K


def _dgrad_shapes(dY, W, dX):
    M, N = _dim2("dY", dY)
    K = _dim2("W", W)[0]
    _mat("dY", dY, _F16, (M, N)); _mat("W", W, _F16, (K, N)); _mat("dX", dX, _F16, (M, K))
    return M, N, K


def mpt_gemm_fwd(X, W, Y, ws=None):
    M, N, K = _fwd_shapes(X, W, Y, "Y")
    _ws_ok(ws)
    _dev(X, W, Y, ws)
    p, b = _ws(ws)
    _check("mpt_gemm_fwd", lib().mpt_gemm_fwd(_stream(), M, N, K, _p(X), X.stride(0), _p(W), W.stride(0), _p(Y), Y.stride(0), p, b))


def mpt_gemm_dgrad(dY, W, dX, ws=None):
    M, N, K = _dgrad_shapes(dY, W, dX)
    _ws_ok(ws)
    _dev(dY, W, dX, ws)
    p, b = _ws(ws)
    _check("mpt_gemm_dgrad", lib().mpt_gemm_dgrad(_stream(), M, N, K, _p(dY), dY.stride(0), _p(W), W.stride(0), _p(dX), dX.stride(0), p, b))


def mpt_gemm_fwd_relu(X, W, H, ws=None):
    M, N, K = _fwd_shapes(X, W, H, "H")
    _ws_ok(ws)
    _dev(X, W, H, ws)
    p, b = _ws(ws)
    _check("mpt_gemm_fwd_relu", lib().mpt_gemm_fwd_relu(_stream(), M, N, K, _p(X), X.stride(0), _p(W), W.stride(0), _p(H), H.stride(0), p, b))


def mpt_gemm_dgrad_relu(dY, W, H, dX, ws=None):
    M, N, K = _dgrad_shapes(dY, W, dX)
    _mat("H", H, _F16, (M, K))
    _ws_ok(ws)
    _dev(dY, W, H, dX, ws)
    p, b = _ws(ws)
    _check("mpt_gemm_dgrad_relu", lib().mpt_gemm_dgrad_relu(_stream(), M, N, K, _p(dY), dY.stride(0), _p(W), W.stride(0),
                                                            _p(H), H.stride(0), _p(dX), dX.stride(0), p, b))


def mpt_gemm_wgrad(X, dY, dW, accumulate=False, flag=None, ws=None):
    M, K = _dim2("X", X)
    N = _dim2("dY", dY)[1]
    _mat("X", X, _F16, (M, K)); _mat("dY", dY, _F16, (M, N)); _mat("dW", dW, (_F16, _F32), (K, N))
    _want("flag", flag, _I32, numel=1, optional=True)
    _ws_ok(ws)
    out_fp32 = 1 if dW.dtype == torch.float32 else 0
    if accumulate and not out_fp32:
        raise ValueError("dW: accumulate needs an FP32 output")
    _dev(X, dY, dW, flag, ws)
    p, b = _ws(ws)
    _check("mpt_gemm_wgrad", lib().mpt_gemm_wgrad(_stream(), M, N, K, _p(X), X.stride(0), _p(dY), dY.stride(0), _p(dW), dW.stride(0),
                                                  out_fp32, 1 if accumulate else 0, _p(flag), p, b))


STATIC_SCRATCH_BYTES = 32 << 20


def mpt_gemm_wgrad_static(X, dY, dW, accumulate=False, flag=None):
    """mpt_gemm_wgrad with the split partials in the library's own device array (no allocation, no workspace)."""
    M, K = _dim2("X", X)
    N = _dim2("dY", dY)[1]
    _mat("X", X, _F16, (M, K)); _mat("dY", dY, _F16, (M, N)); _mat("dW", dW, (_F16, _F32), (K, N))
    _want("flag", flag, _I32, numel=1, optional=True)
    out_fp32 = 1 if dW.dtype == torch.float32 else 0
    if accumulate and not out_fp32:
        raise ValueError("dW: accumulate needs an FP32 output")
    _dev(X, dY, dW, flag)
    _check("mpt_gemm_wgrad_static", lib().mpt_gemm_wgrad_static(_stream(), M, N, K, _p(X), X.stride(0), _p(dY), dY.stride(0), _p(dW), dW.stride(0),
                                                                out_fp32, 1 if accumulate else 0, _p(flag)))


# ---------------------------------------------------------------- conv
def mpt_conv3x3_workspace_bytes(op, Nb, H, W, C, Kf):
    return lib().mpt_conv3x3_workspace_bytes(op, Nb, H, W, C, Kf)


def _conv_shapes(x, xname, w, y, yname):
    """x-like [Nb,H,W,C], filter-like [Kf,3,3,C], y-like [Nb,H,W,Kf]; all dense FP16."""
    if x is None or x.dim() != 4 or w is None or w.dim() != 4 or y is None:
        raise ValueError("conv: expected 4-d tensors %s [Nb,H,W,C], filter [Kf,3,3,C], %s [Nb,H,W,Kf]" % (xname, yname))
    Nb, H, W, C = x.shape
    Kf = w.shape[0]
    _want(xname, x, _F16); _want("filter", w, _F16, shape=(Kf, 3, 3, C)); _want(yname, y, _F16, shape=(Nb, H, W, Kf))
    _flat(xname, x); _flat("filter", w); _flat(yname, y)
    return Nb, H, W, C, Kf


def mpt_conv3x3_fwd(x, w, y, ws=None):
    Nb, H, W, C, Kf = _conv_shapes(x, "x", w, y, "y")
    _ws_ok(ws)
    _dev(x, w, y, ws)
    p, b = _ws(ws)
    _check("mpt_conv3x3_fwd", lib().mpt_conv3x3_fwd(_stream(), Nb, H, W, C, Kf, _p(x), _p(w), _p(y), p, b))


def mpt_conv3x3_dgrad(dy, w, dx, ws=None):
    Nb, H, W, C, Kf = _conv_shapes(dx, "dx", w, dy, "dy")
    _ws_ok(ws)
    _dev(dy, w, dx, ws)
    p, b = _ws(ws)
    _check("mpt_conv3x3_dgrad", lib().mpt_conv3x3_dgrad(_stream(), Nb, H, W, C, Kf, _p(dy), _p(w), _p(dx), p, b))


def mpt_conv3x3_wgrad(x, dy, dw, flag=None, ws=None):
    Nb, H, W, C, Kf = _conv_shapes(x, "x", dw, dy, "dy")
    _want("flag", flag, _I32, numel=1, optional=True)
    _ws_ok(ws)
    _dev(x, dy, dw, flag, ws)
    p, b = _ws(ws)
    _check("mpt_conv3x3_wgrad", lib().mpt_conv3x3_wgrad(_stream(), Nb, H, W, C, Kf, _p(x), _p(dy), _p(dw), _p(flag), p, b))


# ---------------------------------------------------------------- loss-scaled update path
def mpt_unscale_check(grad, inv_scale, flag, g32_out=None):
    _want("grad", grad, (_F16, _F32)); _flat("grad", grad)
    _want("flag", flag, _I32, numel=1)
    _want("g32_out", g32_out, _F32, numel=grad.numel(), optional=True); _flat("g32_out", g32_out, optional=True)
    _dev(grad, flag, g32_out)
    _check("mpt_unscale_check", lib().mpt_unscale_check(_stream(), _p(grad), 1 if grad.dtype == torch.float32 else 0,
                                                        grad.numel(), inv_scale, _p(g32_out), _p(flag)))


def _update_buffers(w32, states, grad, w16, flag, scaler_dev):
    """The flat buffers of one update: same element count everywhere, documented dtypes, dense."""
    _want("w32", w32, _F32); _flat("w32", w32)
    n = w32.numel()
    for name, t in states:
        _want(name, t, _F32, numel=n, optional=True); _flat(name, t, optional=True)
    _want("grad", grad, (_F16, _F32), numel=n); _flat("grad", grad)
    _want("w16", w16, _F16, numel=n); _flat("w16", w16)
    _want("flag", flag, _I32, numel=1, optional=True)
    _want("scaler_dev", scaler_dev, _U8, numel=ctypes.sizeof(mpt_scaler), optional=True)
    return n


def mpt_master_update(w32, m32, grad, w16, inv_scale, lr, momentum, flag=None, scaler_dev=None):
    _update_buffers(w32, [("m32", m32)], grad, w16, flag, scaler_dev)
    _dev(w32, m32, grad, w16, flag, scaler_dev)
    _check("mpt_master_update", lib().mpt_master_update(_stream(), w32.numel(), _p(w32), _p(m32), _p(grad),
                                                        1 if grad.dtype == torch.float32 else 0, _p(w16),
                                                        inv_scale, _p(scaler_dev), lr, momentum, _p(flag)))


def mpt_master_update_multi(tensors, inv_scale, lr, momentum, flag=None, scaler_dev=None):
    """tensors: a sequence of (w32, m32 or None, grad, w16) device tensors, one entry per parameter tensor; the gradients
    share one dtype and the momentum buffers are given for all entries or for none."""
    tensors = list(tensors)
    if not tensors:
        return
    gdt = tensors[0][2].dtype if tensors[0][2] is not None else None
    items = (mpt_update_item * len(tensors))()
    counts = []
    for k, (w32, m32, grad, w16) in enumerate(tensors):          # every entry is checked before the device check
        counts.append(_update_buffers(w32, [("m32", m32)], grad, w16, flag, scaler_dev))
        if grad.dtype != gdt:
            raise TypeError("tensors[%d]: gradient dtype %s differs from the first entry's %s" % (k, grad.dtype, gdt))
        if (m32 is None) != (tensors[0][1] is None):
            raise ValueError("tensors[%d]: momentum buffers for all entries or for none" % k)
    for k, (w32, m32, grad, w16) in enumerate(tensors):
        _dev(w32, m32, grad, w16)
        items[k].w32_dev, items[k].m32_dev, items[k].grad_dev, items[k].w16_dev, items[k].n = _p(w32), _p(m32), _p(grad), _p(w16), counts[k]
    _dev(flag, scaler_dev)
    _check("mpt_master_update_multi", lib().mpt_master_update_multi(_stream(), len(tensors), ctypes.cast(items, c_vp),
                                                                    1 if gdt == torch.float32 else 0, inv_scale, _p(scaler_dev),
                                                                    lr, momentum, _p(flag)))


def mpt_master_update_fused(w32_in, m32_in, grad, w32_out, m32_out, w16_out, inv_scale, lr, momentum, flag, scaler_dev=None):
    n = _update_buffers(w32_in, [("m32_in", m32_in), ("m32_out", m32_out)], grad, w16_out, flag, scaler_dev)
    _want("w32_out", w32_out, _F32, numel=n); _flat("w32_out", w32_out)
    _want("flag", flag, _I32, numel=1)
    if (m32_in is None) != (m32_out is None):
        raise ValueError("m32_in and m32_out: both or neither")
    _dev(w32_in, m32_in, grad, w32_out, m32_out, w16_out, flag, scaler_dev)
    _check("mpt_master_update_fused", lib().mpt_master_update_fused(_stream(), w32_in.numel(), _p(w32_in), _p(m32_in), _p(grad),
                                                                    1 if grad.dtype == torch.float32 else 0, _p(w32_out), _p(m32_out),
                                                                    _p(w16_out), inv_scale, _p(scaler_dev), lr, momentum, _p(flag)))


def mpt_optimizer_update(kind, hp, w32, state1, state2, grad, w16, inv_scale, flag=None, scaler_dev=None):
    """kind: a key of OPT_KINDS; hp: an mpt_opt_params (host struct; its clip_factor_dev is a device address or None)."""
    if kind not in OPT_KINDS:
        raise ValueError("kind: %r, expected one of %s" % (kind, sorted(OPT_KINDS)))
    _update_buffers(w32, [("state1", state1), ("state2", state2)], grad, w16, flag, scaler_dev)
    if state1 is None or (kind == "adam" and state2 is None):
        raise ValueError("optimizer state: state1 is required (and state2 for adam)")
    _dev(w32, state1, state2, grad, w16, flag, scaler_dev)
    _check("mpt_optimizer_update", lib().mpt_optimizer_update(_stream(), w32.numel(), OPT_KINDS[kind], ctypes.byref(hp), _p(w32), _p(state1),
                                                              _p(state2), _p(grad), 1 if grad.dtype == torch.float32 else 0, _p(w16),
                                                              inv_scale, _p(scaler_dev), _p(flag)))


def mpt_grad_norm_workspace_bytes():
    return lib().mpt_grad_norm_workspace_bytes()


def mpt_grad_sumsq(grad, inv_scale, sumsq, ws, flag=None, accumulate=False, scaler_dev=None):
    """sumsq: float64[1] device tensor; ws: device scratch of mpt_grad_norm_workspace_bytes() bytes."""
    _want("grad", grad, (_F16, _F32)); _flat("grad", grad)
    _want("sumsq", sumsq, torch.float64, numel=1)
    _want("flag", flag, _I32, numel=1, optional=True)
    _want("scaler_dev", scaler_dev, _U8, numel=ctypes.sizeof(mpt_scaler), optional=True)
    _ws_ok(ws)
    _dev(grad, sumsq, ws, flag, scaler_dev)
    p, b = _ws(ws)
    _check("mpt_grad_sumsq", lib().mpt_grad_sumsq(_stream(), _p(grad), 1 if grad.dtype == torch.float32 else 0, grad.numel(), inv_scale,
                                                  _p(scaler_dev), 1 if accumulate else 0, _p(sumsq), _p(flag), p, b))


def mpt_clip_factor(sumsq, max_norm, factor, norm=None):
    """factor (and the optional norm): float32[1] device tensors."""
    _want("sumsq", sumsq, torch.float64, numel=1); _want("factor", factor, _F32, numel=1); _want("norm", norm, _F32, numel=1, optional=True)
    _dev(sumsq, factor, norm)
    _check("mpt_clip_factor", lib().mpt_clip_factor(_stream(), _p(sumsq), max_norm, _p(factor), _p(norm)))


def mpt_grad_stats(grad, hist, absmax_bits, accumulate=False):
    """hist: int64[42] device tensor; absmax_bits: int32[1] device tensor."""
    _want("grad", grad, _F16); _flat("grad", grad)
    _want("hist", hist, _I64, numel=42); _flat("hist", hist)
    _want("absmax_bits", absmax_bits, _I32, numel=1)
    _dev(grad, hist, absmax_bits)
    _check("mpt_grad_stats", lib().mpt_grad_stats(_stream(), _p(grad), grad.numel(), 1 if accumulate else 0, _p(hist), _p(absmax_bits)))


def mpt_suggest_loss_scale_log2(absmax_bits, if_zero=0):
    return lib().mpt_suggest_loss_scale_log2(int(absmax_bits) & 0xFFFFFFFF, if_zero)


def mpt_scaler_init(scale, growth_interval):
    s = mpt_scaler()
    _check("mpt_scaler_init", lib().mpt_scaler_init(ctypes.byref(s), scale, growth_interval))
    return s


def mpt_loss_scale_update(s, overflow):
    _check("mpt_loss_scale_update", lib().mpt_loss_scale_update(ctypes.byref(s), 1 if overflow else 0))
    return s.scale


def mpt_loss_scale_update_dev(scaler_dev, flag):
    _want("scaler_dev", scaler_dev, _U8, numel=ctypes.sizeof(mpt_scaler)); _want("flag", flag, _I32, numel=1)
    _dev(scaler_dev, flag)
    _check("mpt_loss_scale_update_dev", lib().mpt_loss_scale_update_dev(_stream(), _p(scaler_dev), _p(flag)))


def scaler_to_device(s, device="cuda"):
    """Copy a host mpt_scaler struct into a fresh 32-byte device buffer."""
    raw = bytes(s)
    return torch.frombuffer(bytearray(raw), dtype=torch.uint8).to(device)


def scaler_from_device(buf):
    return mpt_scaler.from_buffer_copy(bytes(buf.cpu().numpy().tobytes()))


def mpt_probe_mfma(iters, random_operands, sink):
    _want("sink", sink, _F32, numel=1)
    _dev(sink)
    _check("mpt_probe_mfma", lib().mpt_probe_mfma(_stream(), iters, 1 if random_operands else 0, _p(sink)))


# ---------------------------------------------------------------- glue
def mpt_add_fp16(a, b, out):
    _want("a", a, _F16); _flat("a", a)
    _want("b", b, _F16, numel=a.numel()); _flat("b", b); _want("out", out, _F16, numel=a.numel()); _flat("out", out)
    _dev(a, b, out)
    _check("mpt_add_fp16", lib().mpt_add_fp16(_stream(), a.numel(), _p(a), _p(b), _p(out)))


def mpt_relu_fwd(y, h):
    _want("y", y, _F16); _flat("y", y); _want("h", h, _F16, numel=y.numel()); _flat("h", h)
    _dev(y, h)
    _check("mpt_relu_fwd", lib().mpt_relu_fwd(_stream(), y.numel(), _p(y), _p(h)))


def mpt_relu_bwd(dh, y, dy):
    _want("y", y, _F16); _flat("y", y)
    _want("dh", dh, _F16, numel=y.numel()); _flat("dh", dh); _want("dy", dy, _F16, numel=y.numel()); _flat("dy", dy)
    _dev(dh, y, dy)
    _check("mpt_relu_bwd", lib().mpt_relu_bwd(_stream(), y.numel(), _p(dh), _p(y), _p(dy)))


def mpt_softmax_xent_scaled(logits, labels, scale, dlogits, loss=None, row_loss=None):
    B, C = _dim2("logits", logits)
    _mat("logits", logits, _F16, (B, C)); _mat("dlogits", dlogits, _F16, (B, C))
    _want("labels", labels, _I32, numel=B); _flat("labels", labels)
    _want("loss", loss, _F32, numel=1, optional=True)
    _want("row_loss", row_loss, _F32, numel=B, optional=True); _flat("row_loss", row_loss, optional=True)
    if loss is not None and row_loss is None:
        raise ValueError("row_loss: required when loss is given")
    _dev(logits, labels, dlogits, loss, row_loss)
    _check("mpt_softmax_xent_scaled", lib().mpt_softmax_xent_scaled(_stream(), B, C, _p(logits), logits.stride(0), _p(labels),
                                                                    scale, _p(loss), _p(row_loss), _p(dlogits), dlogits.stride(0)))


# ---------------------------------------------------------------- batch normalisation (x viewed as [P, C])
def mpt_bn_workspace_bytes(P, C):
    return lib().mpt_bn_workspace_bytes(P, C)


def _bn_shapes(x, vectors, tensors):
    """x [P, C] FP16; per-channel FP32 vectors of C elements; further FP16 tensors of x's shape."""
    P, C = _dim2("x", x)
    _mat("x", x, _F16, (P, C))
    for name, v in vectors:
        _want(name, v, _F32, numel=C); _flat(name, v)
    for name, t in tensors:
        _mat(name, t, _F16, (P, C))
    return P, C


def mpt_bn_stats(x, mean, var, ws):
    P, C = _bn_shapes(x, [("mean", mean), ("var", var)], [])
    _ws_ok(ws)
    _dev(x, mean, var, ws)
    p, b = _ws(ws)
    _check("mpt_bn_stats", lib().mpt_bn_stats(_stream(), P, C, _p(x), x.stride(0), _p(mean), _p(var), p, b))


def mpt_bn_apply(x, mean, var, gamma, beta, eps, y, relu=False):
    P, C = _bn_shapes(x, [("mean", mean), ("var", var), ("gamma", gamma), ("beta", beta)], [("y", y)])
    _dev(x, mean, var, gamma, beta, y)
    _check("mpt_bn_apply", lib().mpt_bn_apply(_stream(), P, C, _p(x), x.stride(0), _p(mean), _p(var), _p(gamma), _p(beta),
                                              eps, 1 if relu else 0, _p(y), y.stride(0)))


def mpt_bn_bwd_reduce(x, dy, mean, var, eps, dgamma, dbeta, ws):
    P, C = _bn_shapes(x, [("mean", mean), ("var", var), ("dgamma", dgamma), ("dbeta", dbeta)], [("dy", dy)])
    _ws_ok(ws)
    _dev(x, dy, mean, var, dgamma, dbeta, ws)
    p, b = _ws(ws)
    _check("mpt_bn_bwd_reduce", lib().mpt_bn_bwd_reduce(_stream(), P, C, _p(x), x.stride(0), _p(dy), dy.stride(0), _p(mean), _p(var),
                                                        eps, _p(dgamma), _p(dbeta), p, b))


def mpt_bn_bwd_apply(x, dy, mean, var, gamma, eps, dgamma, dbeta, dx):
    P, C = _bn_shapes(x, [("mean", mean), ("var", var), ("gamma", gamma), ("dgamma", dgamma), ("dbeta", dbeta)], [("dy", dy), ("dx", dx)])
    _dev(x, dy, mean, var, gamma, dgamma, dbeta, dx)
    _check("mpt_bn_bwd_apply", lib().mpt_bn_bwd_apply(_stream(), P, C, _p(x), x.stride(0), _p(dy), dy.stride(0), _p(mean), _p(var),
                                                      _p(gamma), eps, _p(dgamma), _p(dbeta), _p(dx), dx.stride(0)))


# ---------------------------------------------------------------- LSTM cell (pointwise part)
def _ld(t):
    return 0 if t is None else t.stride(0)


def mpt_lstm_cell_fwd(gx, gr, bias, c_prev, act, c, h):
    B, H = _dim2("c_prev", c_prev)
    _mat("c_prev", c_prev, _F16, (B, H)); _mat("c", c, _F16, (B, H)); _mat("h", h, _F16, (B, H))
    _mat("gx", gx, _F16, (B, 4 * H)); _mat("gr", gr, _F16, (B, 4 * H), optional=True); _mat("act", act, _F16, (B, 4 * H))
    _want("bias", bias, _F32, numel=4 * H, optional=True); _flat("bias", bias, optional=True)
    _dev(gx, gr, bias, c_prev, act, c, h)
    _check("mpt_lstm_cell_fwd", lib().mpt_lstm_cell_fwd(_stream(), B, H, _p(gx), _ld(gx), _p(gr), _ld(gr), _p(bias), _p(c_prev), _ld(c_prev),
                                                        _p(act), _ld(act), _p(c), _ld(c), _p(h), _ld(h)))


def mpt_lstm_cell_bwd(dh, dc_next, act, c, c_prev, da, dc_prev):
    B, H = _dim2("c", c)
    for name, t in (("dh", dh), ("c", c), ("c_prev", c_prev), ("dc_prev", dc_prev)):
        _mat(name, t, _F16, (B, H))
    _mat("dc_next", dc_next, _F16, (B, H), optional=True)
    _mat("act", act, _F16, (B, 4 * H)); _mat("da", da, _F16, (B, 4 * H))
    _dev(dh, dc_next, act, c, c_prev, da, dc_prev)
    _check("mpt_lstm_cell_bwd", lib().mpt_lstm_cell_bwd(_stream(), B, H, _p(dh), _ld(dh), _p(dc_next), _ld(dc_next), _p(act), _ld(act), _p(c), _ld(c),
                                                        _p(c_prev), _ld(c_prev), _p(da), _ld(da), _p(dc_prev), _ld(dc_prev)))
