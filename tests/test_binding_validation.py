"""The Python binding rejects tensors that do not fit each other before anything reaches the C ABI (which sees only
pointers and sizes): wrong dtype, transposed or strided views, element counts that differ between the buffers of one
update, inconsistent GEMM / convolution / batch-norm / LSTM shapes.  All on CPU tensors: the checks run before the
device check and before the library is loaded, so a well-formed CPU call ends in the "device tensors only" error."""
import pytest
import torch

from paper_1710_03740_amd import binding as mpt

F16, F32, I32 = torch.float16, torch.float32, torch.int32


def h(*shape):
    return torch.zeros(*shape, dtype=F16)


def f(*shape):
    return torch.zeros(*shape, dtype=F32)


def flag():
    return torch.zeros(1, dtype=I32)


def reaches_device_check(fn, *a, **k):
    with pytest.raises(ValueError, match="device tensors only"):
        fn(*a, **k)


def rejected(match, fn, *a, **k):
    with pytest.raises(ValueError, match=match):
        fn(*a, **k)


def test_gemm_shapes_dtypes_and_views():
    X, W, Y = h(8, 16), h(16, 24), h(8, 24)
    reaches_device_check(mpt.mpt_gemm_fwd, X, W, Y)
    rejected("W: shape", mpt.mpt_gemm_fwd, X, h(15, 24), Y)                    # X.shape[1] != W.shape[0]
    rejected("Y: shape", mpt.mpt_gemm_fwd, X, W, h(8, 23))
    rejected("X: dtype", mpt.mpt_gemm_fwd, f(8, 16), W, Y)                     # FP32 passed as FP16
    rejected("last-axis stride", mpt.mpt_gemm_fwd, h(16, 8).t(), W, Y)         # a transposed view is not row-major
    rejected("last-axis stride", mpt.mpt_gemm_fwd, h(8, 32)[:, ::2], W, Y)
    rejected("expected a matrix", mpt.mpt_gemm_fwd, h(8 * 16), W, Y)
    reaches_device_check(mpt.mpt_gemm_fwd, h(8, 32)[:, :16], W, Y)             # a row-strided view is fine
    reaches_device_check(mpt.mpt_gemm_fwd_relu, X, W, Y)
    dY, dX = h(8, 24), h(8, 16)
    reaches_device_check(mpt.mpt_gemm_dgrad, dY, W, dX)
    rejected("W: shape", mpt.mpt_gemm_dgrad, dY, h(16, 23), dX)
    rejected("dX: shape", mpt.mpt_gemm_dgrad, dY, W, h(8, 24))
    rejected("H: shape", mpt.mpt_gemm_dgrad_relu, dY, W, h(8, 15), dX)
    reaches_device_check(mpt.mpt_gemm_wgrad, X, dY, h(16, 24))
    reaches_device_check(mpt.mpt_gemm_wgrad, X, dY, f(16, 24), accumulate=True, flag=flag())
    rejected("dY: shape", mpt.mpt_gemm_wgrad, X, h(9, 24), h(16, 24))
    rejected("dW: shape", mpt.mpt_gemm_wgrad, X, dY, h(24, 16))
    rejected("accumulate needs an FP32", mpt.mpt_gemm_wgrad, X, dY, h(16, 24), accumulate=True)
    rejected("flag: dtype", mpt.mpt_gemm_wgrad, X, dY, h(16, 24), flag=torch.zeros(1, dtype=torch.int64))
    rejected("contiguous", mpt.mpt_gemm_fwd, X, W, Y, ws=f(4, 8).t())


def test_conv_shapes():
    x, w, y = h(2, 5, 6, 8), h(16, 3, 3, 8), h(2, 5, 6, 16)
    reaches_device_check(mpt.mpt_conv3x3_fwd, x, w, y)
    reaches_device_check(mpt.mpt_conv3x3_dgrad, y, w, x)
    reaches_device_check(mpt.mpt_conv3x3_wgrad, x, y, w)
    rejected("filter: shape", mpt.mpt_conv3x3_fwd, x, h(16, 3, 3, 16), y)
    rejected("filter: shape", mpt.mpt_conv3x3_fwd, x, h(16, 5, 5, 8), y)
    rejected("y: shape", mpt.mpt_conv3x3_fwd, x, w, h(2, 5, 6, 8))
    rejected("dy: shape", mpt.mpt_conv3x3_wgrad, x, h(2, 6, 5, 16), w)
    rejected("contiguous", mpt.mpt_conv3x3_fwd, h(2, 6, 5, 8).transpose(1, 2), w, y)
    rejected("x: dtype", mpt.mpt_conv3x3_fwd, f(2, 5, 6, 8), w, y)
    rejected("4-d", mpt.mpt_conv3x3_fwd, h(60, 8), w, y)


def test_update_buffers_must_agree_in_length_and_dtype():
    n = 100
    w32, m32, g, w16 = f(n), f(n), h(n), h(n)
    reaches_device_check(mpt.mpt_master_update, w32, m32, g, w16, 1.0, 0.1, 0.9, flag())
    reaches_device_check(mpt.mpt_master_update, w32, None, f(n), w16, 1.0, 0.1, 0.9)
    rejected("m32: 99 elements", mpt.mpt_master_update, w32, f(n - 1), g, w16, 1.0, 0.1, 0.9)
    rejected("grad: 99 elements", mpt.mpt_master_update, w32, m32, h(n - 1), w16, 1.0, 0.1, 0.9)
    rejected("w16: 50 elements", mpt.mpt_master_update, w32, m32, g, h(n // 2), 1.0, 0.1, 0.9)
    rejected("w16: dtype", mpt.mpt_master_update, w32, m32, g, f(n), 1.0, 0.1, 0.9)
    rejected("w32: dtype", mpt.mpt_master_update, h(n), m32, g, w16, 1.0, 0.1, 0.9)
    rejected("contiguous", mpt.mpt_master_update, f(2 * n)[::2], m32, g, w16, 1.0, 0.1, 0.9)
    rejected("scaler_dev", mpt.mpt_master_update, w32, m32, g, w16, 1.0, 0.1, 0.9, None, torch.zeros(16, dtype=torch.uint8))
    o32, om, o16 = f(n), f(n), h(n)
    reaches_device_check(mpt.mpt_master_update_fused, w32, m32, g, o32, om, o16, 1.0, 0.1, 0.9, flag())
    rejected("w32_out: 101 elements", mpt.mpt_master_update_fused, w32, m32, g, f(n + 1), om, o16, 1.0, 0.1, 0.9, flag())
    rejected("m32_out: 7 elements", mpt.mpt_master_update_fused, w32, m32, g, o32, f(7), o16, 1.0, 0.1, 0.9, flag())
    rejected("both or neither", mpt.mpt_master_update_fused, w32, m32, g, o32, None, o16, 1.0, 0.1, 0.9, flag())
    rejected("flag", mpt.mpt_master_update_fused, w32, m32, g, o32, om, o16, 1.0, 0.1, 0.9, None)
    hp = mpt.mpt_opt_params()
    reaches_device_check(mpt.mpt_optimizer_update, "adam", hp, w32, m32, f(n), g, w16, 1.0)
    rejected("state2: 3 elements", mpt.mpt_optimizer_update, "adam", hp, w32, m32, f(3), g, w16, 1.0)
    rejected("state2 for adam", mpt.mpt_optimizer_update, "adam", hp, w32, m32, None, g, w16, 1.0)
    rejected("kind", mpt.mpt_optimizer_update, "lamb", hp, w32, m32, None, g, w16, 1.0)
    reaches_device_check(mpt.mpt_unscale_check, g, 1.0, flag(), f(n))
    rejected("g32_out: 99 elements", mpt.mpt_unscale_check, g, 1.0, flag(), f(n - 1))
    rejected("flag: a tensor is required", mpt.mpt_unscale_check, g, 1.0, None)
    rejected("hist: 41 elements", mpt.mpt_grad_stats, g, torch.zeros(41, dtype=torch.int64), flag())
    rejected("hist: dtype", mpt.mpt_grad_stats, g, torch.zeros(42, dtype=I32), flag())
    rejected("grad: dtype", mpt.mpt_grad_stats, f(n), torch.zeros(42, dtype=torch.int64), flag())


def test_glue_norm_and_lstm_shapes():
    reaches_device_check(mpt.mpt_relu_fwd, h(10), h(10))
    rejected("h: 9 elements", mpt.mpt_relu_fwd, h(10), h(9))
    rejected("dy: 11 elements", mpt.mpt_relu_bwd, h(10), h(10), h(11))
    lab = torch.zeros(4, dtype=I32)
    reaches_device_check(mpt.mpt_softmax_xent_scaled, h(4, 10), lab, 8.0, h(4, 10), f(1), f(4))
    rejected("labels: dtype", mpt.mpt_softmax_xent_scaled, h(4, 10), lab.long(), 8.0, h(4, 10))
    rejected("labels: 3 elements", mpt.mpt_softmax_xent_scaled, h(4, 10), lab[:3], 8.0, h(4, 10))
    rejected("dlogits: shape", mpt.mpt_softmax_xent_scaled, h(4, 10), lab, 8.0, h(4, 9))
    rejected("row_loss: required", mpt.mpt_softmax_xent_scaled, h(4, 10), lab, 8.0, h(4, 10), f(1), None)
    x, c = h(12, 8), f(8)
    reaches_device_check(mpt.mpt_bn_stats, x, c, f(8), f(64))
    rejected("var: 7 elements", mpt.mpt_bn_stats, x, c, f(7), f(64))
    rejected("y: shape", mpt.mpt_bn_apply, x, c, c, c, c, 1e-5, h(12, 16))
    rejected("gamma: dtype", mpt.mpt_bn_apply, x, c, c, h(8), c, 1e-5, h(12, 8))
    rejected("dy: shape", mpt.mpt_bn_bwd_reduce, x, h(11, 8), c, c, 1e-5, f(8), f(8), f(64))
    rejected("dx: shape", mpt.mpt_bn_bwd_apply, x, x, c, c, c, 1e-5, c, c, h(8, 12))
    B, H = 3, 8
    reaches_device_check(mpt.mpt_lstm_cell_fwd, h(B, 4 * H), h(B, 4 * H), f(4 * H), h(B, H), h(B, 4 * H), h(B, H), h(B, H))
    reaches_device_check(mpt.mpt_lstm_cell_fwd, h(B, 4 * H), None, None, h(B, H), h(B, 4 * H), h(B, H), h(B, H))
    rejected("gx: shape", mpt.mpt_lstm_cell_fwd, h(B, 3 * H), None, None, h(B, H), h(B, 4 * H), h(B, H), h(B, H))
    rejected("bias: 8 elements", mpt.mpt_lstm_cell_fwd, h(B, 4 * H), None, f(H), h(B, H), h(B, 4 * H), h(B, H), h(B, H))
    reaches_device_check(mpt.mpt_lstm_cell_bwd, h(B, H), None, h(B, 4 * H), h(B, H), h(B, H), h(B, 4 * H), h(B, H))
    rejected("da: shape", mpt.mpt_lstm_cell_bwd, h(B, H), None, h(B, 4 * H), h(B, H), h(B, H), h(B, H), h(B, H))
    rejected("dc_next: shape", mpt.mpt_lstm_cell_bwd, h(B, H), h(B, 2 * H), h(B, 4 * H), h(B, H), h(B, H), h(B, 4 * H), h(B, H))


def test_many_tensor_update_entries_are_checked_one_by_one():
    good = (f(8), f(8), h(8), h(8))
    reaches_device_check(mpt.mpt_master_update_multi, [good, (f(5), f(5), h(5), h(5))], 1.0, 0.1, 0.9)
    mpt.mpt_master_update_multi([], 1.0, 0.1, 0.9)                                                   # nothing to do
    rejected("grad: 4 elements", mpt.mpt_master_update_multi, [good, (f(5), f(5), h(4), h(5))], 1.0, 0.1, 0.9)       # a short gradient
    rejected("momentum buffers", mpt.mpt_master_update_multi, [good, (f(5), None, h(5), h(5))], 1.0, 0.1, 0.9)
    with pytest.raises(TypeError, match="gradient dtype"):
        mpt.mpt_master_update_multi([good, (f(5), f(5), f(5), h(5))], 1.0, 0.1, 0.9)
