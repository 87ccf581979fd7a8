"""Pins for the oracle's 3x3 convolution: explicit loops on tiny inputs,
torch's float64 conv2d and its autograd (an independent library routine),
reduction to a plain GEMM for a 1x1 image, identity filter, integer exactness."""
import numpy as np
import torch

from oracle import conv, fp16, gemm


def _rand(rng, shape, s=1.0):
    return (rng.standard_normal(shape) * s).astype(np.float16)


def test_loops_definition_matches():
    rng = np.random.default_rng(0)
    x, w, dy = _rand(rng, (2, 3, 4, 3)), _rand(rng, (2, 3, 3, 3), 0.3), _rand(rng, (2, 3, 4, 2), 0.1)
    assert np.array_equal(fp16.bits(conv.conv3x3_fwd(x, w)[0]), fp16.bits(conv.conv3x3_fwd_loops(x, w)))
    assert np.array_equal(fp16.bits(conv.conv3x3_dgrad(dy, w)[0]), fp16.bits(conv.conv3x3_dgrad_loops(dy, w)))
    assert np.array_equal(fp16.bits(conv.conv3x3_wgrad(x, dy)[0]), fp16.bits(conv.conv3x3_wgrad_loops(x, dy)))


def test_against_torch_conv2d_and_autograd():
    rng = np.random.default_rng(1)
    x, w, dy = _rand(rng, (3, 5, 6, 8)), _rand(rng, (4, 3, 3, 8), 0.2), _rand(rng, (3, 5, 6, 4), 0.05)
    tx = torch.tensor(x.astype(np.float64)).permute(0, 3, 1, 2).requires_grad_(True)   # NCHW view
    tw = torch.tensor(w.astype(np.float64)).permute(0, 3, 1, 2).requires_grad_(True)   # KCRS view
    ty = torch.nn.functional.conv2d(tx, tw, stride=1, padding=1)
    ty.backward(torch.tensor(dy.astype(np.float64)).permute(0, 3, 1, 2))
    with np.errstate(over="ignore"):
        want_y = ty.detach().permute(0, 2, 3, 1).numpy().astype(np.float16)
        want_dx = tx.grad.permute(0, 2, 3, 1).numpy().astype(np.float16)
        want_dw = tw.grad.permute(0, 2, 3, 1).numpy().astype(np.float16)
    # torch sums in a different order; allow the last FP16 step on near-ties only
    for got, want in ((conv.conv3x3_fwd(x, w)[0], want_y), (conv.conv3x3_dgrad(dy, w)[0], want_dx),
                      (conv.conv3x3_wgrad(x, dy)[0], want_dw)):
        d = fp16.ulpdist16(fp16.bits(got), fp16.bits(want))
        assert d.max() <= 1 and (d > 0).mean() < 0.01


def test_integer_exact():
    rng = np.random.default_rng(2)
    x = rng.integers(-3, 4, (2, 4, 4, 5)).astype(np.float16)
    w = rng.integers(-3, 4, (3, 3, 3, 5)).astype(np.float16)
    dy = rng.integers(-3, 4, (2, 4, 4, 3)).astype(np.float16)
    tx = torch.tensor(x.astype(np.int64)).permute(0, 3, 1, 2).double().requires_grad_(True)
    tw = torch.tensor(w.astype(np.int64)).permute(0, 3, 1, 2).double().requires_grad_(True)
    ty = torch.nn.functional.conv2d(tx, tw, padding=1)
    ty.backward(torch.tensor(dy.astype(np.float64)).permute(0, 3, 1, 2))
    assert np.array_equal(conv.conv3x3_fwd(x, w)[0].astype(np.float64), ty.detach().permute(0, 2, 3, 1).numpy())
    assert np.array_equal(conv.conv3x3_dgrad(dy, w)[0].astype(np.float64), tx.grad.permute(0, 2, 3, 1).numpy())
    assert np.array_equal(conv.conv3x3_wgrad(x, dy)[0].astype(np.float64), tw.grad.permute(0, 2, 3, 1).numpy())


def test_one_pixel_image_reduces_to_gemm_on_centre_tap():
    rng = np.random.default_rng(3)
    x, w, dy = _rand(rng, (7, 1, 1, 6)), _rand(rng, (5, 3, 3, 6), 0.3), _rand(rng, (7, 1, 1, 5), 0.1)
    wc = np.ascontiguousarray(w[:, 1, 1, :].T)                       # [C, Kf]
    y, _ = conv.conv3x3_fwd(x, w)
    assert np.array_equal(fp16.bits(y.reshape(7, 5)), fp16.bits(gemm.gemm_fwd(x.reshape(7, 6), wc)[0]))
    dx, _ = conv.conv3x3_dgrad(dy, w)
    assert np.array_equal(fp16.bits(dx.reshape(7, 6)), fp16.bits(gemm.gemm_dgrad(dy.reshape(7, 5), wc)[0]))
    dw, _ = conv.conv3x3_wgrad(x, dy)
    want = gemm.gemm_wgrad(x.reshape(7, 6), dy.reshape(7, 5))[0]     # [C, Kf]
    assert np.array_equal(fp16.bits(dw[:, 1, 1, :]), fp16.bits(np.ascontiguousarray(want.T)))
    off = dw.copy(); off[:, 1, 1, :] = 0
    assert not off.any()                                             # other taps see only padding


def test_identity_and_shift_filters():
    rng = np.random.default_rng(4)
    x = _rand(rng, (2, 5, 5, 4))
    w = np.zeros((4, 3, 3, 4), dtype=np.float16)
    for c in range(4):
        w[c, 1, 1, c] = 1
    assert np.array_equal(fp16.bits(conv.conv3x3_fwd(x, w)[0]), fp16.bits(x))
    w[:] = 0
    for c in range(4):
        w[c, 0, 2, c] = 1                                            # tap (r=0,s=2): y[p,q] = x[p-1,q+1]
    y, _ = conv.conv3x3_fwd(x, w)
    assert np.array_equal(y[:, 1:, :-1, :], x[:, :-1, 1:, :])
    assert not y[:, 0].any() and not y[:, :, -1].any()
