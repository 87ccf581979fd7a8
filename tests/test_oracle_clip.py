"""Pins for the clipping oracle (paper Sec. 3.2: gradients are unscaled before clipping, so the clip threshold is
the FP32 one).  Closed forms on exactly representable values, the 3-4-5 triangle, invariance under the loss scale,
torch's clip_grad_norm_ in FP64, and planted mistakes (scaled instead of unscaled norm, per-buffer instead of
global norm, factor applied after weight decay)."""
import numpy as np
import torch

from oracle import clip, optim

F = np.float32


def test_three_four_five_and_threshold_edges():
    g = np.array([3.0, 4.0], dtype=np.float16)
    assert clip.unscaled_sumsq(g, 1.0) == 25.0
    f, n = clip.clip_factor(25.0, 10.0)
    assert (f, n) == (F(1.0), 5.0)                           # below the threshold: untouched
    f, n = clip.clip_factor(25.0, 5.0)
    assert f == F(1.0)                                        # exactly at it: untouched
    f, n = clip.clip_factor(25.0, 2.5)
    assert f == F(0.5) and n == 5.0
    out, f, n = clip.clip_by_global_norm(g, 1.0, 2.5)
    assert np.array_equal(out[0], np.array([1.5, 2.0], dtype=F))
    assert abs(float(np.sqrt((out[0].astype(np.float64) ** 2).sum())) - 2.5) < 1e-7


def test_norm_is_taken_on_the_unscaled_gradient_and_does_not_move_with_the_loss_scale():
    rng = np.random.default_rng(0)
    true = (rng.standard_normal(4096) * 2.0 ** -9)
    results = []
    for S in (1.0, 128.0, 8192.0):
        g16 = (true * S).astype(np.float32).astype(np.float16)
        # keep only values that are FP16-normal at S = 1 so that all three quantisations hold the same numbers
        keep = np.abs(true) >= 2.0 ** -13
        g16 = np.where(keep, g16, np.float16(0))
        results.append(clip.unscaled_sumsq(g16, 1.0 / S))
    assert results[1] == results[2]                           # power-of-two scaling is exact on normals
    assert abs(results[0] - results[1]) <= 2.0 ** -11 * results[1]   # S = 1 only differs by its coarser quantisation
    # a planted mistake (norm of the scaled gradient) would be S^2 larger
    g16 = (true * 128.0).astype(np.float32).astype(np.float16)
    assert clip.unscaled_sumsq(g16, 1.0) > 1e4 * clip.unscaled_sumsq(g16, 1.0 / 128.0)


def test_global_norm_spans_all_buffers_and_matches_torch():
    rng = np.random.default_rng(1)
    bufs = [rng.standard_normal(n).astype(np.float32) for n in (7, 1000, 33)]
    S = 64.0
    scaled = [(b * S).astype(np.float32) for b in bufs]
    out, f, n = clip.clip_by_global_norm(scaled, 1.0 / S, 3.0)
    ps = [torch.nn.Parameter(torch.zeros(len(b), dtype=torch.float64)) for b in bufs]
    for p, b in zip(ps, bufs):
        p.grad = torch.from_numpy(b.astype(np.float64))
    tn = float(torch.nn.utils.clip_grad_norm_(ps, 3.0, foreach=False))
    assert abs(tn - n) <= 1e-12 * n and n > 3.0
    for p, o in zip(ps, out):
        # torch divides by (norm + 1e-6); the oracle's factor is max_norm / norm: they differ by 1e-6 / norm relatively
        assert np.allclose(p.grad.numpy(), o.astype(np.float64), rtol=1e-6, atol=0)
    # per-buffer clipping (a planted mistake) gives a different factor for the small buffer
    _, f_small, _ = clip.clip_by_global_norm(scaled[0], 1.0 / S, 3.0)
    assert f_small != f


def test_factor_is_one_rounding_of_the_fp64_quotient():
    sumsq = 7.0
    f, n = clip.clip_factor(sumsq, 1.0)
    assert f == F(1.0 / np.sqrt(7.0)) and f.dtype == np.float32
    f_nan, _ = clip.clip_factor(float("nan"), 1.0)
    assert f_nan == F(1.0)
    f_inf, _ = clip.clip_factor(float("inf"), 1.0)
    assert f_inf == F(0.0)


def test_clip_enters_the_update_before_weight_decay():
    w = np.array([1.0, -2.0], dtype=F)
    m = np.zeros(2, dtype=F)
    g = np.array([8.0, 6.0], dtype=np.float16)                # unscaled with inv = 1/2: (4, 3), norm 5
    p = optim.OptParams(lr=0.5, momentum=0.0, weight_decay=0.25)
    factor, _ = clip.clip_factor(clip.unscaled_sumsq(g, 0.5), 2.5)
    assert factor == F(0.5)
    w2, m2, _, w16 = optim.optimizer_update("momentum", w, m, None, g, 0.5, p, 0, clip=factor)
    # g = (4, 3) * 0.5 = (2, 1.5); + 0.25 * w = (2.25, 1.0); w - 0.5 * g = (1 - 1.125, -2 - 0.5)
    assert np.array_equal(m2, np.array([2.25, 1.0], dtype=F))
    assert np.array_equal(w2, np.array([-0.125, -2.5], dtype=F))
    # the planted order (decay first, then clip) would give g = ((4, 3) + 0.25 w) * 0.5 = (2.125, 1.25)
    assert not np.array_equal(m2, np.array([2.125, 1.25], dtype=F))
    # no clipping = the function as it was
    a = optim.optimizer_update("momentum", w, m, None, g, 0.5, p, 0)
    b = optim.optimizer_update("momentum", w, m, None, g, 0.5, p, 0, clip=F(1.0))
    assert all(np.array_equal(x, y) for x, y in zip(a[:2], b[:2]))
