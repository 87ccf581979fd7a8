"""Pins of the optimizer oracle (paper Sec. 4 names the optimizers; Sec. 3.1 / 3.2 fix where they sit): closed
forms on exactly representable values, reductions to the already pinned momentum step, agreement with a wide
evaluation, and planted mistakes."""
import numpy as np
import pytest

from oracle import optim, update, fp16

F = np.float32


def _rand(n, seed):
    rng = np.random.default_rng(seed)
    w = rng.uniform(-0.5, 0.5, n).astype(F)
    g = (np.exp2(rng.uniform(-14, 2, n)) * rng.choice([-1, 1], n)).astype(np.float16)
    return rng, w, g


def test_momentum_kind_is_the_pinned_master_update():
    rng, w, g = _rand(4096, 1)
    m = rng.standard_normal(4096).astype(F) * F(0.01)
    p = optim.OptParams(lr=0.01, momentum=0.9)
    w2, m2, _, h2 = optim.optimizer_update("momentum", w, m, None, g, 2.0 ** -10, p, 0)
    rw, rm, rh = update.master_update(w, m, g, 2.0 ** -10, 0.01, 0.9, 0)
    assert np.array_equal(w2.view(np.uint32), rw.view(np.uint32)) and np.array_equal(m2.view(np.uint32), rm.view(np.uint32))
    assert np.array_equal(fp16.bits(h2), fp16.bits(rh))


def test_nesterov_closed_form_and_zero_momentum():
    # constant g = 1, mu = 1/2, lr = 2^-6, S = 1: m_t = 2 - 2^(1-t); step_t = lr * (1 + m_t / 2) = lr * (2 - 2^-t)
    w = np.array([1.0], dtype=F); m = np.zeros(1, dtype=F)
    g = np.array([1.0], dtype=np.float16)
    p = optim.OptParams(lr=2.0 ** -6, momentum=0.5)
    total = 0.0
    for t in range(1, 11):
        w, m, _, h = optim.optimizer_update("nesterov", w, m, None, g, 1.0, p, 0)
        total += 2.0 ** -6 * (2.0 - 2.0 ** -t)
        assert float(m[0]) == 2.0 - 2.0 ** (1 - t)
        assert float(w[0]) == 1.0 - total                       # everything here is exact in FP32
    assert float(fp16.to_f64(h)[0]) == float(np.float16(w[0]))
    # mu = 0: the look-ahead term vanishes and the step is plain SGD
    rng, w, g = _rand(1000, 2)
    p0 = optim.OptParams(lr=0.05, momentum=0.0)
    a = optim.optimizer_update("nesterov", w, np.zeros(1000, F), None, g, 0.25, p0, 0)
    b = update.master_update(w, None, g, 0.25, 0.05, 0.0, 0)
    assert np.array_equal(a[0].view(np.uint32), b[0].view(np.uint32))


def test_adagrad_exact_steps_on_perfect_squares():
    # h: 0 -> 9 -> 25 with g = 3 then 4; eps = 0, lr = 2^-4: steps lr*3/3 = lr, then lr*4/5
    w = np.array([1.0], dtype=F); h = np.zeros(1, dtype=F)
    p = optim.OptParams(lr=2.0 ** -4, eps=0.0)
    w, h, _, _ = optim.optimizer_update("adagrad", w, h, None, np.array([3.0], np.float16), 1.0, p, 0)
    assert float(h[0]) == 9.0 and float(w[0]) == 1.0 - 2.0 ** -4
    w, h, _, _ = optim.optimizer_update("adagrad", w, h, None, np.array([-4.0], np.float16), 1.0, p, 0)
    assert float(h[0]) == 25.0
    assert float(w[0]) == float(F(F(1.0 - 2.0 ** -4) + F(F(0.25) / F(5.0))))      # 0.25 / 5 rounded, then added
    # the loss scale is removed before squaring: S = 1024 on the gradient, 1/S on the way in
    w3, h3, _, _ = optim.optimizer_update("adagrad", np.array([1.0], F), np.zeros(1, F), None, np.array([3072.0], np.float16), 2.0 ** -10, p, 0)
    assert float(h3[0]) == 9.0 and float(w3[0]) == 1.0 - 2.0 ** -4


def test_adam_first_step_has_magnitude_lr():
    # beta1 = 1/2, beta2 = 3/4: at t = 1 the bias corrections cancel the (1 - beta) factors exactly, so
    # m_hat = g, v_hat = g^2 (exact for FP16 gradients), and with eps = 0 the step is lr * sign(g) whatever |g| is.
    rng, w, g = _rand(2000, 3)
    p = optim.adam_params(lr=2.0 ** -8, beta1=0.5, beta2=0.75, eps=0.0, step=1)
    assert p.bias_corr1 == 0.5 and p.bias_corr2 == 0.25
    w2, m2, v2, _ = optim.optimizer_update("adam", w, np.zeros(2000, F), np.zeros(2000, F), g, 1.0, p, 0)
    gf = g.astype(np.float64)
    assert np.array_equal(m2.astype(np.float64), 0.5 * gf) and np.array_equal(v2.astype(np.float64), 0.25 * gf * gf)
    assert np.array_equal(w2, (w - F(2.0 ** -8) * np.sign(gf).astype(F)).astype(F))


@pytest.mark.parametrize("kind", optim.KINDS)
def test_agreement_with_wide_evaluation_and_weight_decay(kind):
    rng, w, g = _rand(20000, 4)
    s1 = np.abs(rng.standard_normal(20000)).astype(F) * F(0.01)
    s2 = np.abs(rng.standard_normal(20000)).astype(F) * F(1e-4) if kind == "adam" else None
    for wd in (0.0, 1e-4):
        p = optim.adam_params(1e-3, 0.9, 0.999, 1e-8, 7, wd) if kind == "adam" else optim.OptParams(lr=1e-2, momentum=0.9, eps=1e-7, weight_decay=wd)
        w2, a2, b2, h2 = optim.optimizer_update(kind, w, s1, s2, g, 2.0 ** -7, p, 0)
        ww, aw, bw = optim.optimizer_update_wide(kind, w, s1, s2, g, 2.0 ** -7, p)
        ulp_w = np.spacing(np.abs(w2).astype(F)).astype(np.float64)
        assert (np.abs(w2.astype(np.float64) - ww) <= 1.0 * ulp_w + 8 * 2.0 ** -24 * np.abs(ww - w.astype(np.float64))).all()
        gu = np.abs(g.astype(np.float64)) * 2.0 ** -7 + wd * np.abs(w.astype(np.float64))     # |unscaled gradient|, an upper bound
        terms = np.abs(s1.astype(np.float64)) + gu + gu * gu                                       # magnitudes entering the state update
        assert (np.abs(a2.astype(np.float64) - aw) <= 4 * 2.0 ** -24 * terms).all()
        if b2 is not None:
            assert (np.abs(b2.astype(np.float64) - bw) <= 4 * 2.0 ** -24 * (np.abs(s2.astype(np.float64)) + gu * gu)).all()
        assert np.array_equal(fp16.bits(h2), fp16.bits(fp16.rne16(w2.astype(np.float64))))
    # weight decay acts on the unscaled gradient: w = 1, g = 0, wd = 1/4 -> effective gradient 1/4
    p = optim.OptParams(lr=0.5, momentum=0.0, weight_decay=0.25)
    w2, _, _, _ = optim.optimizer_update("momentum", np.ones(1, F), np.zeros(1, F), None, np.zeros(1, np.float16), 2.0 ** -10, p, 0)
    assert float(w2[0]) == 1.0 - 0.5 * 0.25


@pytest.mark.parametrize("kind", optim.KINDS)
def test_skipped_step_changes_nothing(kind):
    rng, w, g = _rand(100, 5)
    g[7] = np.inf
    s1 = rng.standard_normal(100).astype(F); s2 = np.abs(rng.standard_normal(100)).astype(F)
    h = fp16.rne16(w.astype(np.float64))
    p = optim.adam_params(1e-3, 0.9, 0.999, 1e-8, 3)
    w2, a2, b2, h2 = optim.optimizer_update(kind, w, s1, s2 if kind == "adam" else None, g, 1.0, p, update.overflow_flag(g), w16=h)
    assert np.array_equal(w2.view(np.uint32), w.view(np.uint32)) and np.array_equal(a2.view(np.uint32), s1.view(np.uint32))
    assert np.array_equal(fp16.bits(h2), fp16.bits(h))
    if kind == "adam":
        assert np.array_equal(b2.view(np.uint32), s2.view(np.uint32))


def test_planted_mistakes_are_caught():
    """A dropped look-ahead term, a missing bias correction, squaring before unscaling: each fails a pin above."""
    w = np.array([1.0], dtype=F); g = np.array([1.0], np.float16)
    p = optim.OptParams(lr=2.0 ** -6, momentum=0.5)
    w_n, m_n, _, _ = optim.optimizer_update("nesterov", w, np.ones(1, F), None, g, 1.0, p, 0)
    w_m, _, _, _ = optim.optimizer_update("momentum", w, np.ones(1, F), None, g, 1.0, p, 0)
    assert float(w_n[0]) != float(w_m[0])                       # the look-ahead term matters
    pa = optim.adam_params(2.0 ** -8, 0.5, 0.75, 0.0, 1)
    pb = optim.OptParams(**{**pa.__dict__, "bias_corr1": 1.0})
    a = optim.optimizer_update("adam", w, np.zeros(1, F), np.zeros(1, F), g, 1.0, pa, 0)[0]
    b = optim.optimizer_update("adam", w, np.zeros(1, F), np.zeros(1, F), g, 1.0, pb, 0)[0]
    assert float(a[0]) == 1.0 - 2.0 ** -8 and float(b[0]) != float(a[0])
