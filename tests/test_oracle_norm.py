"""Pins of the batch-normalisation oracle (paper Sec. 3.3: wide reductions over
FP16 tensors) to closed forms, a library routine, invariants and a numerical
gradient; none of them re-uses the oracle's own formulas."""
import numpy as np

from oracle import norm, fp16

F = np.float32


def test_stats_of_an_integer_ramp_closed_form():
    # values 0..15 repeated: mean 7.5, variance (16^2 - 1) / 12 = 21.25; second channel shifted and doubled
    P = 16 * 40
    x = np.stack([np.arange(P) % 16, 2.0 * (np.arange(P) % 16) + 3.0], axis=1).astype(np.float16)
    mean, var = norm.bn_stats(x)
    assert mean[0] == 7.5 and var[0] == 21.25
    assert mean[1] == 18.0 and var[1] == 85.0


def test_stats_constant_channel_and_library_agreement():
    rng = np.random.default_rng(1)
    x = (rng.standard_normal((1000, 6)) * 3 + 5).astype(np.float16)
    x[:, 2] = np.float16(0.3330078125)
    mean, var = norm.bn_stats(x)
    assert var[2] == 0.0 and mean[2] == float(np.float16(0.3330078125))
    x64 = x.astype(np.float64)
    assert np.allclose(mean, np.mean(x64, axis=0), rtol=1e-14)
    assert np.allclose(var, np.var(x64, axis=0), rtol=1e-12)       # numpy's var is the biased one by default


def test_stats_affine_map():
    rng = np.random.default_rng(2)
    x = rng.integers(-40, 40, (512, 4)).astype(np.float16)
    m1, v1 = norm.bn_stats(x)
    m2, v2 = norm.bn_stats((x.astype(np.float32) * 4 - 8).astype(np.float16))   # exact in FP16
    assert np.allclose(m2, 4 * m1 - 8, rtol=0, atol=1e-12) and np.allclose(v2, 16 * v1, rtol=1e-14)


def test_apply_two_point_channel_is_exactly_plus_minus_one():
    # a channel holding 1 and 3 equally often: mean 2, variance 1; with eps = 0, gamma = 1, beta = 0 -> -1 / +1
    x = np.tile(np.array([[1.0], [3.0]], dtype=np.float16), (8, 1))
    y = norm.bn_apply(x, F([2.0]), F([1.0]), F([1.0]), F([0.0]), 0.0)
    assert np.array_equal(y[:, 0], np.tile(np.array([-1.0, 1.0], dtype=np.float16), 8))
    y = norm.bn_apply(x, F([2.0]), F([1.0]), F([0.5]), F([0.25]), 0.0, relu=True)
    assert np.array_equal(y[:, 0], np.tile(np.array([0.0, 0.75], dtype=np.float16), 8))


def test_apply_output_moments():
    rng = np.random.default_rng(3)
    P, C = 4096, 5
    x = (rng.standard_normal((P, C)) * np.array([0.1, 1, 4, 0.5, 2]) + np.array([0, 3, -2, 10, 0.01])).astype(np.float16)
    mean, var = norm.bn_stats(x)
    gamma, beta = F([1, 2, 0.5, 1.5, 1]), F([0, 1, -1, 0.5, 3])
    eps = 1e-5
    y = norm.bn_apply(x, mean.astype(F), var.astype(F), gamma, beta, eps).astype(np.float64)
    assert np.allclose(y.mean(axis=0), beta, atol=2e-3)                       # FP16 output rounding is the only slack
    assert np.allclose(y.var(axis=0), gamma.astype(np.float64) ** 2 * var / (var + eps), rtol=5e-3)


def _bn_forward_f64(x, gamma, beta, eps):
    mean = x.mean(axis=0)
    var = ((x - mean) ** 2).mean(axis=0)
    return gamma * (x - mean) / np.sqrt(var + eps) + beta


def test_backward_against_numerical_gradient():
    rng = np.random.default_rng(4)
    P, C = 12, 3
    x16 = rng.standard_normal((P, C)).astype(np.float16)
    dy16 = rng.standard_normal((P, C)).astype(np.float16)
    gamma, beta, eps = np.array([1.5, 0.5, 2.0]), np.array([0.1, -0.2, 0.3]), 1e-3
    x, dy = x16.astype(np.float64), dy16.astype(np.float64)
    loss = lambda xx, gg, bb: float((dy * _bn_forward_f64(xx, gg, bb, eps)).sum())
    h = 1e-6
    num_dx = np.zeros_like(x)
    for p in range(P):
        for c in range(C):
            e = np.zeros_like(x); e[p, c] = h
            num_dx[p, c] = (loss(x + e, gamma, beta) - loss(x - e, gamma, beta)) / (2 * h)
    num_dg = np.array([(loss(x, gamma + h * np.eye(C)[c], beta) - loss(x, gamma - h * np.eye(C)[c], beta)) / (2 * h) for c in range(C)])
    num_db = np.array([(loss(x, gamma, beta + h * np.eye(C)[c]) - loss(x, gamma, beta - h * np.eye(C)[c])) / (2 * h) for c in range(C)])
    mean, var = norm.bn_stats(x16)
    dg, db = norm.bn_bwd_reduce(x16, dy16, mean.astype(F), var.astype(F), eps)
    assert np.allclose(dg, num_dg, rtol=1e-5, atol=1e-6) and np.allclose(db, num_db, rtol=1e-6, atol=1e-7)
    dx = norm.bn_bwd_apply(x16, dy16, mean.astype(F), var.astype(F), gamma.astype(F), eps, dg.astype(F), db.astype(F))
    assert np.allclose(dx.astype(np.float64), num_dx, rtol=2e-3, atol=2e-3)   # FP16 store of dx


def test_backward_invariants_and_linearity_in_the_loss_scale():
    rng = np.random.default_rng(5)
    P, C = 2048, 4
    x16 = (rng.standard_normal((P, C)) * 2 + 1).astype(np.float16)
    dy16 = (rng.standard_normal((P, C)) * 2.0 ** -6).astype(np.float16)
    gamma = F([1, 0.5, 2, 1])
    mean, var = norm.bn_stats(x16)
    m32, v32 = mean.astype(F), var.astype(F)
    dg, db = norm.bn_bwd_reduce(x16, dy16, m32, v32, 1e-5)
    dx = norm.bn_bwd_apply(x16, dy16, m32, v32, gamma, 1e-5, dg.astype(F), db.astype(F)).astype(np.float64)
    xhat = (x16.astype(np.float64) - mean) / np.sqrt(var + 1e-5)
    scale = np.abs(dx).sum(axis=0)
    assert (np.abs(dx.sum(axis=0)) <= 2e-3 * scale).all()                      # dx is orthogonal to 1 ...
    assert (np.abs((dx * xhat).sum(axis=0)) <= 2e-3 * scale).all()             # ... and to xhat, per channel
    # a power-of-two loss scale passes through exactly while nothing leaves the FP16 normal range
    S = 64.0
    dyS = (dy16.astype(np.float32) * S).astype(np.float16)
    dgS, dbS = norm.bn_bwd_reduce(x16, dyS, m32, v32, 1e-5)
    assert np.array_equal(dgS, dg * S) and np.array_equal(dbS, db * S)
    dxS = norm.bn_bwd_apply(x16, dyS, m32, v32, gamma, 1e-5, dgS.astype(F), dbS.astype(F)).astype(np.float64)
    normal = np.abs(dx) >= 2.0 ** -14
    exact_inputs = (dg.astype(F).astype(np.float64) * S == dgS.astype(F)) & (db.astype(F).astype(np.float64) * S == dbS.astype(F))
    assert exact_inputs.all()
    assert np.array_equal(dxS[normal], dx[normal] * S)
    assert not (fp16.bits(norm.bn_bwd_apply(x16, dy16, m32, v32, gamma, 1e-5, dg.astype(F), db.astype(F))) == 0x7C00).any()
