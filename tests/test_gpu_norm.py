"""GPU parity of batch normalisation against the oracle, through the C ABI.

Pointwise passes (apply, backward apply): bit-exact FP16 against the oracle's FP32 op-by-op sequence, both sides fed
the same FP32 statistics.  Reductions (statistics, dgamma/dbeta): the kernel sums FP32 chains of at most 16 rows and
everything above that in FP64, so for a channel with addends t_p the sum is within 16 * 2^-24 * sum|t_p| of exact
(plus one rounding for products formed in FP32); the bounds below are that, written out per quantity.
"""
import numpy as np
import pytest
import torch

from oracle import norm, fp16
from paper_1710_03740_amd import binding as mpt
from gpu_util import dev, dev16, host, host16

pytestmark = pytest.mark.gpu
F = np.float32
U32 = 2.0 ** -24
CHAIN = 16


def _ws(P, C):
    return torch.empty(max(mpt.mpt_bn_workspace_bytes(P, C), 16) // 8, dtype=torch.float64, device="cuda")


def _data(P, C, seed, big_mean=False):
    rng = np.random.default_rng(seed)
    std = np.exp2(rng.uniform(-3, 2, C))
    mu = rng.uniform(-2, 2, C) * (50.0 if big_mean else 1.0)
    x = (rng.standard_normal((P, C)) * std + mu).astype(np.float16)
    dy = (np.exp2(rng.uniform(-16, -4, (P, C))) * rng.choice([-1, 1], (P, C))).astype(np.float16)
    gamma = rng.uniform(0.5, 1.5, C).astype(F)
    beta = rng.uniform(-1, 1, C).astype(F)
    return x, dy, gamma, beta


def _check_stats(x, mean_g, var_g):
    mean, var = norm.bn_stats(x)
    x64 = x.astype(np.float64)
    d = x64 - x64[0]                                   # the kernel sums about the channel's first element
    P = x.shape[0]
    e1 = (CHAIN + 1) * U32 * np.abs(d).sum(axis=0) / P
    e2 = (CHAIN + 2) * U32 * (d * d).sum(axis=0) / P
    tol_mean = e1 + U32 * np.abs(mean) + 1e-30
    tol_var = e2 + 2 * np.abs(d.mean(axis=0)) * e1 + e1 * e1 + U32 * var + 1e-30
    assert (np.abs(mean_g.astype(np.float64) - mean) <= tol_mean).all(), np.abs(mean_g - mean).max()
    assert (np.abs(var_g.astype(np.float64) - var) <= tol_var).all(), (np.abs(var_g - var) / tol_var).max()
    # how tight that is in practice: report the worst relative deviations
    return np.abs(mean_g - mean).max(), (np.abs(var_g - var) / np.maximum(var, 1e-30)).max()


SHAPES = [(1, 8), (37, 8), (1000, 64), (4099, 256), (513, 24), (300, 7), (129, 1), (64, 2056), (50, 4100)]


@pytest.mark.parametrize("P,C", SHAPES)
def test_forward_statistics_and_apply(P, C):
    x, _, gamma, beta = _data(P, C, 100 + P + C)
    d_x = dev16(x)
    mean = torch.empty(C, dtype=torch.float32, device="cuda"); var = torch.empty_like(mean)
    mpt.mpt_bn_stats(d_x, mean, var, _ws(P, C))
    mean_g, var_g = host(mean), host(var)
    _check_stats(x, mean_g, var_g)
    for relu in (False, True):
        y = torch.full((P, C), float("nan"), dtype=torch.float16, device="cuda")
        mpt.mpt_bn_apply(d_x, mean, var, dev(gamma), dev(beta), 1e-5, y, relu=relu)
        want = norm.bn_apply(x, mean_g, var_g, gamma, beta, 1e-5, relu=relu)        # same statistics on both sides
        assert np.array_equal(fp16.bits(host16(y)), fp16.bits(want))


def test_statistics_with_mean_far_above_spread_and_constant_channel():
    P, C = 5000, 16
    x, _, _, _ = _data(P, C, 7, big_mean=True)
    x[:, 3] = np.float16(77.25)
    mean = torch.empty(C, dtype=torch.float32, device="cuda"); var = torch.empty_like(mean)
    mpt.mpt_bn_stats(dev16(x), mean, var, _ws(P, C))
    mean_g, var_g = host(mean), host(var)
    _check_stats(x, mean_g, var_g)
    assert var_g[3] == 0.0 and mean_g[3] == 77.25
    m, v = norm.bn_stats(x)
    assert (np.abs(var_g - v) <= 1e-5 * v + 1e-12).all()          # no cancellation although |mean| is ~50x the spread


@pytest.mark.parametrize("P,C", SHAPES)
def test_backward(P, C):
    x, dy, gamma, _ = _data(P, C, 200 + P + C)
    mean64, var64 = norm.bn_stats(x)
    m32, v32 = mean64.astype(F), var64.astype(F)
    eps = 1e-5
    d_x, d_dy, d_m, d_v = dev16(x), dev16(dy), dev(m32), dev(v32)
    dgamma = torch.empty(C, dtype=torch.float32, device="cuda"); dbeta = torch.empty_like(dgamma)
    mpt.mpt_bn_bwd_reduce(d_x, d_dy, d_m, d_v, eps, dgamma, dbeta, _ws(P, C))
    dg, db = norm.bn_bwd_reduce(x, dy, m32, v32, eps)
    dy64 = dy.astype(np.float64)
    with np.errstate(divide="ignore"):
        xhat = (x.astype(np.float64) - m32.astype(np.float64)) * (F(1.0) / np.sqrt(v32 + F(eps))).astype(np.float64)
    tol_b = (CHAIN + 1) * U32 * np.abs(dy64).sum(axis=0) + U32 * np.abs(db) + 1e-30
    tol_g = (CHAIN + 4) * U32 * np.abs(dy64 * xhat).sum(axis=0) + U32 * np.abs(dg) + 1e-30   # + 3 roundings forming dy * xhat
    assert (np.abs(host(dbeta).astype(np.float64) - db) <= tol_b).all()
    assert (np.abs(host(dgamma).astype(np.float64) - dg) <= tol_g).all()
    dx = torch.full((P, C), float("nan"), dtype=torch.float16, device="cuda")
    mpt.mpt_bn_bwd_apply(d_x, d_dy, d_m, d_v, dev(gamma), eps, dgamma, dbeta, dx)
    want = norm.bn_bwd_apply(x, dy, m32, v32, gamma, eps, host(dgamma), host(dbeta))     # the kernel's own sums on both sides
    assert np.array_equal(fp16.bits(host16(dx)), fp16.bits(want))


def test_strided_views_and_reproducibility():
    P, C = 777, 40
    x, dy, gamma, beta = _data(P, C, 9)
    xb = torch.zeros((P, C + 8), dtype=torch.float16, device="cuda"); xb[:, :C] = dev16(x)
    mean = torch.empty(C, dtype=torch.float32, device="cuda"); var = torch.empty_like(mean)
    ws = _ws(P, C)
    mpt.mpt_bn_stats(xb[:, :C], mean, var, ws)
    m1, v1 = host(mean).copy(), host(var).copy()
    _check_stats(x, m1, v1)
    mpt.mpt_bn_stats(xb[:, :C], mean, var, ws)
    assert np.array_equal(m1, host(mean)) and np.array_equal(v1, host(var))
    # an odd column offset forces the scalar path: same contract
    xo = torch.zeros((P, C + 9), dtype=torch.float16, device="cuda"); xo[:, 1:C + 1] = dev16(x)
    mpt.mpt_bn_stats(xo[:, 1:C + 1], mean, var, ws)
    _check_stats(x, host(mean), host(var))
    yb = torch.full((P, C + 9), 5.0, dtype=torch.float16, device="cuda")
    mpt.mpt_bn_apply(xo[:, 1:C + 1], mean, var, dev(gamma), dev(beta), 1e-3, yb[:, 1:C + 1])
    out = host16(yb)
    want = norm.bn_apply(x, host(mean), host(var), gamma, beta, 1e-3)
    assert np.array_equal(fp16.bits(np.ascontiguousarray(out[:, 1:C + 1])), fp16.bits(want))
    assert (out[:, 0] == 5.0).all() and (out[:, C + 1:] == 5.0).all()


def test_conv_block_activation_shape():
    """The activation of the convolution workload: 256 x 14 x 14 positions, 256 channels, ReLU-like input."""
    P, C = 256 * 14 * 14, 256
    rng = np.random.default_rng(44)
    x = np.maximum(rng.standard_normal((P, C)) * 0.7 + 0.2, 0).astype(np.float16)
    mean = torch.empty(C, dtype=torch.float32, device="cuda"); var = torch.empty_like(mean)
    mpt.mpt_bn_stats(dev16(x), mean, var, _ws(P, C))
    dm, dv = _check_stats(x, host(mean), host(var))
    assert dm < 1e-6 and dv < 1e-5


def test_tensor_beyond_the_memory_side_cache():
    """205 MB activation (first-stage ResNet size, 256 x 56 x 56 positions x 128 channels): the streamed variants of
    all four kernels.  Statistics against the oracle in full; pointwise outputs bit-exact on every 997th row."""
    P, C = 256 * 56 * 56, 128
    rng = np.random.default_rng(12)
    x = (rng.standard_normal((P, C), dtype=np.float32) * 0.7 + 0.2).astype(np.float16)
    dy = (rng.standard_normal((P, C), dtype=np.float32) * 2.0 ** -7).astype(np.float16)
    gamma = rng.uniform(0.5, 1.5, C).astype(F); beta = rng.uniform(-1, 1, C).astype(F)
    d_x, d_dy = dev16(x), dev16(dy)
    mean = torch.empty(C, dtype=torch.float32, device="cuda"); var = torch.empty_like(mean)
    ws = _ws(P, C)
    mpt.mpt_bn_stats(d_x, mean, var, ws)
    m32, v32 = host(mean), host(var)
    dm, dv = _check_stats(x, m32, v32)
    assert dm < 1e-6 and dv < 1e-5
    rows = np.arange(0, P, 997)
    y = torch.empty_like(d_x)
    mpt.mpt_bn_apply(d_x, mean, var, dev(gamma), dev(beta), 1e-5, y, relu=True)
    want = norm.bn_apply(x[rows], m32, v32, gamma, beta, 1e-5, relu=True)
    assert np.array_equal(fp16.bits(host16(y[torch.from_numpy(rows).cuda()])), fp16.bits(want))
    dgamma = torch.empty(C, dtype=torch.float32, device="cuda"); dbeta = torch.empty_like(dgamma)
    mpt.mpt_bn_bwd_reduce(d_x, d_dy, mean, var, 1e-5, dgamma, dbeta, ws)
    dg, db = norm.bn_bwd_reduce(x, dy, m32, v32, 1e-5)
    dy64 = dy.astype(np.float64)
    assert (np.abs(host(dbeta) - db) <= (CHAIN + 1) * U32 * np.abs(dy64).sum(axis=0) + U32 * np.abs(db)).all()
    xhat = (x.astype(np.float64) - m32.astype(np.float64)) * (F(1.0) / np.sqrt(v32 + F(1e-5))).astype(np.float64)
    assert (np.abs(host(dgamma) - dg) <= (CHAIN + 4) * U32 * np.abs(dy64 * xhat).sum(axis=0) + U32 * np.abs(dg)).all()
    del xhat, dy64
    dx = torch.empty_like(d_x)
    mpt.mpt_bn_bwd_apply(d_x, d_dy, mean, var, dev(gamma), 1e-5, dgamma, dbeta, dx)
    # the oracle's pointwise formula takes P from the row count: give it the sampled rows but the full P
    Pf = F(P)
    invstd = F(1.0) / np.sqrt(v32 + F(1e-5))
    a = gamma * invstd; b = host(dbeta) / Pf; g = host(dgamma) / Pf
    t = (dy[rows].astype(F) - b) - ((x[rows].astype(F) - m32) * invstd) * g
    want = fp16.rne16((a * t).astype(np.float64))
    assert np.array_equal(fp16.bits(host16(dx[torch.from_numpy(rows).cuda()])), fp16.bits(want))
