"""GPU parity of the Nesterov / Adagrad / Adam master updates and of the gradient statistics, through the C ABI.
Updates: bit-exact FP32 masters and state, bit-exact FP16 copies, against the oracle's op-by-op FP32 sequence.
Statistics: integer counts and a bit pattern, bit-exact."""
import numpy as np
import pytest
import torch

import workloads
from oracle import optim, gradstats, fp16, update
from paper_1710_03740_amd import binding as mpt
from gpu_util import dev, dev16, host, host16

pytestmark = pytest.mark.gpu
F = np.float32


def _hp(p):
    return mpt.mpt_opt_params(p.lr, p.momentum, p.beta2, p.eps, p.weight_decay, p.one_minus_beta1, p.one_minus_beta2, p.bias_corr1, p.bias_corr2)


def _params(kind, step, wd):
    if kind == "adam":
        return optim.adam_params(1e-3, 0.9, 0.999, 1e-8, step, wd)
    return optim.OptParams(lr=1e-2, momentum=0.9, eps=1e-7, weight_decay=wd)


def _eq32(t, ref):
    return np.array_equal(host(t).view(np.uint32), np.asarray(ref, dtype=F).view(np.uint32))


@pytest.mark.parametrize("kind", optim.KINDS)
@pytest.mark.parametrize("n", [1, 2, 7, 4096, 100003])
def test_steps_bit_exact(kind, n):
    rng = np.random.default_rng(n * 13 + len(kind))
    w = rng.uniform(-0.5, 0.5, n).astype(F)
    s1 = np.zeros(n, F); s2 = np.zeros(n, F) if kind == "adam" else None
    h = fp16.rne16(w.astype(np.float64))
    d_w, d_1, d_h = dev(w), dev(s1), dev16(h)
    d_2 = dev(s2) if s2 is not None else None
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    S = 2.0 ** 9
    for step in range(1, 6):
        g = (np.exp2(rng.uniform(-18, 1, n)) * rng.choice([-1, 1], n) * S).astype(np.float16)
        if step == 3:
            g[n // 2] = np.inf                                   # an overflowing step: everything must stay put
        p = _params(kind, step, 1e-4 if step % 2 == 0 else 0.0)
        fl = update.overflow_flag(g)
        w, s1, s2, h = optim.optimizer_update(kind, w, s1, s2, g, 1.0 / S, p, fl, w16=h)
        d_g = dev16(g)
        flag.zero_()
        mpt.mpt_unscale_check(d_g, 1.0 / S, flag)
        assert int(flag.item()) == fl
        mpt.mpt_optimizer_update(kind, _hp(p), d_w, d_1, d_2, d_g, d_h, 1.0 / S, flag)
        assert _eq32(d_w, w) and _eq32(d_1, s1), (kind, n, step)
        if s2 is not None:
            assert _eq32(d_2, s2)
        assert np.array_equal(fp16.bits(host16(d_h)), fp16.bits(h))


@pytest.mark.parametrize("kind", ["nesterov", "adam"])
def test_fp32_gradients_device_scale_and_unaligned_views(kind):
    n = 5001
    rng = np.random.default_rng(3)
    w = rng.uniform(-0.5, 0.5, n + 1).astype(F); s1 = rng.standard_normal(n + 1).astype(F) * F(0.01)
    s2 = np.abs(rng.standard_normal(n + 1)).astype(F) * F(1e-4)
    g32 = (rng.standard_normal(n + 1) * 3).astype(F)
    p = _params(kind, 4, 1e-5)
    sc = mpt.mpt_scaler_init(256.0, 1000)
    d_sc = mpt.scaler_to_device(sc)
    # views starting at element 1: FP32 arrays only 4-byte aligned, FP16 copy only 2-byte aligned -> element-wise path
    d_w, d_1, d_2, d_g = dev(w), dev(s1), dev(s2), dev(g32)
    d_h = torch.zeros(n + 1, dtype=torch.float16, device="cuda")
    mpt.mpt_optimizer_update(kind, _hp(p), d_w[1:], d_1[1:], d_2[1:] if kind == "adam" else None, d_g[1:], d_h[1:], 123.0, None, scaler_dev=d_sc)
    rw, r1, r2, rh = optim.optimizer_update(kind, w[1:], s1[1:], s2[1:] if kind == "adam" else None, g32[1:], 1.0 / 256.0, p, 0)
    assert _eq32(d_w[1:], rw) and _eq32(d_1[1:], r1) and np.array_equal(fp16.bits(host16(d_h[1:])), fp16.bits(rh))
    assert host(d_w)[0] == w[0] and host16(d_h)[0] == 0          # the element before the view is untouched
    if kind == "adam":
        assert _eq32(d_2[1:], r2)


def test_adam_on_the_flat_parameter_buffer_sampled():
    """116M elements (the update workload's size): one Adam step, checked bit-exactly on strided samples and the ends."""
    n = 116_000_000
    fu = workloads.FlatUpdate(n, steps=2, n_inject=0)
    S = 2.0 ** 16
    g = fu.grad16(0, S)
    w = fu.w32
    s1 = np.zeros(n, F); s2 = np.zeros(n, F)
    p = optim.adam_params(1e-3, 0.9, 0.999, 1e-8, 1)
    d_w, d_1, d_2, d_g = dev(w), dev(s1), dev(s2), dev16(g)
    d_h = torch.zeros(n, dtype=torch.float16, device="cuda")
    mpt.mpt_optimizer_update("adam", _hp(p), d_w, d_1, d_2, d_g, d_h, 1.0 / S, None)
    idx = np.unique(np.concatenate([np.arange(0, n, 9973), np.arange(0, 4096), np.arange(n - 4096, n)]))
    rw, r1, r2, rh = optim.optimizer_update("adam", w[idx], s1[idx], s2[idx], g[idx], 1.0 / S, p, 0)
    t = torch.from_numpy(idx).cuda()
    assert _eq32(d_w[t], rw) and _eq32(d_1[t], r1) and _eq32(d_2[t], r2)
    assert np.array_equal(fp16.bits(host16(d_h[t])), fp16.bits(rh))


@pytest.mark.parametrize("n", [0, 1, 7, 8, 1000, 65536 + 3, 3_000_001])
def test_gradient_statistics_bit_exact(n):
    rng = np.random.default_rng(n + 5)
    with np.errstate(over="ignore"):                              # values beyond 65504 become Inf on purpose
        g = (np.exp2(rng.uniform(-30, 17, n)) * rng.choice([-1, 1], n)).astype(np.float16)
    if n > 100:
        g[5] = np.nan; g[n - 1] = -np.inf; g[17] = 0.0; g[18] = -0.0
    hist = torch.full((42,), 7, dtype=torch.int64, device="cuda")
    amax = torch.full((1,), 9, dtype=torch.int32, device="cuda")
    d_g = dev16(g) if n else torch.zeros(0, dtype=torch.float16, device="cuda")
    mpt.mpt_grad_stats(d_g, hist, amax)
    want = gradstats.exponent_histogram(g)
    assert np.array_equal(host(hist), want)
    am = gradstats.absmax(g)
    assert int(amax.item()) == int(fp16.bits(np.array([am], dtype=np.float16))[0])
    if n > 8:
        # accumulate a second buffer (an odd-offset view: element-wise path) into the same histogram
        mpt.mpt_grad_stats(d_g[1:], hist, amax, accumulate=True)
        assert np.array_equal(host(hist), want + gradstats.exponent_histogram(g[1:]))
        k = mpt.mpt_suggest_loss_scale_log2(int(amax.item()), -99)
        assert k == max(-24, min(40, gradstats.suggest_scale_log2(am)))


def test_all_fp16_patterns_census_on_device():
    allv = np.arange(65536, dtype=np.uint16).view(np.float16)
    hist = torch.zeros(42, dtype=torch.int64, device="cuda"); amax = torch.zeros(1, dtype=torch.int32, device="cuda")
    mpt.mpt_grad_stats(dev16(allv), hist, amax)
    assert np.array_equal(host(hist), gradstats.exponent_histogram(allv)) and int(amax.item()) == 0x7BFF
