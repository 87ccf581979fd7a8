"""Pins for the unscale/check/update path: the paper's two failure modes of
FP16-only updates (Sec. 3.1), exact power-of-two unscaling (Sec. 3.2), the
overflow truth table and skip rule (Sec. 3.2), and arithmetic cross-checks."""
import numpy as np
import pytest

from oracle import fp16, update

F32 = np.float32


def h(*v):
    return np.array(v, dtype=np.float16)


# ---- Sec. 3.1, first reason: the update itself underflows in FP16
def test_small_update_vanishes_in_fp16_but_not_in_fp32_master():
    g = h(2.0 ** -16)
    lr = 2.0 ** -10                                   # lr*g = 2^-26 < 2^-25
    w16 = h(0.0)
    assert fp16.bits(update.fp16_only_update(w16, g, lr))[0] in (0x0000, 0x8000)
    w, _, _ = update.master_update(F32([0.0]), None, g, 1.0, lr, 0.0, 0)
    assert w[0] == F32(-2.0 ** -26)


# ---- Sec. 3.1, second reason: weight/update ratio of 2048 and beyond
def test_swamping_closed_forms():
    one = h(1.0)
    assert update.fp16_only_update(one, h(-2.0 ** -12), 1.0)[0] == 1.0        # ratio 4096: always lost
    assert update.fp16_only_update(one, h(-2.0 ** -11), 1.0)[0] == 1.0        # ratio 2048, tie to even: lost
    odd = h(1.0 + 2.0 ** -10)
    got = update.fp16_only_update(odd, h(-2.0 ** -11), 1.0)[0]
    assert got == np.float16(1.0 + 2.0 ** -9)                                  # tie rounds up: "rounding can recover"
    assert update.fp16_only_update(one, h(-2.0 ** -10), 1.0)[0] == np.float16(1.0 + 2.0 ** -10)


def test_4096_tiny_updates_master_reaches_two_fp16_stays_one():
    w16 = h(1.0)
    w32 = F32([1.0])
    g = h(-2.0 ** -12)
    for _ in range(4096):
        w16 = update.fp16_only_update(w16, g, 1.0)
        w32, _, copy16 = update.master_update(w32, None, g, 1.0, 1.0, 0.0, 0)
    assert w16[0] == 1.0
    assert w32[0] == 2.0 and copy16[0] == 2.0


# ---- Sec. 3.2: unscaling by a power of two is exact
def test_unscale_round_trip_exact_for_normals():
    allb = np.arange(0x0400, 0x7C00, dtype=np.uint16)
    x = fp16.bits_to_f64(allb)
    for S in (8.0, 128.0, 1024.0, 8192.0, 65536.0):
        ok = x * S <= 65504
        g16 = fp16.rne16(x[ok] * S)
        g32, flag = update.unscale_check(g16, F32(1.0 / S))
        assert flag == 0
        assert np.array_equal(g32.astype(np.float64), x[ok])


def test_flush_without_scale_survive_with_scale():
    true = np.exp2(np.arange(-27.0, -24.0))           # the band the paper says scale 8 rescued
    assert not fp16.rne16(true).view(np.uint16).any()
    g16 = fp16.rne16(true * 8)
    g32, _ = update.unscale_check(g16, F32(1 / 8))
    assert np.array_equal(g32.astype(np.float64), true)


# ---- Sec. 3.2: overflow detection and skip
@pytest.mark.parametrize("pattern", [0x7C00, 0xFC00, 0x7E00, 0x7C01, 0xFFFF])
@pytest.mark.parametrize("pos", [0, 5, 10])
def test_flag_truth_table(pattern, pos):
    g = np.zeros(11, dtype=np.float16)
    g[3] = 65504.0
    assert update.unscale_check(g, 1.0)[1] == 0
    g.view(np.uint16)[pos] = pattern
    assert update.unscale_check(g, 1.0)[1] == 1


def test_flag_fp32_storage():
    g = F32([1.0, 3.4e38, -0.0])
    assert update.overflow_flag(g) == 0
    for bad in (np.inf, -np.inf, np.nan):
        g2 = g.copy(); g2[2] = bad
        assert update.overflow_flag(g2) == 1


def test_natural_overflow_sets_flag():
    g16 = fp16.rne16(np.array([3.0 * 32768.0]))        # scaled value past 65520 -> Inf
    assert update.unscale_check(g16, F32(2.0 ** -15))[1] == 1


def test_skip_leaves_everything_bit_identical():
    rng = np.random.default_rng(0)
    w = rng.standard_normal(100).astype(F32)
    m = rng.standard_normal(100).astype(F32)
    w16 = fp16.rne16(w.astype(np.float64))
    w16.view(np.uint16)[7] ^= 1                        # a stale copy must not be refreshed either
    g = rng.standard_normal(100).astype(np.float16)
    wn, mn, hn = update.master_update(w, m, g, 0.5, 0.1, 0.9, 1, w16)
    assert np.array_equal(wn.view(np.uint32), w.view(np.uint32))
    assert np.array_equal(mn.view(np.uint32), m.view(np.uint32))
    assert np.array_equal(fp16.bits(hn), fp16.bits(w16))


# ---- arithmetic cross-checks
def test_zero_momentum_reduces_to_plain_sgd():
    rng = np.random.default_rng(1)
    w = rng.standard_normal(1000).astype(F32)
    g = (rng.standard_normal(1000) * 4).astype(np.float16)
    a, _, a16 = update.master_update(w, None, g, 0.25, 0.01, 0.0, 0)
    b, mb, b16 = update.master_update(w, np.zeros(1000, F32), g, 0.25, 0.01, 0.0, 0)
    assert np.array_equal(a, b) and np.array_equal(fp16.bits(a16), fp16.bits(b16))
    assert np.array_equal(mb, g.astype(F32) * F32(0.25))


def test_hand_computed_step():
    # w=1, m=0.5, g16=4 (S=8 -> g=0.5), mu=0.5, lr=0.25: m'=0.75, w'=0.8125
    w, m, w16 = update.master_update(F32([1.0]), F32([0.5]), h(4.0), 0.125, 0.25, 0.5, 0)
    assert m[0] == 0.75 and w[0] == 0.8125 and w16[0] == np.float16(0.8125)
    # sign of the step: positive gradient lowers the weight
    w, _, _ = update.master_update(F32([1.0]), None, h(1.0), 1.0, 0.5, 0.0, 0)
    assert w[0] == 0.5


def test_each_operation_is_rounded_separately():
    """A fused multiply-add would give a different master on these operands:
    lr*g is inexact in FP32 and the subtraction exposes its rounding."""
    lr = F32(0.1)
    g = F32(3.0)
    t = F32(lr * g)                                    # rounded product
    w0 = t                                             # w - t == 0 exactly when rounded separately
    w, _, _ = update.master_update(F32([w0]), None, h(3.0), 1.0, 0.1, 0.0, 0)
    assert w[0] == 0.0
    fused = F32(np.float64(w0) - np.float64(lr) * np.float64(g))
    assert fused != 0.0


def test_within_one_ulp_of_wide_reference():
    rng = np.random.default_rng(3)
    n = 200000
    w = rng.uniform(-0.05, 0.05, n).astype(F32)
    m = (rng.standard_normal(n) * 1e-3).astype(F32)
    g = (np.exp2(rng.uniform(-12, 4, n)) * np.sign(m)).astype(np.float16)   # same sign: no cancellation in mu*m + g
    wn, mn, _ = update.master_update(w, m, g, 2.0 ** -16, 1e-3, 0.9, 0)
    ww, mw = update.master_update_wide(w, m, g, 2.0 ** -16, 1e-3, 0.9)
    assert fp16.ulpdist32(mn, mw).max() <= 1
    assert fp16.ulpdist32(wn, ww).max() <= 1


def test_fp16_copy_is_rne_of_master():
    rng = np.random.default_rng(4)
    w = rng.uniform(-1, 1, 50000).astype(F32)
    g = rng.standard_normal(50000).astype(np.float16)
    wn, _, w16 = update.master_update(w, None, g, 1.0, 0.01, 0.0, 0)
    assert np.array_equal(fp16.bits(w16), wn.astype(np.float16).view(np.uint16))


def test_fp32_gradient_input():
    w, _, _ = update.master_update(F32([1.0]), None, F32([2.0 ** -30 * 1024]), 2.0 ** -10, 1.0, 0.0, 0)
    assert w[0] == F32(1.0) - F32(2.0 ** -30) or w[0] == F32(1.0)
    w, _, _ = update.master_update(F32([0.0]), None, F32([2.0 ** -30 * 1024]), 2.0 ** -10, 1.0, 0.0, 0)
    assert w[0] == -F32(2.0 ** -30)


def test_single_pass_form_is_check_plus_unconditional_update():
    """master_update_fused: flag of the stored gradient; outputs of the step as if taken.  Pinned to the two parts it is
    made of (each pinned above) and to hand values: w = 1, g = 2^-3 * S, lr = 0.5 -> 1 - 2^-4 exactly; an Inf anywhere
    raises the flag and leaves the inputs alone."""
    S = 1024.0
    w = np.array([1.0, -2.0, 0.5], dtype=np.float32)
    m = np.zeros(3, dtype=np.float32)
    g = (np.array([2.0 ** -3, 0.0, -2.0 ** -5]) * S).astype(np.float16)
    flag, w2, m2, h2 = update.master_update_fused(w, m, g, 1.0 / S, 0.5, 0.9)
    assert flag == 0
    assert np.array_equal(m2, np.array([2.0 ** -3, 0.0, -2.0 ** -5], dtype=np.float32))
    assert np.array_equal(w2, np.array([1.0 - 2.0 ** -4, -2.0, 0.5 + 2.0 ** -6], dtype=np.float32))
    assert np.array_equal(fp16.bits(h2), fp16.bits(w2.astype(np.float16)))
    wa, ma, ha = update.master_update(w, m, g, 1.0 / S, 0.5, 0.9, update.unscale_check(g, 1.0 / S)[1])
    assert np.array_equal(wa, w2) and np.array_equal(ma, m2) and np.array_equal(fp16.bits(ha), fp16.bits(h2))
    g_bad = g.copy(); g_bad[1] = np.float16(np.inf)
    w_keep, m_keep = w.copy(), m.copy()
    flag, _, _, _ = update.master_update_fused(w, m, g_bad, 1.0 / S, 0.5, 0.9)
    assert flag == 1 and np.array_equal(w, w_keep) and np.array_equal(m, m_keep)
    assert update.master_update_fused(w, None, g, 1.0 / S, 0.5, 0.0)[2] is None
