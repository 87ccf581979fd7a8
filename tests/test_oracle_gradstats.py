"""Pins of the gradient-statistics oracle: the exhaustive FP16 census has a closed form, a library routine (frexp)
gives the same bins, and the scale rule is checked on the paper's bound (Sec. 3.2: scale * max below 65504)."""
import numpy as np

from oracle import gradstats, fp16


def test_census_of_all_fp16_patterns():
    allv = np.arange(65536, dtype=np.uint16).view(np.float16)
    h = gradstats.exponent_histogram(allv)
    assert h.sum() == 65536 and h[0] == 2 and h[41] == 2 * 1024
    for k in range(10):                       # subnormals: leading bit k -> 2^k patterns per sign, exponent -24 + k
        assert h[1 + k] == 2 * 2 ** k
    for e in range(-14, 16):                  # normals: 1024 mantissas per sign
        assert h[1 + e + 24] == 2048
    assert gradstats.absmax(allv) == 65504.0


def test_bins_agree_with_frexp_and_named_values():
    rng = np.random.default_rng(0)
    with np.errstate(over="ignore"):
        g = (np.exp2(rng.uniform(-30, 17, 50000)) * rng.choice([-1, 1], 50000)).astype(np.float16)
    h = gradstats.exponent_histogram(g)
    f = g.astype(np.float64); fin = np.isfinite(f) & (f != 0)
    _, ex = np.frexp(np.abs(f[fin]))          # |x| = m * 2^ex with m in [0.5, 1): floor(log2) = ex - 1
    want = np.bincount(ex - 1 + 24 + 1, minlength=42)
    want[0] = int((f == 0).sum()); want[41] = int((~np.isfinite(f)).sum())
    assert np.array_equal(h, want) and h[0] > 0 and h[41] > 0
    one = lambda v: int(np.argmax(gradstats.exponent_histogram(np.array([v], dtype=np.float16))))
    assert one(2.0 ** -24) == 1 and one(2.0 ** -14) == 11 and one(1.0) == 25 and one(1.5) == 25 and one(65504.0) == 40
    assert one(0.0) == 0 and one(np.inf) == 41 and one(np.nan) == 41


def test_scale_rule():
    assert gradstats.suggest_scale_log2(1.0) == 15            # 32768 <= 65504 < 65536
    assert gradstats.suggest_scale_log2(65504.0) == 0
    assert gradstats.suggest_scale_log2(2.0 ** -24) == 39
    assert gradstats.suggest_scale_log2(2.0) == 14 and gradstats.suggest_scale_log2(1.999) == 15 and gradstats.suggest_scale_log2(0.999) == 16
    assert gradstats.suggest_scale_log2(0.0) is None
    for a in (3.1e-5, 0.37, 12.0, 40000.0):
        k = gradstats.suggest_scale_log2(a)
        assert 2.0 ** k * a <= 65504.0 < 2.0 ** (k + 1) * a
