"""Pins for the oracle's binary16 conversion: the paper's printed facts, an
exhaustive round trip, and two independent library casts (numpy, torch)."""
import os

import numpy as np
import torch

from oracle import fp16

HERE = os.path.dirname(os.path.abspath(__file__))


def test_golden_paper_facts():
    n = 0
    for line in open(os.path.join(HERE, "golden", "fp16_facts.txt")):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        x, want = line.split()[:2]
        got = int(fp16.rne16_bits(np.array([float.fromhex(x)]))[0])
        assert got == int(want, 16), line
        gotn = int(fp16.rne16_bits(np.array([-float.fromhex(x)]))[0])
        assert gotn == (int(want, 16) | 0x8000), line
        n += 1
    assert n >= 10


def test_max_and_overflow_boundary():
    r = lambda v: int(fp16.rne16_bits(np.array([v], dtype=np.float64))[0])
    assert r(65504.0) == 0x7BFF
    assert r(65519.99) == 0x7BFF          # still rounds down to the maximum
    assert r(np.nextafter(65520.0, 0)) == 0x7BFF
    assert r(65520.0) == 0x7C00           # tie to even -> Inf, no clamping
    assert r(1e30) == 0x7C00 and r(-1e30) == 0xFC00
    assert r(np.inf) == 0x7C00 and r(-np.inf) == 0xFC00
    assert (r(np.nan) & 0x7FFF) > 0x7C00


def test_underflow_band():
    r = lambda v: int(fp16.rne16_bits(np.array([v], dtype=np.float64))[0])
    assert r(2.0 ** -24) == 1
    assert r(2.0 ** -25) == 0                              # exact tie -> even (zero)
    assert r(np.nextafter(2.0 ** -25, 1)) == 1             # IEEE reading of the open band
    assert r(1.5 * 2.0 ** -24) == 2                        # tie -> even
    assert r(2.5 * 2.0 ** -24) == 2
    assert r(2.0 ** -14) == 0x0400
    assert r(2.0 ** -14 - 2.0 ** -25) == 0x0400            # tie between 1023 and 1024 steps -> even
    assert r(1023 * 2.0 ** -24) == 0x03FF
    assert r(5e-324) == 0 and r(0.0) == 0 and r(-0.0) == 0x8000


def test_exhaustive_round_trip_and_decode():
    allb = np.arange(65536, dtype=np.uint16)
    v = fp16.bits_to_f64(allb)
    ref = allb.view(np.float16).astype(np.float64)         # numpy's decode, independent
    nan = np.isnan(ref)
    assert np.array_equal(np.isnan(v), nan)
    assert np.array_equal(v[~nan], ref[~nan])
    assert np.array_equal(np.signbit(v[~nan]), np.signbit(ref[~nan]))
    back = fp16.rne16_bits(v)
    assert np.array_equal(back[~nan], allb[~nan])
    assert np.all((back[nan] & 0x7FFF) > 0x7C00)


def _midpoint_cases():
    allb = np.arange(0, 0x7C00, dtype=np.uint16)
    lo = fp16.bits_to_f64(allb)
    hi = fp16.bits_to_f64(allb + 1)
    hi[-1] = 65536.0
    mid = (lo + hi) / 2                                    # exact in float64
    m32 = mid.astype(np.float32)
    cases = [mid, np.nextafter(m32, np.float32(0)).astype(np.float64),
             np.nextafter(m32, np.float32(1e9)).astype(np.float64),
             np.nextafter(mid, 0), np.nextafter(mid, 1e9)]
    x = np.concatenate(cases)
    return np.concatenate([x, -x])


def test_against_numpy_cast_midpoints_and_random():
    rng = np.random.default_rng(7)
    x = np.concatenate([
        _midpoint_cases(),
        rng.standard_normal(200000) * np.exp2(rng.uniform(-30, 17, 200000)),
        rng.uniform(-70000, 70000, 100000),
        np.exp2(rng.uniform(-27, -13, 100000)),
    ])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    got = fp16.rne16_bits(x)
    assert np.array_equal(got, want)


def test_against_numpy_cast_float32_sweep():
    # every 2^9-th float32 pattern whose magnitude is below 2^17 (0x48000000), both signs
    u = np.arange(0, 0x48000000, 1 << 9, dtype=np.uint32)
    u = np.concatenate([u, u | np.uint32(0x80000000)])
    x = u.view(np.float32)
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)
    assert np.array_equal(fp16.rne16_bits(x.astype(np.float64)), want)


def test_against_torch_cast():
    rng = np.random.default_rng(11)
    x = np.concatenate([_midpoint_cases().astype(np.float32),
                        (rng.standard_normal(300000) * np.exp2(rng.uniform(-28, 17, 300000))).astype(np.float32)])
    x = x[np.isfinite(x)]
    want = torch.from_numpy(x).to(torch.float16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(fp16.rne16_bits(x.astype(np.float64)), want)


def test_ulpdist():
    a = np.array([0x3C00, 0x0000, 0x8001, 0x7BFF, 0x7E00, 0x7E00], dtype=np.uint16)
    b = np.array([0x3C02, 0x8000, 0x0001, 0x7C00, 0x7E01, 0x3C00], dtype=np.uint16)
    d = fp16.ulpdist16(a, b)
    assert list(d[:5]) == [2, 0, 2, 1, 0] and d[5] > 1000
    assert list(fp16.ulpdist32(np.float32([1.0, -0.0]), np.float32([np.nextafter(np.float32(1), np.float32(2)), 0.0]))) == [1, 0]


def test_power_of_two_scaling_is_exact():
    """Sec. 3.2: scaling by 8 only raises exponents; for values that stay normal
    scale then unscale is the identity on the FP16 grid."""
    allb = np.arange(0x0400, 0x7C00, dtype=np.uint16)      # positive normals
    v = fp16.bits_to_f64(allb)
    for k in (3, 7, 10, 13):
        ok = v * 2.0 ** k <= 65504
        s = fp16.rne16_bits(v[ok] * 2.0 ** k)
        assert np.array_equal(fp16.bits_to_f64(s) / 2.0 ** k, v[ok])
        assert np.array_equal(s, allb[ok] + (k << 10))     # exponent field += k
