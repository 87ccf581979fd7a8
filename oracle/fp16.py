"""IEEE binary16 encode/decode by bit manipulation (oracle; test infrastructure only).

Paper facts this file encodes: the FP16 maximum is 65504 (Sec. 3.2), normal
exponents span [-14, 15] (Sec. 3.2), and 2^-24 is the smallest non-zero
magnitude (Sec. 3.1).  Rounding is round-to-nearest-even in ONE step from the
wide value; overflow produces an infinity, never a clamp.

Reading taken where the paper is loose: Sec. 3.1 says magnitudes below 2^-24
become zero.  Under round-to-nearest-even only |x| <= 2^-25 gives zero; the
open band (2^-25, 2^-24) rounds UP to 2^-24.  The oracle follows IEEE.

FP16 tensors are carried as numpy arrays of dtype float16 used purely as a
16-bit container; every conversion goes through the functions below, and the
tests pin them against numpy's and torch's independent casts.
"""
import numpy as np

_U64 = np.uint64


def rne16_bits(x):
    """float64 array -> uint16 binary16 bit patterns, single RNE rounding."""
    x = np.ascontiguousarray(x, dtype=np.float64)
    b = x.view(np.uint64)
    sign = ((b >> _U64(63)).astype(np.uint16)) << np.uint16(15)
    ebits = ((b >> _U64(52)) & _U64(0x7FF)).astype(np.int64)
    frac = b & _U64((1 << 52) - 1)
    is_nan = (ebits == 0x7FF) & (frac != 0)
    is_inf = (ebits == 0x7FF) & (frac == 0)
    e = ebits - 1023                      # unbiased exponent of a normal double
    sig = frac | _U64(1 << 52)            # 53-bit significand, value = sig * 2^(e-52)
    # number of low bits dropped: 42 for an FP16 normal, more below 2^-14
    extra = np.clip(-14 - e, 0, None)
    shift = np.minimum(42 + extra, 63).astype(np.uint64)
    floor = sig >> shift
    rem = sig & ((_U64(1) << shift) - _U64(1))
    half = _U64(1) << (shift - _U64(1))
    up = (rem > half) | ((rem == half) & ((floor & _U64(1)) == _U64(1)))
    q = (floor + up.astype(np.uint64)).astype(np.int64)   # rounded significand
    # normals: q in [1024, 2048]; exponent field e+15, carry folds in naturally
    normal = e >= -14
    field = np.where(normal, ((e + 15) << 10) + (q - 1024), q)
    # doubles that are zero/subnormal, or far below 2^-25, round to zero
    tiny = (ebits == 0) | (e < -26)
    field = np.where(tiny, 0, field)
    field = np.where(field >= 0x7C00, 0x7C00, field)      # overflow -> Inf
    field = np.where(is_inf, 0x7C00, field)
    field = np.where(is_nan, 0x7E00, field)
    return (field.astype(np.uint16) | sign).reshape(x.shape)


def rne16(x):
    """float64/float32 array -> float16 container (own rounding, see rne16_bits)."""
    return rne16_bits(np.asarray(x, dtype=np.float64)).view(np.float16)


def bits_to_f64(h):
    """uint16 binary16 patterns -> float64, exact."""
    h = np.asarray(h, dtype=np.uint16)
    s = np.where((h >> 15) & 1, -1.0, 1.0)
    ef = ((h >> 10) & 0x1F).astype(np.int64)
    mf = (h & 0x3FF).astype(np.float64)
    sub = np.ldexp(mf, -24)
    nor = np.ldexp(1024.0 + mf, np.where(ef > 0, ef - 25, 0))
    v = np.where(ef == 0, sub, nor)
    v = np.where(ef == 31, np.where(mf == 0, np.inf, np.nan), v)
    return s * v


def to_f64(h16):
    """float16 container -> float64, exact (own decode)."""
    h16 = np.asarray(h16)
    assert h16.dtype == np.float16, h16.dtype
    return bits_to_f64(h16.view(np.uint16))


def bits(h16):
    h16 = np.asarray(h16)
    assert h16.dtype == np.float16
    return h16.view(np.uint16)


def is_special_bits(hb):
    """True where the pattern is +-Inf or NaN (exponent field all ones)."""
    hb = np.asarray(hb, dtype=np.uint16)
    return (hb & 0x7C00) == 0x7C00


def _ordered(hb):
    """Map patterns to integers monotone in value (+0 and -0 coincide)."""
    hb = np.asarray(hb, dtype=np.uint16).astype(np.int64)
    mag = hb & 0x7FFF
    return np.where(hb & 0x8000, -mag, mag)


def ulpdist16(a_bits, b_bits):
    """Distance in representable FP16 steps; NaN vs NaN = 0, NaN vs number = huge."""
    a_bits = np.asarray(a_bits, dtype=np.uint16)
    b_bits = np.asarray(b_bits, dtype=np.uint16)
    d = np.abs(_ordered(a_bits) - _ordered(b_bits))
    an = (a_bits & 0x7FFF) > 0x7C00
    bn = (b_bits & 0x7FFF) > 0x7C00
    d = np.where(an & bn, 0, d)
    d = np.where(an ^ bn, 1 << 20, d)
    return d


def ulpdist32(a, b):
    """Distance in representable FP32 steps between float32 arrays."""
    def o(x):
        u = np.asarray(x, dtype=np.float32).view(np.uint32).astype(np.int64)
        mag = u & 0x7FFFFFFF
        return np.where(u & 0x80000000, -mag, mag)
    a = np.asarray(a, dtype=np.float32)
    b = np.asarray(b, dtype=np.float32)
    d = np.abs(o(a) - o(b))
    an, bn = np.isnan(a), np.isnan(b)
    d = np.where(an & bn, 0, d)
    d = np.where(an ^ bn, 1 << 40, d)
    return d
