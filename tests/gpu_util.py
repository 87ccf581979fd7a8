"""Helpers for the GPU parity tests: numpy <-> device carriers, and the GEMM
acceptance rule.

GEMM acceptance (paper Sec. 3.3 leaves the kernel free only in the order and
rounding of its FP32 additions): an element passes if it is within 2 FP16 steps
of the oracle, or if it is the FP16 rounding of some value within the FP32
accumulation allowance  C_ACC * 2^-24 * sum|a*b|  of the exact sum (this second
clause only matters where the sum cancels to far below sum|a*b|).  Elements
whose exact sum is at least 2^-6 of sum|a*b| are "well conditioned" and must be
within 2 steps unconditionally.
"""
import numpy as np
import torch

from oracle import fp16

C_ACC = 4.0
U32 = 2.0 ** -24


def dev16(a):
    """float16 numpy container -> device tensor of the same bits."""
    a = np.ascontiguousarray(a)
    assert a.dtype == np.float16
    return torch.from_numpy(a.view(np.int16)).cuda().view(torch.float16)


def dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float16:
        return dev16(a)
    return torch.from_numpy(a).cuda()


def host16(t):
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.float16)


def host(t):
    if t.dtype == torch.float16:
        return host16(t)
    return t.detach().cpu().numpy()


def _ordered(hb):
    hb = np.asarray(hb, dtype=np.uint16).astype(np.int64)
    mag = hb & 0x7FFF
    return np.where(hb & 0x8000, -mag, mag)


def gemm_check(got16, want16, sabs, s64, label=""):
    """Apply the acceptance rule; returns a stats dict and asserts."""
    gb, wb = fp16.bits(got16), fp16.bits(want16)
    d = fp16.ulpdist16(gb, wb)
    tol = C_ACC * U32 * sabs
    with np.errstate(invalid="ignore", over="ignore"):
        lo = _ordered(fp16.rne16_bits(s64 - tol))
        hi = _ordered(fp16.rne16_bits(s64 + tol))
    g = _ordered(gb)
    finite = np.isfinite(s64)
    in_band = finite & (g >= lo) & (g <= hi) & ((gb & 0x7C00) != 0x7C00)
    # Inf from overflow: both must be the same Inf; NaN: both NaN (ulpdist handles it)
    ok = (d <= 2) | in_band
    # how many elements the rule would reject with half the allowance (C_ACC / 2)
    with np.errstate(invalid="ignore", over="ignore"):
        lo4 = _ordered(fp16.rne16_bits(s64 - 0.5 * tol))
        hi4 = _ordered(fp16.rne16_bits(s64 + 0.5 * tol))
    in_band4 = finite & (g >= lo4) & (g <= hi4) & ((gb & 0x7C00) != 0x7C00)
    well = finite & (np.abs(s64) >= sabs * 2.0 ** -6)
    stats = dict(label=label, n=int(d.size), exact=float((d == 0).mean()), max_ulp=int(d.max()),
                 max_ulp_well=int(d[well].max()) if well.any() else 0,
                 needed_band=float(((d > 2) & in_band).mean()), bad=int((~ok).sum()),
                 bad_at_half_allowance=int((~((d <= 2) | in_band4)).sum()))
    print("[gemm_check]", stats, flush=True)
    assert stats["bad"] == 0, stats
    assert stats["max_ulp_well"] <= 2, stats
    return stats
