"""The C-ABI library loads, exports every symbol the header declares, and
rejects bad arguments before touching the GPU (no compute calls here)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "mpt.h")


@pytest.fixture(scope="module")
def L():
    from paper_1710_03740_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_1710_03740_amd import build
        build.build(verbose=False)
    return binding.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mpt_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_exported(L):
    names = declared_symbols()
    assert len(names) >= 18
    for n in names:
        assert hasattr(L, n), n


def test_binding_covers_header():
    from paper_1710_03740_amd import binding
    assert sorted(binding.SIGNATURES) == declared_symbols()
    for n in declared_symbols():
        if n not in ("mpt_scaler_init",):
            assert hasattr(binding, n) or n == "mpt_status_string", n


def test_status_strings(L):
    for st in range(0, -7, -1):
        assert L.mpt_status_string(st)
    assert b"unknown" in L.mpt_status_string(-99)
    assert L.mpt_version() >= 100


def test_scaler_host_policy(L):
    from paper_1710_03740_amd import binding
    s = binding.mpt_scaler_init(65536.0, 5)
    assert (s.scale, s.inv_scale, s.growth_interval, s.growth, s.backoff) == (65536.0, 2.0 ** -16, 5, 2.0, 0.5)
    from oracle.scaler import Scaler
    o = Scaler(scale=65536.0, growth_interval=5)
    seq = [0, 0, 1, 0, 0, 0, 0, 0, 0, 1, 1] + [0] * 12
    for ov in seq:
        assert binding.mpt_loss_scale_update(s, ov) == o.update(ov)
        assert s.good_steps == o.good_steps and s.inv_scale == 1.0 / o.scale
    assert L.mpt_scaler_init(None, 1.0, 5) == -1
    assert L.mpt_scaler_init(ctypes.byref(s), -1.0, 5) == -5
    assert L.mpt_scaler_init(ctypes.byref(s), 1.0, 0) == -5


def test_argument_errors_before_any_launch(L):
    P = ctypes.c_void_p(0x1000)      # never dereferenced: every call below must fail validation first
    Z = ctypes.c_void_p(0)
    odd = ctypes.c_void_p(0x1001)
    assert L.mpt_gemm_fwd(Z, 8, 8, 8, Z, 8, P, 8, P, 8, Z, 0) == -1
    assert L.mpt_gemm_fwd(Z, 0, 8, 8, P, 8, P, 8, P, 8, Z, 0) == -2
    assert L.mpt_gemm_fwd(Z, 8, 8, 8, P, 7, P, 8, P, 8, Z, 0) == -2
    assert L.mpt_gemm_fwd(Z, 8, 8, 8, odd, 8, P, 8, P, 8, Z, 0) == -3
    assert L.mpt_gemm_dgrad(Z, 8, 8, 8, P, 8, P, 8, Z, 8, Z, 0) == -1
    assert L.mpt_gemm_dgrad(Z, 8, 8, -1, P, 8, P, 8, P, 8, Z, 0) == -2
    assert L.mpt_gemm_wgrad(Z, 8, 8, 8, P, 8, P, 8, P, 8, 0, 1, Z, Z, 0) == -5      # accumulate needs FP32 out
    assert L.mpt_gemm_wgrad(Z, 8, 8, 8, P, 8, P, 8, P, 4, 0, 0, Z, Z, 0) == -2
    # workspace given but too small for the split the planner picks
    need = L.mpt_gemm_workspace_bytes(2, 50176, 2304, 256)
    assert need > 0
    assert L.mpt_gemm_wgrad(Z, 50176, 2304, 256, P, 256, P, 2304, P, 2304, 0, 0, Z, P, need - 1) == -4
    assert L.mpt_gemm_workspace_bytes(7, 8, 8, 8) == 0
    assert L.mpt_conv3x3_fwd(Z, 1, 4, 4, 12, 8, P, P, P, Z, 0) == -2               # C % 8 != 0
    assert L.mpt_conv3x3_dgrad(Z, 1, 4, 4, 8, 8, P, Z, P, Z, 0) == -1
    assert L.mpt_conv3x3_wgrad(Z, 1, 4, 4, 8, 8, P, P, odd, Z, Z, 0) == -3
    assert L.mpt_gemm_fwd_relu(Z, 8, 8, 8, P, 8, P, 8, Z, 8, Z, 0) == -1
    assert L.mpt_gemm_dgrad_relu(Z, 8, 8, 8, P, 8, P, 8, Z, 8, P, 8, Z, 0) == -1       # the mask is required
    assert L.mpt_gemm_dgrad_relu(Z, 8, 8, 8, P, 8, P, 8, P, 7, P, 8, Z, 0) == -2       # mask row stride below K
    assert L.mpt_gemm_dgrad_relu(Z, 8, 8, 8, P, 8, P, 8, odd, 8, P, 8, Z, 0) == -3
    need = L.mpt_bn_workspace_bytes(1000, 64)
    assert need > 0 and L.mpt_bn_workspace_bytes(0, 64) == 0
    assert L.mpt_bn_stats(Z, 1000, 64, P, 64, P, P, Z, 0) == -1                        # the reductions need their scratch
    assert L.mpt_bn_stats(Z, 1000, 64, P, 63, P, P, P, need) == -2
    assert L.mpt_bn_stats(Z, 1000, 64, P, 64, P, P, P, need - 1) == -4
    assert L.mpt_bn_stats(Z, 1000, 64, odd, 64, P, P, P, need) == -3
    assert L.mpt_bn_apply(Z, 1000, 64, P, 64, P, P, P, P, -1.0, 0, P, 64) == -5
    assert L.mpt_bn_apply(Z, 1000, 64, P, 64, P, P, P, Z, 1e-5, 0, P, 64) == -1
    assert L.mpt_bn_apply(Z, 1000, 64, P, 64, P, P, P, P, 1e-5, 0, P, 8) == -2
    assert L.mpt_bn_bwd_reduce(Z, 1000, 64, P, 64, P, 64, P, P, 1e-5, P, P, P, need - 8) == -4
    assert L.mpt_bn_bwd_reduce(Z, 1000, 64, P, 64, Z, 64, P, P, 1e-5, P, P, P, need) == -1
    assert L.mpt_bn_bwd_apply(Z, 1000, 64, P, 64, P, 64, P, P, P, float("nan"), P, P, P, 64) == -5
    assert L.mpt_bn_bwd_apply(Z, 1000, 0, P, 64, P, 64, P, P, P, 1e-5, P, P, P, 64) == -2
    hp = (ctypes.c_float * 9)(0.1, 0.9, 0.999, 1e-8, 0.0, 0.1, 0.001, 0.1, 0.001)
    assert L.mpt_optimizer_update(Z, 8, 3, hp, P, P, Z, P, 0, P, 1.0, Z, Z) == -1          # Adam needs its second moment
    assert L.mpt_optimizer_update(Z, 8, 9, hp, P, P, P, P, 0, P, 1.0, Z, Z) == -5
    assert L.mpt_optimizer_update(Z, 8, 1, Z, P, P, P, P, 0, P, 1.0, Z, Z) == -1
    assert L.mpt_optimizer_update(Z, 8, 2, hp, P, odd, P, P, 0, P, 1.0, Z, Z) == -3
    assert L.mpt_optimizer_update(Z, 8, 0, hp, P, P, P, P, 0, P, 0.0, Z, Z) == -5
    bad = (ctypes.c_float * 9)(0.1, 0.9, 0.999, 1e-8, 0.0, 0.1, 0.001, 0.0, 0.001)
    assert L.mpt_optimizer_update(Z, 8, 3, bad, P, P, P, P, 0, P, 1.0, Z, Z) == -5          # bias correction must be > 0
    assert L.mpt_optimizer_update(Z, 0, 3, Z, Z, Z, Z, Z, 0, Z, 1.0, Z, Z) == 0
    assert L.mpt_grad_stats(Z, P, 8, 0, Z, P) == -1
    assert L.mpt_grad_stats(Z, odd, 8, 0, P, P) == -3
    assert L.mpt_unscale_check(Z, Z, 0, 8, 1.0, Z, P) == -1
    assert L.mpt_unscale_check(Z, P, 0, 8, 0.0, Z, P) == -5
    assert L.mpt_unscale_check(Z, P, 0, 8, float("inf"), Z, P) == -5
    assert L.mpt_unscale_check(Z, odd, 0, 8, 1.0, Z, P) == -3
    assert L.mpt_unscale_check(Z, Z, 0, 0, 1.0, Z, Z) == 0                          # n = 0: no-op
    assert L.mpt_master_update(Z, 8, Z, Z, P, 0, P, 1.0, Z, 0.1, 0.9, Z) == -1
    assert L.mpt_master_update(Z, 8, P, Z, P, 0, P, -1.0, Z, 0.1, 0.9, Z) == -5
    assert L.mpt_master_update(Z, 8, P, Z, P, 0, P, 1.0, Z, float("nan"), 0.9, Z) == -5
    assert L.mpt_master_update(Z, 8, ctypes.c_void_p(0x1002), Z, P, 0, P, 1.0, Z, 0.1, 0.9, Z) == -3
    assert L.mpt_master_update(Z, 0, Z, Z, Z, 0, Z, 1.0, Z, 0.1, 0.9, Z) == 0
    Q = ctypes.c_void_p(0x200000)                                                   # a second, non-overlapping "buffer"
    assert L.mpt_master_update_fused(Z, 8, P, Z, P, 0, Z, Z, Q, 1.0, Z, 0.1, 0.9, P) == -1
    assert L.mpt_master_update_fused(Z, 8, P, Z, P, 0, Q, Z, Q, 1.0, Z, 0.1, 0.9, Z) == -1          # the flag is required
    assert L.mpt_master_update_fused(Z, 8, P, P, P, 0, Q, Z, Q, 1.0, Z, 0.1, 0.9, P) == -5          # one momentum pointer only
    assert L.mpt_master_update_fused(Z, 8, P, Z, P, 0, P, Z, Q, 1.0, Z, 0.1, 0.9, P) == -5          # output overlaps input
    assert L.mpt_master_update_fused(Z, 8, P, Z, P, 0, ctypes.c_void_p(P.value + 16), Z, Q, 1.0, Z, 0.1, 0.9, P) == -5
    assert L.mpt_master_update_fused(Z, 8, P, Z, P, 0, Q, Z, Q, 0.0, Z, 0.1, 0.9, P) == -5
    assert L.mpt_master_update_fused(Z, 8, P, Z, P, 0, ctypes.c_void_p(0x200002), Z, Q, 1.0, Z, 0.1, 0.9, P) == -3
    assert L.mpt_master_update_fused(Z, 0, Z, Z, Z, 0, Z, Z, Z, 1.0, Z, 0.1, 0.9, Z) == 0
    class Item(ctypes.Structure):
        _fields_ = [("w32", ctypes.c_void_p), ("m32", ctypes.c_void_p), ("grad", ctypes.c_void_p), ("w16", ctypes.c_void_p), ("n", ctypes.c_size_t)]
    items = (Item * 2)(Item(P.value, None, P.value, P.value, 8), Item(Q.value, None, Q.value, Q.value, 8))
    ip = ctypes.cast(items, ctypes.c_void_p)
    assert L.mpt_master_update_multi(Z, 0, Z, 0, 1.0, Z, 0.1, 0.9, Z) == 0                   # no tensors: no-op
    assert L.mpt_master_update_multi(Z, -1, ip, 0, 1.0, Z, 0.1, 0.9, Z) == -5
    assert L.mpt_master_update_multi(Z, 2, Z, 0, 1.0, Z, 0.1, 0.9, Z) == -1
    assert L.mpt_master_update_multi(Z, 2, ip, 0, 0.0, Z, 0.1, 0.9, Z) == -5
    assert L.mpt_master_update_multi(Z, 2, ip, 0, 1.0, Z, float("inf"), 0.9, Z) == -5
    items[1].w16 = None
    assert L.mpt_master_update_multi(Z, 2, ip, 0, 1.0, Z, 0.1, 0.9, Z) == -1                 # the second tensor lacks a buffer: nothing is launched
    items[1].w16 = Q.value; items[1].m32 = Q.value
    assert L.mpt_master_update_multi(Z, 2, ip, 0, 1.0, Z, 0.1, 0.9, Z) == -5                 # momentum for one tensor only
    items[1].m32 = None; items[1].grad = 0x200001
    assert L.mpt_master_update_multi(Z, 2, ip, 0, 1.0, Z, 0.1, 0.9, Z) == -3
    items[0].n = 0; items[1].n = 0; items[1].grad = None
    assert L.mpt_master_update_multi(Z, 2, ip, 0, 1.0, Z, 0.1, 0.9, Z) == 0                  # empty tensors are skipped, whatever their pointers
    assert L.mpt_probe_mfma(Z, 10, 0, Z) == -1
    assert L.mpt_probe_mfma(Z, 0, 0, P) == -5
    assert L.mpt_loss_scale_update_dev(Z, Z, P) == -1
    assert L.mpt_relu_fwd(Z, 8, Z, P) == -1
    assert L.mpt_relu_bwd(Z, 8, P, P, Z) == -1
    assert L.mpt_softmax_xent_scaled(Z, 4, 5000, P, 4999, P, 1.0, Z, Z, P, 5000) == -2
    assert L.mpt_softmax_xent_scaled(Z, 4, 10, P, 10, P, 0.0, Z, Z, P, 10) == -5
    assert L.mpt_softmax_xent_scaled(Z, 4, 10, P, 10, P, 1.0, P, Z, P, 10) == -1      # a mean loss needs the per-row buffer


def test_missing_library_is_an_error(monkeypatch):
    from paper_1710_03740_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libmpt.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        binding.lib()


def test_suggested_scale_matches_the_oracle_for_every_fp16_magnitude(L):
    """Host-only function: checked exhaustively against the oracle's rule (largest 2^k with 2^k * max <= 65504)."""
    import numpy as np
    from oracle import gradstats
    L.mpt_suggest_loss_scale_log2.restype = ctypes.c_int
    L.mpt_suggest_loss_scale_log2.argtypes = [ctypes.c_uint32, ctypes.c_int]
    vals = np.arange(1, 0x7C00, dtype=np.uint16).view(np.float16).astype(np.float64)
    for bits in list(range(1, 0x7C00, 37)) + [1, 0x3FF, 0x400, 0x3C00, 0x7BFF]:
        k = gradstats.suggest_scale_log2(float(vals[bits - 1]))
        assert L.mpt_suggest_loss_scale_log2(bits, -99) == max(-24, min(40, k)), bits
    assert L.mpt_suggest_loss_scale_log2(0, -99) == -99 and L.mpt_suggest_loss_scale_log2(0x7C00, 7) == 7
    assert L.mpt_suggest_loss_scale_log2(0x8000 | 0x3C00, 0) == 15          # the sign bit is ignored: |-1.0|


def test_lstm_cell_argument_errors(L):
    P, Z, odd = ctypes.c_void_p(0x1000), ctypes.c_void_p(0), ctypes.c_void_p(0x1001)
    i64 = ctypes.c_int64
    f = L.mpt_lstm_cell_fwd
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.c_void_p, i64, i64] + [ctypes.c_void_p, i64, ctypes.c_void_p, i64, ctypes.c_void_p, ctypes.c_void_p, i64] + [ctypes.c_void_p, i64] * 3
    assert f(Z, 4, 8, Z, 32, P, 32, Z, P, 8, P, 32, P, 8, P, 8) == -1
    assert f(Z, 4, 8, P, 31, P, 32, Z, P, 8, P, 32, P, 8, P, 8) == -2
    assert f(Z, 0, 8, P, 32, P, 32, Z, P, 8, P, 32, P, 8, P, 8) == -2
    assert f(Z, 4, 8, P, 32, odd, 32, Z, P, 8, P, 32, P, 8, P, 8) == -3
    b = L.mpt_lstm_cell_bwd
    b.restype = ctypes.c_int
    b.argtypes = [ctypes.c_void_p, i64, i64] + [ctypes.c_void_p, i64] * 7
    assert b(Z, 4, 8, Z, 8, Z, 0, P, 32, P, 8, P, 8, P, 32, P, 8) == -1
    assert b(Z, 4, 8, P, 8, Z, 0, P, 32, P, 8, P, 8, P, 16, P, 8) == -2


def test_workspace_size_is_a_whole_number_of_partial_outputs(L):
    """mpt_gemm_workspace_bytes depends on the shape only and always asks for a whole number (0, or 2 to 64) of FP32
    partial outputs [I][J], whichever way of splitting the library would pick; an invalid shape or pass asks for 0."""
    L.mpt_gemm_workspace_bytes.restype = ctypes.c_size_t
    L.mpt_gemm_workspace_bytes.argtypes = [ctypes.c_int, ctypes.c_int64, ctypes.c_int64, ctypes.c_int64]
    shapes = [(1, 1, 1), (256, 10, 1024), (256, 1024, 1024), (256, 1024, 8192), (256, 32768, 2048), (256, 32768, 1024), (128, 4096, 4160),
              (384, 768, 8192), (4096, 4096, 4096), (2048, 2048, 1024), (5120, 32768, 1024), (1000, 520, 776), (100, 72, 2048)]
    for (M, N, K) in shapes:
        for op, (I, J) in ((0, (M, N)), (1, (M, K)), (2, (K, N))):
            b = L.mpt_gemm_workspace_bytes(op, M, N, K)
            assert b % (I * J * 4) == 0, (op, M, N, K, b)
            assert b // (I * J * 4) in [0] + list(range(2, 65)), (op, M, N, K, b)
            assert b == L.mpt_gemm_workspace_bytes(op, M, N, K)
    assert L.mpt_gemm_workspace_bytes(0, 4096, 4096, 4096) == 0                      # 256 tiles: nothing to split
    # the larger of the plans' needs: 64 splits of 256-row tiles (taken when the operands are not aligned for the streamed
    # kernel), although aligned operands run as 128-row tiles with 32 splits
    assert L.mpt_gemm_workspace_bytes(1, 256, 32768, 1024) == 64 * 256 * 1024 * 4
    assert L.mpt_gemm_workspace_bytes(3, 256, 256, 256) == 0
    assert L.mpt_gemm_workspace_bytes(0, 0, 256, 256) == 0
