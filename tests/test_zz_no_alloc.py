"""mpt_gemm_wgrad_static (the weight gradient for callers that cannot allocate: its split partials live in a device
array inside the library) gives mpt_gemm_wgrad's results bit for bit.  Called through the raw C ABI, twice in a row,
the second call on a smaller problem (the array then still holds the first call's partials), for the FP16 store,
the FP32 store and the FP32 accumulation with the overflow flag; a shape whose split would not fit the array is
refused before anything is launched."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import gemm
from paper_1710_03740_amd import binding as mpt
from gpu_util import dev16, gemm_check, host16

pytestmark = pytest.mark.gpu

vp, i64, ci, sz = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_size_t


def _inputs(M, N, K, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((M, K)).astype(np.float16)
    dY = (np.exp2(rng.uniform(-20, -4, (M, N))) * rng.choice([-1.0, 1.0], (M, N)) * 128.0).astype(np.float16)
    return X, dY


def _both(L, M, N, K, X, dY, out_fp32, accumulate, start=None):
    """Runs the workspace form and the static form on the same inputs; returns (reference, static, flags)."""
    s = vp(torch.cuda.current_stream().cuda_stream)
    need = L.mpt_gemm_workspace_bytes(mpt.OP_WGRAD, M, N, K)
    assert 0 < need <= mpt.STATIC_SCRATCH_BYTES, need          # the split path, and it fits the array
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    dX, dG = dev16(X), dev16(dY)
    dt = torch.float32 if out_fp32 else torch.float16
    outs, flags = [], []
    for static in (False, True):
        out = torch.full((K, N), 3.0, dtype=dt, device="cuda") if start is None else start.clone()
        flag = torch.zeros(1, dtype=torch.int32, device="cuda")
        if static:
            st = L.mpt_gemm_wgrad_static(s, i64(M), i64(N), i64(K), vp(dX.data_ptr()), i64(K), vp(dG.data_ptr()), i64(N),
                                         vp(out.data_ptr()), i64(N), ci(out_fp32), ci(accumulate), vp(flag.data_ptr()))
        else:
            st = L.mpt_gemm_wgrad(s, i64(M), i64(N), i64(K), vp(dX.data_ptr()), i64(K), vp(dG.data_ptr()), i64(N),
                                  vp(out.data_ptr()), i64(N), ci(out_fp32), ci(accumulate), vp(flag.data_ptr()),
                                  vp(ws.data_ptr()), sz(need))
        assert st == 0, (static, st)
        torch.cuda.synchronize()
        outs.append(out)
        flags.append(int(flag.item()))
    return outs[0], outs[1], flags


def test_static_scratch_weight_gradient_matches_the_workspace_form():
    L = mpt.lib()
    big, small = (4096, 512, 256), (1024, 256, 128)            # (M, N, K): reduction over M, output K x N
    for out_fp32, accumulate in ((0, 0), (1, 0), (1, 1)):
        for call, (M, N, K) in enumerate((big, small)):       # two calls in a row, the second smaller
            print("static wgrad: out_fp32=%d accumulate=%d call %d M=%d N=%d K=%d" % (out_fp32, accumulate, call, M, N, K), flush=True)
            X, dY = _inputs(M, N, K, 10 * out_fp32 + call)
            start = None
            if accumulate:
                start = torch.from_numpy(np.random.default_rng(5).standard_normal((K, N)).astype(np.float32)).cuda()
            ref, got, flags = _both(L, M, N, K, X, dY, out_fp32, accumulate, start)
            assert torch.equal(ref.view(torch.int32 if out_fp32 else torch.int16), got.view(torch.int32 if out_fp32 else torch.int16))
            assert flags == [0, 0]
            if not out_fp32:                                   # and against the oracle, by the usual acceptance rule
                o, sa, s64 = gemm.gemm_wgrad(X, dY, full=True)
                gemm_check(host16(got), o, sa, s64, "static wgrad M=%d N=%d K=%d" % (M, N, K))
    # an overflowing product raises the flag in both forms
    M, N, K = small
    X = np.full((M, K), 256.0, dtype=np.float16)
    dY = np.full((M, N), 256.0, dtype=np.float16)
    ref, got, flags = _both(L, M, N, K, X, dY, 0, 0)
    assert flags == [1, 1] and torch.equal(ref.view(torch.int16), got.view(torch.int16))
    assert np.isinf(host16(got).astype(np.float32)).all()


def test_static_scratch_refuses_what_does_not_fit_and_bad_arguments():
    L = mpt.lib()
    s = vp(torch.cuda.current_stream().cuda_stream)
    M, N, K = 256, 1024, 8192                                 # split partials of a 8192 x 1024 FP32 output: beyond the array
    assert L.mpt_gemm_workspace_bytes(mpt.OP_WGRAD, M, N, K) > mpt.STATIC_SCRATCH_BYTES
    X = torch.zeros((M, K), dtype=torch.float16, device="cuda")
    dY = torch.zeros((M, N), dtype=torch.float16, device="cuda")
    out = torch.full((K, N), 3.0, dtype=torch.float16, device="cuda")
    args = lambda x, g, o: (s, i64(M), i64(N), i64(K), vp(x), i64(K), vp(g), i64(N), vp(o), i64(N), ci(0), ci(0), vp(0))
    assert L.mpt_gemm_wgrad_static(*args(X.data_ptr(), dY.data_ptr(), out.data_ptr())) == -4
    assert b"workspace" in L.mpt_status_string(-4).lower()
    torch.cuda.synchronize()
    assert bool((out == 3.0).all())                           # nothing was launched
    assert L.mpt_gemm_wgrad_static(*args(0, dY.data_ptr(), out.data_ptr())) == -1
    assert L.mpt_gemm_wgrad_static(s, i64(0), i64(N), i64(K), vp(X.data_ptr()), i64(K), vp(dY.data_ptr()), i64(N),
                                   vp(out.data_ptr()), i64(N), ci(0), ci(0), vp(0)) == -2
    assert L.mpt_gemm_wgrad_static(s, i64(M), i64(N), i64(K), vp(X.data_ptr()), i64(K), vp(dY.data_ptr()), i64(N),
                                   vp(out.data_ptr()), i64(N), ci(0), ci(1), vp(0)) == -5        # accumulate needs FP32
    with pytest.raises(mpt.MptError):                          # the binding raises on the same refusal
        mpt.mpt_gemm_wgrad_static(X, dY, out)
