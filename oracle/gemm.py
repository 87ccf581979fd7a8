"""Dense contractions of one layer (oracle; test infrastructure only).

Paper Sec. 3.3: an FP16 dot product accumulates its partial products into a
wider value which is converted to FP16 before it is written to memory.
Sec. 3.1 / Fig. 1 name the three contractions of a layer: forward,
backward-activation and backward-weight, all on FP16 tensors.

Definition used here: every FP16xFP16 product is exact (22 significant bits),
the sum is taken in FP64 (standing in for the exact sum; a conforming kernel is
free only in the order and rounding of its FP32 additions) and rounded once,
RNE, to FP16.  An accumulator at or above 65520 stores Inf: overflow must reach
the weight gradients so that Sec. 3.2's check can see it.

Row-major shapes: X[M,K] activations, W[K,N] weights, Y[M,N], dY[M,N].
Each routine also returns sabs = sum |a*b| per output, the scale against which
FP32 accumulation error of a real kernel is judged; with full=True it returns
the unrounded FP64 sum as a third value.
"""
import numpy as np
from .fp16 import rne16, to_f64


def _contract(A, B):
    """A[I,R] @ B[R,J] in FP64, plus the same contraction of magnitudes."""
    with np.errstate(invalid="ignore", over="ignore"):   # Inf/NaN operands are legal inputs
        return A @ B, np.abs(A) @ np.abs(B)


def _ret(s, sabs, full):
    return (rne16(s), sabs, s) if full else (rne16(s), sabs)


def gemm_fwd(X16, W16, full=False):
    """Y[m,n] = rne16(sum_k X[m,k] W[k,n])."""
    s, sabs = _contract(to_f64(X16), to_f64(W16))
    return _ret(s, sabs, full)


def gemm_dgrad(dY16, W16, full=False):
    """dX[m,k] = rne16(sum_n dY[m,n] W[k,n])."""
    s, sabs = _contract(to_f64(dY16), to_f64(W16).T)
    return _ret(s, sabs, full)


def gemm_fwd_relu(X16, W16, full=False):
    """H[m,n] = rne16(max(sum_k X[m,k] W[k,n], 0)): the layer's pointwise non-linearity
    (Sec. 3.3, third category) applied to the wide sum before its one rounding."""
    s, sabs = _contract(to_f64(X16), to_f64(W16))
    with np.errstate(invalid="ignore"):
        s = np.where(s > 0, s, 0.0)                  # same rule as the stand-alone ReLU: anything not > 0 (NaN too) gives 0
    return _ret(s, sabs, full)


def gemm_dgrad_relu(dY16, W16, H16, full=False):
    """dX[m,k] = rne16(sum_n dY[m,n] W[k,n]) where H[m,k] > 0, else 0: the backward pass of
    the layer below's ReLU folded into the store (H is that layer's FP16 output)."""
    s, sabs = _contract(to_f64(dY16), to_f64(W16).T)
    s = np.where(to_f64(H16) > 0, s, 0.0)
    return _ret(s, sabs, full)


def gemm_wgrad(X16, dY16, out_fp32=False, acc32=None, full=False):
    """dW[k,n] = sum_m X[m,k] dY[m,n].

    out_fp32=False: FP16 store (the paper's stored weight gradient).
    out_fp32=True : FP32 store; with acc32 given the running FP32 buffer becomes
    rne32(acc32 + this call's sum), evaluated in FP64 per call (used to add
    per-timestep contributions without passing through FP16).
    """
    s, sabs = _contract(to_f64(X16).T, to_f64(dY16))
    if not out_fp32:
        assert acc32 is None
        return _ret(s, sabs, full)
    if acc32 is not None:
        s = s + np.asarray(acc32, dtype=np.float32).astype(np.float64)
    with np.errstate(over="ignore"):
        out = s.astype(np.float32)
    return (out, sabs, s) if full else (out, sabs)


# ---- the same three definitions as explicit loops (tiny inputs only) ----

def _scalar(h):
    return float(to_f64(np.asarray(h, dtype=np.float16).reshape(1))[0])


def gemm_fwd_loops(X16, W16):
    M, K = X16.shape
    K2, N = W16.shape
    assert K == K2
    out = np.zeros((M, N), dtype=np.float64)
    for m in range(M):
        for n in range(N):
            acc = 0.0
            for k in range(K):
                acc += _scalar(X16[m, k]) * _scalar(W16[k, n])
            out[m, n] = acc
    return rne16(out)


def gemm_dgrad_loops(dY16, W16):
    M, N = dY16.shape
    K, N2 = W16.shape
    assert N == N2
    out = np.zeros((M, K), dtype=np.float64)
    for m in range(M):
        for k in range(K):
            acc = 0.0
            for n in range(N):
                acc += _scalar(dY16[m, n]) * _scalar(W16[k, n])
            out[m, k] = acc
    return rne16(out)


def gemm_wgrad_loops(X16, dY16):
    M, K = X16.shape
    M2, N = dY16.shape
    assert M == M2
    out = np.zeros((K, N), dtype=np.float64)
    for k in range(K):
        for n in range(N):
            acc = 0.0
            for m in range(M):
                acc += _scalar(X16[m, k]) * _scalar(dY16[m, n])
            out[k, n] = acc
    return rne16(out)
