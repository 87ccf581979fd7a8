"""Seeded synthetic inputs for the five benchmark configurations.

This module serves both the CPU oracle's tests and the GPU path's tests and
benchmark.  It holds input recipes only -- shapes, value distributions, seeds,
and the quantisation of generated values to their FP16 storage type (numpy's
cast) -- and none of the method's arithmetic.  It imports neither the oracle
nor the GPU package.

The inputs are synthetic stand-ins carrying the shapes of the paper's
workloads (a ResNet-style 3x3 block, a bigLSTM-style projected LSTM layer,
a 116M-parameter speech model); no dataset item is reproduced.
"""
import numpy as np

BASE_SEED = 171003740 * 10


def rng_for(cfg, stream=0):
    return np.random.Generator(np.random.Philox(key=BASE_SEED + cfg, counter=[0, 0, 0, stream]))


def _h(x):
    """Quantise generated values to FP16 storage."""
    with np.errstate(over="ignore"):
        return np.asarray(x, dtype=np.float32).astype(np.float16)


def log_uniform_signed(rng, shape, lo_exp, hi_exp):
    """|g| = 2^u, u ~ U[lo_exp, hi_exp), random sign; float32."""
    u = rng.uniform(lo_exp, hi_exp, size=shape)
    sgn = np.where(rng.integers(0, 2, size=shape) == 0, -1.0, 1.0)
    return (sgn * np.exp2(u)).astype(np.float32)


# ---------------------------------------------------------------- cfg 1
def mlp(batch=256, d_in=1024, d_hid=1024, d_out=10):
    """Two-layer perceptron step: x ~ N(0,1); Xavier-uniform weights (FP32
    master + FP16 copy); uniform labels; static loss scale 2^10; SGD lr 0.01."""
    r = rng_for(1)
    x = _h(r.standard_normal((batch, d_in)))
    a1 = np.sqrt(6.0 / (d_in + d_hid))
    a2 = np.sqrt(6.0 / (d_hid + d_out))
    w1 = r.uniform(-a1, a1, size=(d_in, d_hid)).astype(np.float32)
    w2 = r.uniform(-a2, a2, size=(d_hid, d_out)).astype(np.float32)
    labels = r.integers(0, d_out, size=batch).astype(np.int32)
    return dict(x=x, w1_32=w1, w2_32=w2, w1_16=_h(w1), w2_16=_h(w2),
                labels=labels, scale=1024.0, lr=0.01)


# ---------------------------------------------------------------- cfg 2
def square_gemm(n=4096, scale=8192.0, m=None, k=None):
    """A[M,K], B[K,N] ~ 0.05 N(0,1); upstream gradient G[M,N] with |g|
    log-uniform in [2^-30, 2^-5), random sign, stored as FP16 of (scale * g).
    `g_true` keeps the unscaled FP32 values."""
    m = n if m is None else m
    k = n if k is None else k
    r = rng_for(2)
    A = _h(0.05 * r.standard_normal((m, k), dtype=np.float32))
    B = _h(0.05 * r.standard_normal((k, n), dtype=np.float32))
    g = log_uniform_signed(r, (m, n), -30.0, -5.0)
    return dict(A=A, B=B, g_true=g, G=_h(g * np.float32(scale)), scale=scale)


# ---------------------------------------------------------------- cfg 3
def lstmp(batch=256, steps=20, d_in=1024, d_proj=1024, d_cell=8192, scale=128.0):
    """Projected-LSTM layer GEMM operands, teacher-forced per timestep.
    xh_t[B, d_in+d_proj] ~ N(0,1); h_t[B, d_cell] ~ N(0,1) clipped to (-1,1);
    W_g[d_in+d_proj, 4 d_cell], W_p[d_cell, d_proj] ~ U(+-0.05); upstream
    gradients log-uniform as in the square GEMM, stored scaled by `scale`."""
    r = rng_for(3)
    dk = d_in + d_proj
    Wg = _h(r.uniform(-0.05, 0.05, size=(dk, 4 * d_cell)).astype(np.float32))
    Wp = _h(r.uniform(-0.05, 0.05, size=(d_cell, d_proj)).astype(np.float32))
    xh = _h(r.standard_normal((steps, batch, dk), dtype=np.float32))
    h = _h(np.clip(r.standard_normal((steps, batch, d_cell), dtype=np.float32), -0.999, 0.999))
    dgates = _h(log_uniform_signed(r, (steps, batch, 4 * d_cell), -30.0, -5.0) * np.float32(scale))
    dr = _h(log_uniform_signed(r, (steps, batch, d_proj), -30.0, -5.0) * np.float32(scale))
    return dict(Wg=Wg, Wp=Wp, xh=xh, h=h, dgates=dgates, dr=dr, scale=scale)


# ---------------------------------------------------------------- cfg 4
def conv_block(batch=256, hw=14, c=256, kf=256):
    """3x3 stride-1 pad-1 convolution block, NHWC / KRSC.  x = max(0, N(0,1));
    w ~ N(0, 2/(9c)); dy = |N(0,1)| * 2^-6 with half the entries zeroed (a
    ReLU-masked gradient), loss scale 1."""
    r = rng_for(4)
    x = _h(np.maximum(r.standard_normal((batch, hw, hw, c), dtype=np.float32), 0))
    w = _h(r.standard_normal((kf, 3, 3, c), dtype=np.float32) * np.float32(np.sqrt(2.0 / (9 * c))))
    dy = np.abs(r.standard_normal((batch, hw, hw, kf), dtype=np.float32)) * np.float32(2.0 ** -6)
    dy = _h(dy * (r.integers(0, 2, size=dy.shape) == 1))
    return dict(x=x, w=w, dy=dy)


# ---------------------------------------------------------------- cfg 5
SPECIALS = np.array([0x7C00, 0xFC00, 0x7E00, 0x7C01], dtype=np.uint16)  # +Inf -Inf qNaN sNaN


class FlatUpdate:
    """Flat-buffer master update with dynamic loss scaling.

    w32 ~ U(+-0.05), momentum 0, base gradient |g| log-uniform in [2^-28, 2^-2)
    with random sign.  Step t uses the base buffer rotated by a step-dependent
    offset, multiplied by the current scale in FP32 and only then stored as
    FP16 (an already-quantised buffer is never rescaled).  Inf/NaN patterns are
    planted at `inject_steps` (seed-chosen) at element 0, element n-1, one
    element of the last partial 8-group and one random element.
    """

    def __init__(self, n=116_000_000, steps=200, n_inject=8):
        self.n, self.steps = n, steps
        r = rng_for(5)
        self.w32 = r.uniform(-0.05, 0.05, size=n).astype(np.float32)
        self.g_true = log_uniform_signed(r, n, -28.0, -2.0)
        r2 = rng_for(5, stream=1)
        self.inject_steps = sorted(int(s) for s in r2.choice(np.arange(1, steps), size=min(n_inject, steps - 1), replace=False))
        self.offsets = r2.integers(0, n, size=steps)
        self.rand_pos = r2.integers(0, n, size=steps)
        self.lr, self.momentum, self.scale0 = 1e-3, 0.9, 65536.0

    def grad16(self, step, scale):
        g = np.roll(self.g_true, int(self.offsets[step]))
        g16 = _h(g * np.float32(scale))
        if step in self.inject_steps:
            j = self.inject_steps.index(step)
            gb = g16.view(np.uint16)
            tail = (self.n // 8) * 8 if self.n % 8 else self.n - 1
            for i, pos in enumerate((0, self.n - 1, min(tail, self.n - 1), int(self.rand_pos[step]))):
                if (j + i) % 2 == 0 or i == j % 4:
                    gb[pos] = SPECIALS[(i + j) % 4]
        return g16
