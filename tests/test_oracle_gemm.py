"""Pins for the oracle's three contractions: exact integer brute force, the
explicit-loop definition, adjoint identities, power-of-two invariance, a
library routine (torch float64 matmul + autograd), and planted mistakes."""
import numpy as np
import pytest
import torch

from oracle import fp16, gemm

SHAPES = [(1, 1, 1), (3, 5, 7), (33, 10, 65), (8, 16, 64)]


def _ints(rng, shape, lim=4):
    return rng.integers(-lim, lim + 1, size=shape).astype(np.float16)


@pytest.mark.parametrize("M,N,K", SHAPES)
def test_integer_brute_force_bit_exact(M, N, K):
    """|a|,|b| <= 4 and K <= 65 keep every partial sum an integer below 2048, so
    the FP16 result equals integer arithmetic bit-for-bit in all three passes."""
    rng = np.random.default_rng(M * 100 + N * 10 + K)
    X, W, dY = _ints(rng, (M, K)), _ints(rng, (K, N)), _ints(rng, (M, N))
    Xi, Wi, dYi = X.astype(np.int64), W.astype(np.int64), dY.astype(np.int64)
    y, _ = gemm.gemm_fwd(X, W)
    dx, _ = gemm.gemm_dgrad(dY, W)
    dw, _ = gemm.gemm_wgrad(X, dY)
    for got, want in ((y, Xi @ Wi), (dx, dYi @ Wi.T), (dw, Xi.T @ dYi)):
        assert np.abs(want).max() < 2048
        assert got.shape == want.shape
        assert np.array_equal(got.astype(np.float64), want.astype(np.float64))


@pytest.mark.parametrize("M,N,K", [(2, 3, 4), (5, 4, 9)])
def test_loops_definition_matches(M, N, K):
    rng = np.random.default_rng(3)
    X = (rng.standard_normal((M, K))).astype(np.float16)
    W = (rng.standard_normal((K, N)) * 0.1).astype(np.float16)
    dY = (rng.standard_normal((M, N)) * 0.01).astype(np.float16)
    assert np.array_equal(fp16.bits(gemm.gemm_fwd(X, W)[0]), fp16.bits(gemm.gemm_fwd_loops(X, W)))
    assert np.array_equal(fp16.bits(gemm.gemm_dgrad(dY, W)[0]), fp16.bits(gemm.gemm_dgrad_loops(dY, W)))
    assert np.array_equal(fp16.bits(gemm.gemm_wgrad(X, dY)[0]), fp16.bits(gemm.gemm_wgrad_loops(X, dY)))


def test_adjoint_identities_via_torch_autograd():
    """dgrad and wgrad are the adjoints of fwd: torch's float64 autograd of
    <dY, X W> gives the unrounded values the oracle must round."""
    rng = np.random.default_rng(5)
    M, N, K = 17, 9, 23
    X = rng.standard_normal((M, K)).astype(np.float16)
    W = (rng.standard_normal((K, N)) * 0.2).astype(np.float16)
    dY = (rng.standard_normal((M, N)) * 0.05).astype(np.float16)
    tx = torch.tensor(X.astype(np.float64), requires_grad=True)
    tw = torch.tensor(W.astype(np.float64), requires_grad=True)
    ty = tx @ tw
    ty.backward(torch.tensor(dY.astype(np.float64)))
    with np.errstate(over="ignore"):
        assert np.array_equal(gemm.gemm_fwd(X, W)[0], ty.detach().numpy().astype(np.float16))
        assert np.array_equal(gemm.gemm_dgrad(dY, W)[0], tx.grad.numpy().astype(np.float16))
        assert np.array_equal(gemm.gemm_wgrad(X, dY)[0], tw.grad.numpy().astype(np.float16))


def test_power_of_two_invariance():
    """Sec. 3.2: a power-of-two factor only shifts exponents, so scaling an
    operand scales the result bit-for-bit while nothing leaves the normal range."""
    rng = np.random.default_rng(9)
    X = rng.standard_normal((12, 40)).astype(np.float16)
    dY = (rng.uniform(0.5, 1.0, (12, 6)) * 2.0 ** -8).astype(np.float16)
    base, _ = gemm.gemm_wgrad(X, dY)
    scaled, _ = gemm.gemm_wgrad(X, (dY.astype(np.float32) * 128).astype(np.float16))
    b, s = fp16.to_f64(base), fp16.to_f64(scaled)
    normal = np.abs(b) >= 2.0 ** -14
    assert normal.any()
    assert np.array_equal(s[normal], b[normal] * 128)


def test_overflow_stores_inf_not_max():
    X = np.full((1, 4), 200.0, dtype=np.float16)
    W = np.full((4, 1), 100.0, dtype=np.float16)
    y, _ = gemm.gemm_fwd(X, W)
    assert fp16.bits(y)[0, 0] == 0x7C00
    W[0, 0] = -np.inf
    y, _ = gemm.gemm_fwd(X, W)
    assert fp16.bits(y)[0, 0] == 0xFC00
    W[1, 0] = np.inf
    assert np.isnan(gemm.gemm_fwd(X, W)[0][0, 0])


def test_small_gradients_flush_without_scale_and_survive_with_it():
    """Sec. 3.2: products below 2^-25 vanish on the FP16 store; the same
    contraction with the upstream gradient scaled by 2^13 keeps them."""
    X = np.zeros((1, 2), dtype=np.float16); X[0, 0] = 2.0 ** -10
    g = np.float32(2.0 ** -17)
    dY = np.array([[g]], dtype=np.float16)
    dw, _ = gemm.gemm_wgrad(X, dY)
    assert fp16.bits(dw)[0, 0] == 0                      # 2^-27 -> 0
    dYs = np.array([[g * 8192]], dtype=np.float16)
    dws, _ = gemm.gemm_wgrad(X, dYs)
    assert fp16.to_f64(dws)[0, 0] / 8192 == 2.0 ** -27


def test_fp32_accumulate_mode():
    rng = np.random.default_rng(2)
    X = rng.standard_normal((3, 8, 5)).astype(np.float16)
    dY = (rng.standard_normal((3, 8, 4)) * 2.0 ** -12).astype(np.float16)
    acc = None
    for t in range(3):
        acc, _ = gemm.gemm_wgrad(X[t], dY[t], out_fp32=True, acc32=acc)
    want = sum(X[t].astype(np.float64).T @ dY[t].astype(np.float64) for t in range(3))
    assert acc.dtype == np.float32
    assert fp16.ulpdist32(acc, want.astype(np.float32)).max() <= 2
    # going through FP16 partial sums instead loses the small terms
    via16 = sum(gemm.gemm_wgrad(X[t], dY[t])[0].astype(np.float64) for t in range(3))
    assert np.abs(via16 - want).max() > np.abs(acc - want).max()


def test_sabs_is_sum_of_magnitudes():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((4, 6)).astype(np.float16)
    W = rng.standard_normal((6, 3)).astype(np.float16)
    _, sabs = gemm.gemm_fwd(X, W)
    want = np.abs(X.astype(np.float64)) @ np.abs(W.astype(np.float64))
    assert np.allclose(sabs, want, rtol=1e-14)


def test_planted_mistakes_are_caught():
    """A transposed operand or a swapped pass fails the integer brute force."""
    rng = np.random.default_rng(1)
    X, W, dY = _ints(rng, (6, 6)), _ints(rng, (6, 6)), _ints(rng, (6, 6))
    Xi, Wi, dYi = X.astype(np.int64), W.astype(np.int64), dY.astype(np.int64)
    assert not np.array_equal(gemm.gemm_fwd(X, W.T.copy())[0].astype(np.int64), Xi @ Wi)
    assert not np.array_equal(gemm.gemm_dgrad(dY, W)[0].astype(np.int64), dYi @ Wi)
    assert not np.array_equal(gemm.gemm_wgrad(X, dY)[0].astype(np.int64), dYi.T @ Xi)


def test_fused_relu_forms_equal_the_unfused_composition():
    """Rounding commutes with max(., 0) (RNE is monotone and keeps the sign), so folding the ReLU into the store
    must give exactly what the separate pointwise pass gives; same for the backward mask."""
    from oracle import loss
    rng = np.random.default_rng(21)
    X = rng.standard_normal((37, 50)).astype(np.float16)
    W = (rng.standard_normal((50, 29)) * 0.2).astype(np.float16)
    h, _ = gemm.gemm_fwd_relu(X, W)
    y, _ = gemm.gemm_fwd(X, W)
    assert np.array_equal(fp16.bits(h), fp16.bits(loss.relu_fwd(y)))
    assert (h == 0).mean() > 0.3 and (h > 0).mean() > 0.3
    dY = (rng.standard_normal((37, 29)) * 2.0 ** -8).astype(np.float16)
    H = loss.relu_fwd(rng.standard_normal((37, 50)).astype(np.float16))
    dx, _ = gemm.gemm_dgrad_relu(dY, W, H)
    d0, _ = gemm.gemm_dgrad(dY, W)
    assert np.array_equal(fp16.bits(dx), fp16.bits(loss.relu_bwd(d0, H)))
    # a hand-made case: one row, weights +-1
    x = np.array([[1.0, 2.0]], dtype=np.float16); w = np.array([[1.0, -1.0], [1.0, -1.0]], dtype=np.float16)
    assert gemm.gemm_fwd_relu(x, w)[0].tolist() == [[3.0, 0.0]]
    assert gemm.gemm_dgrad_relu(np.array([[1.0, 2.0]], dtype=np.float16), w, np.array([[0.0, 5.0]], dtype=np.float16))[0].tolist() == [[0.0, -1.0]]
