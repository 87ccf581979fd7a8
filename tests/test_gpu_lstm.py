"""GPU parity of the LSTM cell kernels against the oracle (teacher-forced: every step is fed the oracle's FP16
inputs, bit-identical), and a free-running projected layer on the device compared loosely and for sanity."""
import numpy as np
import pytest
import torch

from oracle import lstm, fp16
from paper_1710_03740_amd import binding as mpt
from gpu_util import dev, dev16, host16

pytestmark = pytest.mark.gpu


def _e(*shape):
    return torch.full(shape, float("nan"), dtype=torch.float16, device="cuda")


def _close16(got, want, mag=None, frac=0.03):
    """Within one FP16 step of the oracle; where the value is a sum that cancels (state update, state gradient),
    within 2^-20 of the magnitude of its terms instead (the FP32 evaluation of exp / reciprocal / tanh is good to
    a few FP32 ulps of each term, not of their difference)."""
    d = fp16.ulpdist16(fp16.bits(got), fp16.bits(want))
    ok = d <= 1
    if mag is not None:
        ok |= np.abs(got.astype(np.float64) - want.astype(np.float64)) <= 2.0 ** -20 * mag
    assert ok.all() and (d > 0).mean() < frac, (int(d.max()), float((d > 0).mean()))


def _inputs(B, H, seed):
    rng = np.random.default_rng(seed)
    gx = (rng.standard_normal((B, 4 * H)) * 2).astype(np.float16)
    gr = rng.standard_normal((B, 4 * H)).astype(np.float16)
    bias = (rng.standard_normal(4 * H) * 0.5).astype(np.float32)
    cp = (rng.standard_normal((B, H)) * 1.5).astype(np.float16)
    dh = (np.exp2(rng.uniform(-14, -2, (B, H))) * rng.choice([-1, 1], (B, H))).astype(np.float16)
    dcn = (np.exp2(rng.uniform(-14, -2, (B, H))) * rng.choice([-1, 1], (B, H))).astype(np.float16)
    return gx, gr, bias, cp, dh, dcn


@pytest.mark.parametrize("B,H", [(1, 8), (3, 24), (5, 7), (64, 1024), (256, 8192), (1536, 8192)])   # the last: > 192 MB moved, the streaming instances
def test_cell_forward_and_backward_teacher_forced(B, H):
    gx, gr, bias, cp, dh, dcn = _inputs(B, H, B * 31 + H)
    for use_gr, use_bias in ((True, True), (False, False)):
        act, c, h = lstm.lstm_cell_fwd(gx, gr if use_gr else np.zeros_like(gr), bias if use_bias else None, cp)
        d_act, d_c, d_h = _e(B, 4 * H), _e(B, H), _e(B, H)
        mpt.mpt_lstm_cell_fwd(dev16(gx), dev16(gr) if use_gr else None, dev(bias) if use_bias else None, dev16(cp), d_act, d_c, d_h)
        cmag = np.abs(cp.astype(np.float64)) + 1.0
        _close16(host16(d_act), act); _close16(host16(d_c), c, cmag); _close16(host16(d_h), h, cmag)      # h = o * tanh(c) inherits c's absolute error
    # backward from the oracle's stored tensors
    act, c, h = lstm.lstm_cell_fwd(gx, gr, bias, cp)
    da, dcp = lstm.lstm_cell_bwd(dh, dcn, act, c, cp)
    d_da, d_dcp = _e(B, 4 * H), _e(B, H)
    mpt.mpt_lstm_cell_bwd(dev16(dh), dev16(dcn), dev16(act), dev16(c), dev16(cp), d_da, d_dcp)
    gmag = np.abs(dh.astype(np.float64)) + np.abs(dcn.astype(np.float64))                        # terms of dc
    gmag4 = np.concatenate([gmag, gmag * np.abs(cp.astype(np.float64)), gmag, gmag], axis=1)
    _close16(host16(d_da), da, gmag4); _close16(host16(d_dcp), dcp, gmag)
    da0, dcp0 = lstm.lstm_cell_bwd(dh, np.zeros_like(dcn), act, c, cp)
    mpt.mpt_lstm_cell_bwd(dev16(dh), None, dev16(act), dev16(c), dev16(cp), d_da, d_dcp)       # last step: nothing carried
    _close16(host16(d_da), da0); _close16(host16(d_dcp), dcp0)


def test_in_place_state_and_strided_views():
    B, H = 9, 40
    gx, gr, bias, cp, dh, dcn = _inputs(B, H, 77)
    act, c, h = lstm.lstm_cell_fwd(gx, gr, None, cp)
    big = torch.zeros((B, 4 * H + 8), dtype=torch.float16, device="cuda"); big[:, :4 * H] = dev16(gx)
    state = dev16(cp)
    d_act, d_h = _e(B, 4 * H), _e(B, H)
    mpt.mpt_lstm_cell_fwd(big[:, :4 * H], dev16(gr), None, state, d_act, state, d_h)            # c written over c_prev
    _close16(host16(state), c, np.abs(cp.astype(np.float64)) + 1.0); _close16(host16(d_h), h, np.abs(cp.astype(np.float64)) + 1.0)
    # an odd column offset: element-wise path
    odd = torch.zeros((B, 4 * H + 3), dtype=torch.float16, device="cuda"); odd[:, 1:4 * H + 1] = dev16(gx)
    d_c = _e(B, H)
    mpt.mpt_lstm_cell_fwd(odd[:, 1:4 * H + 1], dev16(gr), None, dev16(cp), d_act, d_c, d_h)
    _close16(host16(d_c), c, np.abs(cp.astype(np.float64)) + 1.0); _close16(host16(d_act), act)
    carried = dev16(dcn)
    da, dcp = lstm.lstm_cell_bwd(dh, dcn, act, c, cp)
    d_da = _e(B, 4 * H)
    mpt.mpt_lstm_cell_bwd(dev16(dh), carried, dev16(act), dev16(c), dev16(cp), d_da, carried)   # dc_prev written over dc_next
    gm = np.abs(dh.astype(np.float64)) + np.abs(dcn.astype(np.float64))
    _close16(host16(carried), dcp, gm); _close16(host16(d_da), da, np.concatenate([gm, gm * np.abs(cp.astype(np.float64)), gm, gm], axis=1))


def test_free_running_projected_layer_on_device():
    """T steps with no host round trip: time-batched input product, then per step the recurrent product, the cell
    and the projection.  Errors of one FP16 step feed back through the recurrence, so the comparison with the
    oracle's free-running layer is loose; the per-step kernels are checked tightly above."""
    rng = np.random.default_rng(5)
    T, B, I, H, R = 6, 64, 256, 1024, 256
    x = rng.standard_normal((T, B, I)).astype(np.float16)
    Wx = (rng.standard_normal((I, 4 * H)) * 0.05).astype(np.float16)
    Wr = (rng.standard_normal((R, 4 * H)) * 0.05).astype(np.float16)
    Wp = (rng.standard_normal((H, R)) * 0.03).astype(np.float16)
    r0 = np.zeros((B, R), np.float16); c0 = np.zeros((B, H), np.float16)
    ref = lstm.lstmp_layer_fwd(x, Wx, Wr, Wp, None, r0, c0)
    d_x, d_Wx, d_Wr, d_Wp = dev16(x.reshape(T * B, I)), dev16(Wx), dev16(Wr), dev16(Wp)
    gx_all = _e(T * B, 4 * H)
    mpt.mpt_gemm_fwd(d_x, d_Wx, gx_all)
    r, c = dev16(r0), dev16(c0)
    gr, act, h = _e(B, 4 * H), _e(B, 4 * H), _e(B, H)
    ws = torch.empty(max(mpt.mpt_gemm_workspace_bytes(0, B, R, H), 16) // 4, dtype=torch.float32, device="cuda")
    for t in range(T):
        mpt.mpt_gemm_fwd(r, d_Wr, gr)
        mpt.mpt_lstm_cell_fwd(gx_all[t * B:(t + 1) * B], gr, None, c, act, c, h)
        r = _e(B, R)
        mpt.mpt_gemm_fwd(h, d_Wp, r, ws)                       # few output tiles, long reduction: split with the workspace
        got, want = host16(r).astype(np.float64), ref[t]["r"].astype(np.float64)
        assert np.isfinite(got).all()
        assert np.abs(got - want).max() <= 2e-3 * max(1.0, np.abs(want).max()), (t, np.abs(got - want).max())
        d = fp16.ulpdist16(fp16.bits(host16(r)), fp16.bits(ref[t]["r"]))
        assert (d <= 2).mean() > 0.9, (t, float((d <= 2).mean()))
    assert np.abs(ref[-1]["r"].astype(np.float64)).max() > 1e-2                                 # the layer is doing something
