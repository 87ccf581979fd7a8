"""Pins of the LSTM-cell oracle: closed forms, a library routine (torch.nn.LSTMCell in FP64 with its autograd), and
the layer as a composition of pinned parts."""
import numpy as np
import torch

from oracle import lstm, fp16, gemm


def _f16(a):
    return np.asarray(a, dtype=np.float64).astype(np.float16)


def test_closed_forms():
    B, H = 2, 3
    z = np.zeros((B, 4 * H), np.float16)
    cp = _f16([[1.0, -2.0, 0.5], [0.0, 0.25, 4.0]])
    act, c, h = lstm.lstm_cell_fwd(z, z, None, cp)
    a = act.astype(np.float64)
    assert (a[:, :2 * H] == 0.5).all() and (a[:, 2 * H:3 * H] == 0).all() and (a[:, 3 * H:] == 0.5).all()
    assert np.array_equal(c, _f16(0.5 * cp.astype(np.float64)))                     # c = f * c_prev with f = 1/2, i * g = 0
    assert np.array_equal(h, _f16(0.5 * np.tanh(0.5 * cp.astype(np.float64))))
    # saturated gates: forget open, input closed -> state carried; output closed -> h = 0
    big = np.zeros((B, 4 * H), np.float16); big[:, H:2 * H] = 30.0; big[:, :H] = -30.0; big[:, 3 * H:] = -30.0
    act, c, h = lstm.lstm_cell_fwd(big, z, None, cp)
    assert np.array_equal(c, cp) and not h.astype(np.float64).any()
    # the bias is added to the sum of the two pre-activations
    b = np.zeros(4 * H, np.float32); b[2 * H:3 * H] = 1.0; b[:H] = 30.0
    act, c, _ = lstm.lstm_cell_fwd(z, z, b, np.zeros((B, H), np.float16))
    assert np.allclose(c.astype(np.float64), np.tanh(1.0), rtol=1e-3)


def _torch_cell(a64, cprev64):
    H = cprev64.shape[1]
    cell = torch.nn.LSTMCell(4 * H, H, bias=False, dtype=torch.float64)
    with torch.no_grad():
        cell.weight_ih.copy_(torch.eye(4 * H, dtype=torch.float64))                 # gates = the given pre-activations
        cell.weight_hh.zero_()
    a = torch.tensor(a64, requires_grad=True); cp = torch.tensor(cprev64, requires_grad=True)
    h, c = cell(a, (torch.zeros_like(cp), cp))
    return a, cp, h, c


def test_forward_and_backward_against_torch_lstmcell():
    rng = np.random.default_rng(0)
    B, H = 5, 7
    gx = _f16(rng.standard_normal((B, 4 * H)) * 2); gr = _f16(rng.standard_normal((B, 4 * H)))
    cp = _f16(rng.standard_normal((B, H)))
    act, c, h = lstm.lstm_cell_fwd(gx, gr, None, cp)
    a64 = gx.astype(np.float64) + gr.astype(np.float64)
    a, cpt, ht, ct = _torch_cell(a64, cp.astype(np.float64))
    assert np.array_equal(fp16.bits(c), fp16.bits(fp16.rne16(ct.detach().numpy())))
    assert np.array_equal(fp16.bits(h), fp16.bits(fp16.rne16(ht.detach().numpy())))
    # backward: feed the cell's own unrounded activations through the oracle's formulas by storing them as FP16
    # inputs that are exact: use the oracle on FP16-exact activations and compare with autograd on the same point
    dh = _f16(rng.standard_normal((B, H)) * 0.1); dcn = _f16(rng.standard_normal((B, H)) * 0.1)
    (ht * torch.tensor(dh.astype(np.float64))).sum().backward(retain_graph=True)
    # autograd gives d/da of <dh, h> with dc_next = 0; add the carried term separately
    da_h = a.grad.clone(); dcp_h = cpt.grad.clone()
    a.grad.zero_(); cpt.grad.zero_()
    (ct * torch.tensor(dcn.astype(np.float64))).sum().backward()
    da_ref = (da_h + a.grad).numpy(); dcp_ref = (dcp_h + cpt.grad).numpy()
    da, dcp = lstm.lstm_cell_bwd(dh, dcn, act, c, cp)
    # the oracle differentiates at the FP16-stored activations, autograd at the unrounded ones: agreement to FP16 accuracy
    assert np.allclose(da.astype(np.float64), da_ref, rtol=4e-3, atol=2e-4)
    assert np.allclose(dcp.astype(np.float64), dcp_ref, rtol=4e-3, atol=2e-4)


def test_backward_exact_point():
    """At gates = 0 and c = 0 everything is closed-form: i = f = o = 1/2, g = 0, tanh(c) = 0."""
    B, H = 1, 2
    act = np.concatenate([np.full((B, H), 0.5), np.full((B, H), 0.5), np.zeros((B, H)), np.full((B, H), 0.5)], axis=1).astype(np.float16)
    c = np.zeros((B, H), np.float16); cp = _f16([[2.0, -4.0]])
    dh = _f16([[1.0, 0.5]]); dcn = _f16([[0.25, 0.0]])
    da, dcp = lstm.lstm_cell_bwd(dh, dcn, act, c, cp)
    dc = dh.astype(np.float64) * 0.5 + dcn.astype(np.float64)                      # dh * o * (1 - 0) + dc_next
    want = np.concatenate([np.zeros((B, H)), dc * cp.astype(np.float64) * 0.25, dc * 0.5, np.zeros((B, H))], axis=1)
    assert np.array_equal(da.astype(np.float64), want)
    assert np.array_equal(dcp.astype(np.float64), dc * 0.5)


def test_layer_is_the_composition_of_cell_and_contractions():
    rng = np.random.default_rng(1)
    T, B, I, H, R = 3, 4, 6, 5, 3
    x = _f16(rng.standard_normal((T, B, I))); Wx = _f16(rng.standard_normal((I, 4 * H)) * 0.3)
    Wr = _f16(rng.standard_normal((R, 4 * H)) * 0.3); Wp = _f16(rng.standard_normal((H, R)) * 0.3)
    r = np.zeros((B, R), np.float16); c = np.zeros((B, H), np.float16)
    out = lstm.lstmp_layer_fwd(x, Wx, Wr, Wp, None, r, c)
    for t in range(T):
        gx, _ = gemm.gemm_fwd(x[t], Wx)
        assert np.array_equal(fp16.bits(gx), fp16.bits(out[t]["gx"]))              # time-batching changes nothing per row
        gr, _ = gemm.gemm_fwd(r, Wr)
        act, c, h = lstm.lstm_cell_fwd(gx, gr, None, c)
        r, _ = gemm.gemm_fwd(h, Wp)
        assert np.array_equal(fp16.bits(r), fp16.bits(out[t]["r"])) and np.array_equal(fp16.bits(c), fp16.bits(out[t]["c"]))
    assert np.abs(out[-1]["r"].astype(np.float64)).max() > 0


def _torch_layer(x, Wx, Wr, Wp, bias, r0, c0):
    """The same layer in FP64 torch, nothing rounded: returns the lists of r_t and c_t."""
    T = x.shape[0]
    H = Wp.shape[0]
    r, c, rs, cs = r0, c0, [], []
    for t in range(T):
        a = x[t] @ Wx + r @ Wr + bias
        i, f, o = torch.sigmoid(a[:, :H]), torch.sigmoid(a[:, H:2 * H]), torch.sigmoid(a[:, 3 * H:])
        g = torch.tanh(a[:, 2 * H:3 * H])
        c = f * c + i * g
        r = (o * torch.tanh(c)) @ Wp
        rs.append(r); cs.append(c)
    return rs, cs


def test_backward_through_time_against_fp64_autograd():
    """lstmp_layer_bwd against autograd of the un-rounded FP64 layer with the loss sum_t <dr_ext_t, r_t> + <dc_last, c_T>,
    whose gradient with respect to r_t is exactly dr_ext_t.  The oracle stores FP16 at every stage, so agreement is to
    FP16 accuracy; a structural mistake (recurrent gradient not carried, the state gradient dropped, W_r and W_p
    confused or not transposed, c_{t-1} taken from the wrong step, the time-batched sums missing a step) is off by
    tens of percent.  Planted versions of three such mistakes are shown to fail the same comparison."""
    rng = np.random.default_rng(11)
    T, B, I, H, P = 5, 6, 10, 12, 8
    x = _f16(rng.standard_normal((T, B, I)))
    Wx, Wr, Wp = _f16(rng.uniform(-0.4, 0.4, (I, 4 * H))), _f16(rng.uniform(-0.4, 0.4, (P, 4 * H))), _f16(rng.uniform(-0.5, 0.5, (H, P)))
    bias = rng.uniform(-0.2, 0.2, 4 * H).astype(np.float32)
    r0, c0 = _f16(rng.standard_normal((B, P)) * 0.5), _f16(rng.standard_normal((B, H)) * 0.5)
    dr_ext = _f16(rng.standard_normal((T, B, P)) * 0.25)
    dc_last = _f16(rng.standard_normal((B, H)) * 0.25)
    fwd = lstm.lstmp_layer_fwd(x, Wx, Wr, Wp, bias, r0, c0)
    out = lstm.lstmp_layer_bwd(x, Wx, Wr, Wp, r0, c0, fwd, dr_ext, dc_last)

    t = lambda a: torch.from_numpy(np.asarray(a, dtype=np.float64)).requires_grad_(True)
    tx, tWx, tWr, tWp, tb, tr0, tc0 = t(x), t(Wx), t(Wr), t(Wp), t(bias), t(r0), t(c0)
    rs, cs = _torch_layer(tx, tWx, tWr, tWp, tb, tr0, tc0)
    loss = sum((torch.from_numpy(dr_ext[k].astype(np.float64)) * rs[k]).sum() for k in range(T)) + (torch.from_numpy(dc_last.astype(np.float64)) * cs[-1]).sum()
    loss.backward()
    # forward first: the stored r_t follow the FP64 layer to FP16 accuracy
    for k in range(T):
        assert np.abs(fwd[k]["r"].astype(np.float64) - rs[k].detach().numpy()).max() < 2.0 ** -7

    def close(got, want, name, tol=2.0 ** -6):
        got, want = np.asarray(got, dtype=np.float64), want.numpy()
        err = np.abs(got - want).max() / np.abs(want).max()
        assert err < tol, (name, err)
        return err

    pairs = (("dx", tx), ("dWx", tWx), ("dWr", tWr), ("dWp", tWp), ("dbias", tb), ("dr0", tr0), ("dc0", tc0))
    for name, ten in pairs:
        close(out[name], ten.grad, name)

    def wrong(mutate):
        bad = mutate()
        return max(np.abs(np.asarray(bad[n], dtype=np.float64) - ten.grad.numpy()).max() / np.abs(ten.grad.numpy()).max() for n, ten in pairs)

    # planted mistakes, each in a copy of the routine's inputs / structure
    assert wrong(lambda: lstm.lstmp_layer_bwd(x, Wx, Wr, Wp, r0, c0, fwd, dr_ext, None)) > 0.05                      # state gradient dropped
    shifted = [fwd[0]] + fwd[:-1]
    assert wrong(lambda: lstm.lstmp_layer_bwd(x, Wx, Wr, Wp, r0, c0, shifted, dr_ext, dc_last)) > 0.05              # stored tensors of the wrong step
    assert wrong(lambda: lstm.lstmp_layer_bwd(x, Wx, np.zeros_like(Wr), Wp, r0, c0, fwd, dr_ext, dc_last)) > 0.05   # recurrent gradient not carried
