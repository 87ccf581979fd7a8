"""Pin for the wiring of oracle.mlp.mlp_step (the composition of the paper's iteration, Fig. 1 caption and
Sec. 3.1-3.3) against torch's FP64 autograd of the same two-layer network.

Two views.  (1) Stage by stage from the oracle's own stored FP16 tensors: every intermediate must be the FP16 rounding
of the FP64 value torch computes for that stage alone - within one FP16 step.  This catches a forgotten ReLU mask,
a transposed operand, a wrong sign, a loss scale applied twice or not at all, a mean taken as a sum.  (2) End to
end: the unscaled weight gradients and the updated masters agree with the un-rounded FP64 network to the accuracy
FP16 storage allows."""
import numpy as np
import torch

import workloads
from oracle import fp16, mlp

F64 = torch.float64


def t64(a16):
    return torch.from_numpy(fp16.to_f64(a16))


def steps16(got16, want64):
    return fp16.ulpdist16(fp16.bits(got16), fp16.bits(fp16.rne16(want64)))


def test_each_stage_is_the_fp16_rounding_of_its_fp64_definition():
    c = workloads.mlp(batch=32, d_in=64, d_hid=48, d_out=10)
    S, lr, B = c["scale"], 0.05, 32
    o = mlp.mlp_step(c["x"], c["labels"], c["w1_32"], c["w2_32"], c["w1_16"], c["w2_16"], S, lr)
    x, w1, w2 = t64(c["x"]), t64(c["w1_16"]), t64(c["w2_16"])
    lab = torch.from_numpy(c["labels"].astype(np.int64))
    # forward stages
    assert steps16(o["y1"], (x @ w1).numpy()).max() <= 1
    assert np.array_equal(fp16.bits(o["h1"]), fp16.bits(fp16.rne16(torch.relu(t64(o["y1"])).numpy())))
    assert steps16(o["logits"], (t64(o["h1"]) @ w2).numpy()).max() <= 1
    # scaled loss gradient from the stored logits (mean over the batch, times S)
    z = t64(o["logits"]).requires_grad_(True)
    L = torch.nn.functional.cross_entropy(z, lab, reduction="mean")
    (S * L).backward()
    assert abs(o["loss"] - float(L.detach())) < 1e-12
    assert steps16(o["dlogits"], z.grad.numpy()).max() <= 1
    # backward stages from the stored tensors: dW2 = h1^T dlogits, dh1 = dlogits W2^T, ReLU mask from y1, dW1 = x^T dy1
    dl = t64(o["dlogits"])
    assert steps16(o["dw2"], (t64(o["h1"]).T @ dl).numpy()).max() <= 1
    assert steps16(o["dh1"], (dl @ w2.T).numpy()).max() <= 1
    y1 = t64(o["y1"]).requires_grad_(True)
    torch.relu(y1).backward(t64(o["dh1"]))
    assert np.array_equal(fp16.bits(o["dy1"]), fp16.bits(fp16.rne16(y1.grad.numpy())))
    masked = (fp16.to_f64(o["y1"]) <= 0)
    assert masked.any() and (fp16.to_f64(o["dy1"])[masked] == 0).all() and (fp16.to_f64(o["dy1"])[~masked] != 0).any()
    assert steps16(o["dw1"], (x.T @ t64(o["dy1"])).numpy()).max() <= 1
    # update from the stored gradients: w' = w - lr * (dw / S) in FP32, FP16 copy of the result
    assert o["flag"] == 0
    for wn, w0, dw, hn in ((o["w1_32"], c["w1_32"], o["dw1"], o["w1_16"]), (o["w2_32"], c["w2_32"], o["dw2"], o["w2_16"])):
        want = w0.astype(np.float64) - lr * fp16.to_f64(dw) / S
        assert np.abs(wn.astype(np.float64) - want).max() <= 2.0 ** -23 * np.abs(want).max()
        assert np.array_equal(fp16.bits(hn), fp16.bits(fp16.rne16(wn.astype(np.float64))))


def test_whole_step_against_the_unrounded_fp64_network():
    c = workloads.mlp(batch=32, d_in=64, d_hid=48, d_out=10)
    S, lr = c["scale"], 0.05
    o = mlp.mlp_step(c["x"], c["labels"], c["w1_32"], c["w2_32"], c["w1_16"], c["w2_16"], S, lr)
    x = t64(c["x"])
    w1 = t64(c["w1_16"]).requires_grad_(True)
    w2 = t64(c["w2_16"]).requires_grad_(True)
    lab = torch.from_numpy(c["labels"].astype(np.int64))
    L = torch.nn.functional.cross_entropy(torch.relu(x @ w1) @ w2, lab, reduction="mean")
    L.backward()
    assert abs(o["loss"] - float(L.detach())) < 2e-3
    for dw16, g in ((o["dw1"], w1.grad.numpy()), (o["dw2"], w2.grad.numpy())):
        got = fp16.to_f64(dw16) / S                                     # unscaled
        assert np.abs(got - g).max() <= 2.0 ** -8 * np.abs(g).max()    # FP16 storage of three chained tensors
        assert np.corrcoef(got.ravel(), g.ravel())[0, 1] > 0.9999
    for wn, w0, g in ((o["w1_32"], c["w1_32"], w1.grad.numpy()), (o["w2_32"], c["w2_32"], w2.grad.numpy())):
        want = w0.astype(np.float64) - lr * g
        assert np.abs(wn - want).max() <= lr * 2.0 ** -8 * np.abs(g).max() + 2.0 ** -23
