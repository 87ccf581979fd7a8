"""Pins for the dynamic loss-scale policy (closed-form trajectories), the
scaled softmax cross-entropy (torch float64 autograd) and the MLP composition."""
import numpy as np
import torch

import workloads
from oracle import fp16, loss, mlp
from oracle.scaler import Scaler


def test_cfg5_closed_form():
    """J overflow steps among 200 with interval 1000: final scale 2^(16-J),
    200-J updates applied."""
    for J in (0, 1, 8):
        s = Scaler()
        bad = set(range(3, 3 + 7 * J, 7))
        applied = 0
        for t in range(200):
            ov = t in bad
            applied += not ov
            s.update(ov)
        assert s.scale == 2.0 ** (16 - J) and applied == 200 - J


def test_growth_hand_trajectory():
    s = Scaler(scale=4.0, growth_interval=3)
    seq = [0, 0, 0, 0, 1, 0, 0, 1, 0, 0, 0, 0]
    got = [s.update(o) for o in seq]
    #      c=1  2  grow  c=1  half  1    2    half 1    2    grow  1
    assert got == [4, 4, 8, 8, 4, 4, 4, 2, 2, 2, 4, 4]
    assert s.good_steps == 1


def test_clamps():
    s = Scaler(scale=2.0, min_scale=1.0)
    s.update(1); s.update(1); s.update(1)
    assert s.scale == 1.0
    s = Scaler(scale=2.0 ** 23, growth_interval=1)
    s.update(0); s.update(0); s.update(0)
    assert s.scale == 2.0 ** 24


def test_softmax_xent_against_torch_autograd():
    rng = np.random.default_rng(0)
    B, C, S = 32, 10, 1024.0
    z = (rng.standard_normal((B, C)) * 3).astype(np.float16)
    y = rng.integers(0, C, B)
    L, d = loss.softmax_xent_scaled(z, y, S)
    tz = torch.tensor(z.astype(np.float64), requires_grad=True)
    tl = torch.nn.functional.cross_entropy(tz, torch.tensor(y), reduction="mean")
    (tl * S).backward()
    assert abs(L - tl.item()) < 1e-12
    want = tz.grad.numpy().astype(np.float16)
    dist = fp16.ulpdist16(fp16.bits(d), fp16.bits(want))
    assert dist.max() <= 1 and (dist > 0).mean() < 0.02
    # rows of the unrounded gradient sum to zero; after rounding nearly so
    assert np.abs(fp16.to_f64(d).sum(axis=1)).max() < S / B * 2.0 ** -9
    # uniform logits: loss is ln C
    L0, _ = loss.softmax_xent_scaled(np.zeros((4, C), np.float16), np.zeros(4, int), 1.0)
    assert abs(L0 - np.log(C)) < 1e-15


def test_relu():
    y = np.array([-1.0, -0.0, 0.0, 2.0, np.inf], dtype=np.float16)
    assert np.array_equal(loss.relu_fwd(y), np.array([0, 0, 0, 2, np.inf], dtype=np.float16))
    d = np.array([5, 5, 5, 5, 5], dtype=np.float16)
    assert np.array_equal(loss.relu_bwd(d, y), np.array([0, 0, 0, 5, 5], dtype=np.float16))


def test_mlp_step_sanity():
    c = workloads.mlp(batch=32, d_in=64, d_hid=48, d_out=10)
    w1, w2, h1, h2 = c["w1_32"], c["w2_32"], c["w1_16"], c["w2_16"]
    losses = []
    for _ in range(5):
        o = mlp.mlp_step(c["x"], c["labels"], w1, w2, h1, h2, c["scale"], 0.2)
        w1, w2, h1, h2 = o["w1_32"], o["w2_32"], o["w1_16"], o["w2_16"]
        losses.append(o["loss"])
        assert o["flag"] == 0
    assert abs(losses[0] - np.log(10)) < 1.0
    assert losses[-1] < losses[0]


def test_workloads_are_seeded_and_shaped():
    a, b = workloads.square_gemm(64), workloads.square_gemm(64)
    assert all(np.array_equal(a[k], b[k]) for k in ("A", "B", "G"))
    assert a["A"].dtype == np.float16 and a["G"].shape == (64, 64)
    f = workloads.FlatUpdate(n=1003, steps=20, n_inject=3)
    assert len(f.inject_steps) == 3
    s = f.inject_steps[0]
    g = f.grad16(s, 65536.0)
    assert ((g.view(np.uint16) & 0x7C00) == 0x7C00).any()
    t = next(t for t in range(20) if t not in f.inject_steps)
    assert np.isfinite(f.grad16(t, 65536.0).astype(np.float32)).all()
    c = workloads.conv_block(batch=2, hw=5, c=8, kf=8)
    assert (c["x"] >= 0).all() and 0.3 < (c["dy"] == 0).mean() < 0.7
