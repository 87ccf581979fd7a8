"""GPU parity for the composed workloads: the two-layer perceptron step (glue
kernels + GEMMs + update) and the projected-LSTM layer's GEMMs, against the
oracle.  Stages are teacher-forced: each GPU stage receives the oracle's FP16
inputs for that stage, so every comparison is per operation."""
import numpy as np
import pytest
import torch

import workloads
from oracle import fp16, gemm, loss, mlp, update
from paper_1710_03740_amd import binding as mpt
from gpu_util import dev, dev16, host, host16, gemm_check, C_ACC, U32

pytestmark = pytest.mark.gpu


def _empty16(*shape):
    return torch.full(shape, float("nan"), dtype=torch.float16, device="cuda")


def test_relu_and_softmax_glue():
    rng = np.random.default_rng(0)
    y = (rng.standard_normal(10007) * 2).astype(np.float16)
    y[:4] = [0.0, -0.0, np.inf, -np.inf]
    dh = rng.standard_normal(10007).astype(np.float16)
    h, dy = _empty16(10007), _empty16(10007)
    mpt.mpt_relu_fwd(dev16(y), h)
    mpt.mpt_relu_bwd(dev16(dh), dev16(y), dy)
    assert np.array_equal(fp16.bits(host16(h)), fp16.bits(loss.relu_fwd(y)))
    assert np.array_equal(fp16.bits(host16(dy)), fp16.bits(loss.relu_bwd(dh, y)))
    # unaligned views take the scalar path
    h2 = _empty16(10008)
    mpt.mpt_relu_fwd(dev16(y)[1:], h2[2:10008])
    assert np.array_equal(fp16.bits(host16(h2)[2:]), fp16.bits(loss.relu_fwd(y[1:])))
    for B, C, S in ((256, 10, 1024.0), (33, 1000, 128.0), (5, 4096, 1.0), (7, 512, 8.0), (9, 2048, 8.0), (6, 8192, 64.0),
                    (3, 32768, 64.0), (3, 40000, 64.0), (2, 65536, 64.0), (2, 131072, 64.0), (2, 70001, 64.0), (5, 1001, 16.0), (4, 8191, 16.0), (130, 24, 2.0)):
        z = (rng.standard_normal((B, C)) * 3).astype(np.float16)
        lab = rng.integers(0, C, B).astype(np.int32)
        lab[0], lab[-1] = 0, C - 1
        L, d = loss.softmax_xent_scaled(z, lab, S)
        d_d, d_L, d_R = _empty16(B, C), torch.zeros(1, dtype=torch.float32, device="cuda"), torch.zeros(B, dtype=torch.float32, device="cuda")
        mpt.mpt_softmax_xent_scaled(dev16(z), dev(lab), S, d_d, d_L, d_R)
        dist = fp16.ulpdist16(fp16.bits(host16(d_d)), fp16.bits(d))
        assert dist.max() <= 1 and (dist > 0).mean() < 0.02, (B, C, dist.max(), (dist > 0).mean())
        assert abs(float(d_L.item()) - L) < 2e-6 * max(1.0, abs(L))
        z64 = z.astype(np.float64); zs = z64 - z64.max(axis=1, keepdims=True)
        rows = np.log(np.exp(zs).sum(axis=1)) - zs[np.arange(B), lab]                  # -log p[label], the plain definition
        assert np.allclose(host(d_R), rows, rtol=2e-6, atol=2e-6)
    # the gradient alone (no loss requested) needs no row buffer; a strided view takes the element-wise path
    B, C = 9, 520
    z = (rng.standard_normal((B, C)) * 3).astype(np.float16); lab = rng.integers(0, C, B).astype(np.int32)
    _, d = loss.softmax_xent_scaled(z, lab, 4.0)
    zb = torch.zeros((B, C + 3), dtype=torch.float16, device="cuda"); zb[:, 1:C + 1] = dev16(z)
    db = torch.full((B, C + 3), 9.0, dtype=torch.float16, device="cuda")
    mpt.mpt_softmax_xent_scaled(zb[:, 1:C + 1], dev(lab), 4.0, db[:, 1:C + 1])
    out = host16(db)
    assert fp16.ulpdist16(fp16.bits(np.ascontiguousarray(out[:, 1:C + 1])), fp16.bits(d)).max() <= 1
    assert (out[:, 0] == 9.0).all() and (out[:, C + 1:] == 9.0).all()


def test_cfg1_mlp_step_teacher_forced():
    c = workloads.mlp()
    o = mlp.mlp_step(c["x"], c["labels"], c["w1_32"], c["w2_32"], c["w1_16"], c["w2_16"], c["scale"], c["lr"])
    x, w1, w2 = dev16(c["x"]), dev16(c["w1_16"]), dev16(c["w2_16"])
    S, inv = c["scale"], 1.0 / c["scale"]

    def chk(got, want16, a16, b16, op, label):
        ref = {"fwd": gemm.gemm_fwd, "dgrad": gemm.gemm_dgrad, "wgrad": gemm.gemm_wgrad}[op](a16, b16, full=True)
        assert np.array_equal(fp16.bits(ref[0]), fp16.bits(want16))
        gemm_check(host16(got), ref[0], ref[1], ref[2], "cfg1 " + label)

    y1 = _empty16(256, 1024); mpt.mpt_gemm_fwd(x, w1, y1)
    chk(y1, o["y1"], c["x"], c["w1_16"], "fwd", "fwd1")
    h1 = _empty16(256, 1024); mpt.mpt_relu_fwd(dev16(o["y1"]), h1)
    assert np.array_equal(fp16.bits(host16(h1)), fp16.bits(o["h1"]))
    logits = _empty16(256, 10); mpt.mpt_gemm_fwd(dev16(o["h1"]), w2, logits)          # N = 10: element-wise loader path
    chk(logits, o["logits"], o["h1"], c["w2_16"], "fwd", "fwd2")
    dlog, L, R = _empty16(256, 10), torch.zeros(1, dtype=torch.float32, device="cuda"), torch.zeros(256, dtype=torch.float32, device="cuda")
    mpt.mpt_softmax_xent_scaled(dev16(o["logits"]), dev(c["labels"]), S, dlog, L, R)
    dist = fp16.ulpdist16(fp16.bits(host16(dlog)), fp16.bits(o["dlogits"]))
    assert dist.max() <= 1 and abs(float(L.item()) - o["loss"]) < 1e-5
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    dw2 = _empty16(1024, 10); mpt.mpt_gemm_wgrad(dev16(o["h1"]), dev16(o["dlogits"]), dw2, flag=flag)
    chk(dw2, o["dw2"], o["h1"], o["dlogits"], "wgrad", "wgrad2")
    dh1 = _empty16(256, 1024); mpt.mpt_gemm_dgrad(dev16(o["dlogits"]), w2, dh1)
    chk(dh1, o["dh1"], o["dlogits"], c["w2_16"], "dgrad", "dgrad2")
    dy1 = _empty16(256, 1024); mpt.mpt_relu_bwd(dev16(o["dh1"]), dev16(o["y1"]), dy1)
    assert np.array_equal(fp16.bits(host16(dy1)), fp16.bits(o["dy1"]))
    dw1 = _empty16(1024, 1024); mpt.mpt_gemm_wgrad(x, dev16(o["dy1"]), dw1, flag=flag)
    chk(dw1, o["dw1"], c["x"], o["dy1"], "wgrad", "wgrad1")
    assert int(flag.item()) == o["flag"] == 0
    # update both tensors from the oracle's gradients: bit-exact masters and copies
    for g16, w32, w16, name in ((o["dw1"], c["w1_32"], c["w1_16"], "w1"), (o["dw2"], c["w2_32"], c["w2_16"], "w2")):
        d_w, d_h = dev(w32.reshape(-1).copy()), dev16(w16.reshape(-1).copy())
        mpt.mpt_unscale_check(dev16(g16.reshape(-1)), inv, flag)
        mpt.mpt_master_update(d_w, None, dev16(g16.reshape(-1)), d_h, inv, c["lr"], 0.0, flag)
        assert np.array_equal(host(d_w).view(np.uint32), o[name + "_32"].reshape(-1).view(np.uint32))
        assert np.array_equal(fp16.bits(host16(d_h)), fp16.bits(o[name + "_16"].reshape(-1)))


def test_cfg1_mlp_free_running_device_only():
    """Three whole steps on the device with no host round trip inside a step; compared loosely (errors of
    one FP16 step propagate) and for sanity: the loss falls."""
    c = workloads.mlp()
    x, lab = dev16(c["x"]), dev(c["labels"])
    w1_32, w2_32 = dev(c["w1_32"].copy()), dev(c["w2_32"].copy())
    w1, w2 = dev16(c["w1_16"]), dev16(c["w2_16"])
    S, inv, lr = c["scale"], 1.0 / c["scale"], 0.05
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    L = torch.zeros(1, dtype=torch.float32, device="cuda")
    R = torch.zeros(256, dtype=torch.float32, device="cuda")
    y1, h1, logits, dlog = _empty16(256, 1024), _empty16(256, 1024), _empty16(256, 10), _empty16(256, 10)
    dw2, dh1, dy1, dw1 = _empty16(1024, 10), _empty16(256, 1024), _empty16(256, 1024), _empty16(1024, 1024)
    ow = (c["w1_32"], c["w2_32"], c["w1_16"], c["w2_16"])
    losses, olosses = [], []
    for _ in range(3):
        mpt.mpt_gemm_fwd(x, w1, y1); mpt.mpt_relu_fwd(y1, h1); mpt.mpt_gemm_fwd(h1, w2, logits)
        mpt.mpt_softmax_xent_scaled(logits, lab, S, dlog, L, R)
        mpt.mpt_gemm_wgrad(h1, dlog, dw2, flag=flag); mpt.mpt_gemm_dgrad(dlog, w2, dh1)
        mpt.mpt_relu_bwd(dh1, y1, dy1); mpt.mpt_gemm_wgrad(x, dy1, dw1, flag=flag)
        mpt.mpt_master_update(w1_32, None, dw1, w1, inv, lr, 0.0, flag)
        mpt.mpt_master_update(w2_32, None, dw2, w2, inv, lr, 0.0, flag)
        losses.append(float(L.item()))
        o = mlp.mlp_step(c["x"], c["labels"], *ow, S, lr)
        ow = (o["w1_32"], o["w2_32"], o["w1_16"], o["w2_16"])
        olosses.append(o["loss"])
    assert int(flag.item()) == 0
    assert losses[-1] < losses[0] and abs(losses[0] - np.log(10)) < 0.8
    assert np.allclose(losses, olosses, rtol=2e-3)
    assert np.abs(host(w1_32) - ow[0]).max() < 1e-4 * np.abs(ow[0]).max() + 1e-6


def test_cfg1_mlp_step_replayed_from_a_hip_graph():
    """The library allocates nothing, never synchronises and clears its scratch with kernels, so a whole step can be
    captured once and replayed.  Three replays, with eager work of the same library and a synchronisation between them,
    must leave exactly the bits that three eager steps leave."""
    c = workloads.mlp()
    x, lab = dev16(c["x"]), dev(c["labels"])
    S, inv, lr = c["scale"], 1.0 / c["scale"], 0.05
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    L = torch.zeros(1, dtype=torch.float32, device="cuda")
    R = torch.zeros(256, dtype=torch.float32, device="cuda")
    h1, logits, dlog = _empty16(256, 1024), _empty16(256, 10), _empty16(256, 10)
    dw2, dy1, dw1 = _empty16(1024, 10), _empty16(256, 1024), _empty16(1024, 1024)
    w1_32, w2_32 = dev(c["w1_32"].copy()), dev(c["w2_32"].copy())
    w1, w2 = dev16(c["w1_16"]), dev16(c["w2_16"])
    ws = torch.empty(max([mpt.mpt_gemm_workspace_bytes(op, 256, n_, 1024) for op in (0, 1, 2) for n_ in (1024, 10)] + [16]) // 4,
                     dtype=torch.float32, device="cuda")

    def step():
        mpt.mpt_gemm_fwd_relu(x, w1, h1, ws); mpt.mpt_gemm_fwd(h1, w2, logits, ws)
        mpt.mpt_softmax_xent_scaled(logits, lab, S, dlog, L, R)
        mpt.mpt_gemm_wgrad(h1, dlog, dw2, flag=flag, ws=ws); mpt.mpt_gemm_dgrad_relu(dlog, w2, h1, dy1, ws)
        mpt.mpt_gemm_wgrad(x, dy1, dw1, flag=flag, ws=ws)
        mpt.mpt_master_update_multi(((w1_32, None, dw1, w1), (w2_32, None, dw2, w2)), inv, lr, 0.0, flag)   # both layers, one launch

    def reset():
        w1_32.copy_(dev(c["w1_32"].copy())); w2_32.copy_(dev(c["w2_32"].copy()))
        w1.copy_(dev16(c["w1_16"])); w2.copy_(dev16(c["w2_16"]))

    eager = []
    for _ in range(3):
        step()
        eager.append((host(w1_32).copy(), host(w2_32).copy(), float(L.item())))
    assert eager[2][2] < eager[0][2]
    reset()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                   # first use of every kernel happens outside the capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    reset()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        step()
    reset()
    scratch = _empty16(256, 1024)
    for k in range(3):
        g.replay()
        torch.cuda.synchronize()
        assert np.array_equal(host(w1_32).view(np.uint32), eager[k][0].view(np.uint32)), "replay %d" % k
        assert np.array_equal(host(w2_32).view(np.uint32), eager[k][1].view(np.uint32)), "replay %d" % k
        assert float(L.item()) == eager[k][2]
        mpt.mpt_gemm_fwd(x, w1, scratch, ws)     # eager work of the same library between replays
        torch.cuda.synchronize()
    assert int(flag.item()) == 0


@pytest.mark.parametrize("t", [0, 19])
def test_cfg3_lstmp_gemms_teacher_forced(t):
    c = workloads.lstmp(steps=20)
    Wg, Wp = dev16(c["Wg"]), dev16(c["Wp"])
    xh, h, dg, dr = c["xh"][t], c["h"][t], c["dgates"][t], c["dr"][t]
    B = xh.shape[0]
    ws = torch.empty(max(mpt.mpt_gemm_workspace_bytes(0, B, 32768, 2048), mpt.mpt_gemm_workspace_bytes(1, B, 32768, 2048),
                         mpt.mpt_gemm_workspace_bytes(0, B, 1024, 8192), mpt.mpt_gemm_workspace_bytes(1, B, 1024, 8192), 16) // 4,
                     dtype=torch.float32, device="cuda")
    gates = _empty16(B, 32768); mpt.mpt_gemm_fwd(dev16(xh), Wg, gates, ws)
    r = gemm.gemm_fwd(xh, c["Wg"], full=True); gemm_check(host16(gates), *r, "cfg3 gate fwd t=%d" % t)
    proj = _empty16(B, 1024); mpt.mpt_gemm_fwd(dev16(h), Wp, proj, ws)
    r = gemm.gemm_fwd(h, c["Wp"], full=True); gemm_check(host16(proj), *r, "cfg3 proj fwd")
    dxh = _empty16(B, 2048); mpt.mpt_gemm_dgrad(dev16(dg), Wg, dxh, ws)
    r = gemm.gemm_dgrad(dg, c["Wg"], full=True); gemm_check(host16(dxh), *r, "cfg3 gate dgrad")
    dh = _empty16(B, 8192); mpt.mpt_gemm_dgrad(dev16(dr), Wp, dh, ws)
    r = gemm.gemm_dgrad(dr, c["Wp"], full=True); gemm_check(host16(dh), *r, "cfg3 proj dgrad")


def test_cfg3_wgrad_over_timesteps():
    """Weight gradients summed over the 20 timesteps two ways: one time-batched contraction with an FP16
    store (rows of the 2048x32768 result sampled for the oracle), and per-timestep FP32 accumulation for
    the projection weights, which then feed the master update as FP32 gradients."""
    c = workloads.lstmp(steps=20)
    T, B = c["xh"].shape[:2]
    xh_all, dg_all = c["xh"].reshape(T * B, -1), c["dgates"].reshape(T * B, -1)
    ws = torch.empty(max(mpt.mpt_gemm_workspace_bytes(2, T * B, 32768, 2048), 16) // 4, dtype=torch.float32, device="cuda")
    dWg = _empty16(2048, 32768)
    mpt.mpt_gemm_wgrad(dev16(xh_all), dev16(dg_all), dWg, ws=ws)
    rows = np.random.default_rng(3).choice(2048, 96, replace=False)
    r = gemm.gemm_wgrad(np.ascontiguousarray(xh_all[:, rows]), dg_all, full=True)
    gemm_check(np.ascontiguousarray(host16(dWg)[rows]), *r, "cfg3 gate wgrad time-batched (96 sampled rows)")
    # projection weights: FP32 running sum across timesteps
    acc_dev = torch.zeros((8192, 1024), dtype=torch.float32, device="cuda")
    acc, sabs = None, 0.0
    for t in range(T):
        mpt.mpt_gemm_wgrad(dev16(c["h"][t]), dev16(c["dr"][t]), acc_dev, accumulate=(t > 0))
        acc, sa = gemm.gemm_wgrad(c["h"][t], c["dr"][t], out_fp32=True, acc32=acc)
        sabs = sabs + sa
    got = host(acc_dev)
    assert (np.abs(got.astype(np.float64) - acc.astype(np.float64)) <= C_ACC * U32 * sabs).all()
    # FP32 gradients into the master update
    w32 = c["Wp"].astype(np.float32).reshape(-1)
    d_w, d_h = dev(w32.copy()), dev16(c["Wp"].reshape(-1).copy())
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    inv = float(np.float32(1.0 / c["scale"]))
    mpt.mpt_unscale_check(acc_dev.view(-1), inv, flag)
    mpt.mpt_master_update(d_w, None, acc_dev.view(-1), d_h, inv, 0.01, 0.0, flag)
    wn, _, hn = update.master_update(w32, None, got.reshape(-1), inv, 0.01, 0.0, 0)
    assert int(flag.item()) == 0
    assert np.array_equal(host(d_w).view(np.uint32), wn.view(np.uint32))
    assert np.array_equal(fp16.bits(host16(d_h)), fp16.bits(hn))


def test_cfg3_all_timesteps_sampled_rows():
    """Every one of the 20 timesteps at the layer's own shapes (the test above compares whole outputs at the first
    and last step): gate and projection products, forward and activation gradient, teacher-forced with the step's
    operands; 16 seeded rows of each output are compared with the oracle by the GEMM acceptance rule."""
    c = workloads.lstmp(steps=20)
    Wg, Wp = dev16(c["Wg"]), dev16(c["Wp"])
    B = c["xh"].shape[1]
    ws = torch.empty(max(mpt.mpt_gemm_workspace_bytes(0, B, 32768, 2048), mpt.mpt_gemm_workspace_bytes(1, B, 32768, 2048),
                         mpt.mpt_gemm_workspace_bytes(0, B, 1024, 8192), mpt.mpt_gemm_workspace_bytes(1, B, 1024, 8192), 16) // 4,
                     dtype=torch.float32, device="cuda")
    gates, proj, dxh, dh = _empty16(B, 32768), _empty16(B, 1024), _empty16(B, 2048), _empty16(B, 8192)
    for t in range(20):
        rows = np.sort(np.random.default_rng(100 + t).choice(B, 16, replace=False))
        xh, h, dg, dr = c["xh"][t], c["h"][t], c["dgates"][t], c["dr"][t]
        print("cfg3 step", t, flush=True)
        mpt.mpt_gemm_fwd(dev16(xh), Wg, gates, ws)
        mpt.mpt_gemm_fwd(dev16(h), Wp, proj, ws)
        mpt.mpt_gemm_dgrad(dev16(dg), Wg, dxh, ws)
        mpt.mpt_gemm_dgrad(dev16(dr), Wp, dh, ws)
        for got, ref, label in ((gates, gemm.gemm_fwd(xh[rows], c["Wg"], full=True), "gate fwd"), (proj, gemm.gemm_fwd(h[rows], c["Wp"], full=True), "proj fwd"),
                                (dxh, gemm.gemm_dgrad(dg[rows], c["Wg"], full=True), "gate dgrad"), (dh, gemm.gemm_dgrad(dr[rows], c["Wp"], full=True), "proj dgrad")):
            gemm_check(np.ascontiguousarray(host16(got)[rows]), *ref, "cfg3 %s t=%d (16 rows)" % (label, t))


def test_cfg3_gate_wgrad_per_timestep_fp32_accumulation():
    """The gate weights' gradient at its own per-timestep shape (2048 x 32768 output, reduction over the batch of 256),
    accumulated in FP32 over all 20 timesteps; 24 seeded rows of the 2048 are followed by the oracle.  Allowance per
    element: the accumulation allowance of every step's product plus one FP32 rounding of the running sum per step."""
    c = workloads.lstmp(steps=20)
    T = c["xh"].shape[0]
    rows = np.sort(np.random.default_rng(7).choice(2048, 24, replace=False))
    acc_dev = torch.full((2048, 32768), float("nan"), dtype=torch.float32, device="cuda")
    acc, allow = None, 0.0
    for t in range(T):
        mpt.mpt_gemm_wgrad(dev16(c["xh"][t]), dev16(c["dgates"][t]), acc_dev, accumulate=(t > 0))
        acc, sa = gemm.gemm_wgrad(np.ascontiguousarray(c["xh"][t][:, rows]), c["dgates"][t], out_fp32=True, acc32=acc)
        allow = allow + C_ACC * U32 * sa + U32 * np.abs(acc.astype(np.float64))
    got = host(acc_dev)[rows].astype(np.float64)
    err = np.abs(got - acc.astype(np.float64))
    print("[cfg3 gate wgrad per step] worst error / allowance = %.3f" % float((err / allow).max()), flush=True)
    assert (err <= allow).all()
    assert np.isfinite(host(acc_dev)).all()


def test_conv_batchnorm_relu_block_teacher_forced():
    """A residual-network style block on the device: 3x3 convolution -> batch-norm statistics -> normalise + ReLU,
    then its backward pass (ReLU mask, batch-norm reductions and input gradient, convolution gradients).  Every stage is
    fed the oracle's FP16 tensors for the stage before (bit-identical inputs) and compared at that stage's own bar."""
    from oracle import conv, norm
    rng = np.random.default_rng(31)
    Nb, H, W, C, Kf = 16, 14, 14, 64, 256                       # 3136 pixels: whole 128-row tiles for the convolution
    S = 256.0
    x = np.maximum(rng.standard_normal((Nb, H, W, C)), 0).astype(np.float16)
    w = (rng.standard_normal((Kf, 3, 3, C)) * np.sqrt(2.0 / (9 * C))).astype(np.float16)
    gamma = rng.uniform(0.5, 1.5, Kf).astype(np.float32); beta = rng.uniform(-0.5, 0.5, Kf).astype(np.float32)
    dz = (rng.standard_normal((Nb, H, W, Kf)) * 2.0 ** -9 * S).astype(np.float16)          # upstream gradient, loss-scaled
    P = Nb * H * W
    # ---- forward
    y_o, sa, s = conv.conv3x3_fwd(x, w, full=True)
    y = _empty16(Nb, H, W, Kf); mpt.mpt_conv3x3_fwd(dev16(x), dev16(w), y)
    gemm_check(host16(y), y_o, sa, s, "block conv fwd")
    y2 = y_o.reshape(P, Kf)
    mean = torch.empty(Kf, dtype=torch.float32, device="cuda"); var = torch.empty_like(mean)
    ws = torch.empty(max(mpt.mpt_bn_workspace_bytes(P, Kf), 16) // 8, dtype=torch.float64, device="cuda")
    mpt.mpt_bn_stats(dev16(y2), mean, var, ws)
    m_o, v_o = norm.bn_stats(y2)
    assert np.allclose(host(mean), m_o, rtol=1e-5, atol=1e-6) and np.allclose(host(var), v_o, rtol=1e-4, atol=1e-8)
    m32, v32 = m_o.astype(np.float32), v_o.astype(np.float32)
    z = _empty16(P, Kf); mpt.mpt_bn_apply(dev16(y2), dev(m32), dev(v32), dev(gamma), dev(beta), 1e-5, z, relu=True)
    z_o = norm.bn_apply(y2, m32, v32, gamma, beta, 1e-5, relu=True)
    assert np.array_equal(fp16.bits(host16(z)), fp16.bits(z_o))
    # ---- backward
    dz2 = dz.reshape(P, Kf)
    da = _empty16(P, Kf); mpt.mpt_relu_bwd(dev16(dz2), dev16(z_o), da)                       # z > 0 exactly where the pre-activation was
    da_o = loss.relu_bwd(dz2, z_o)
    assert np.array_equal(fp16.bits(host16(da)), fp16.bits(da_o))
    dg = torch.empty(Kf, dtype=torch.float32, device="cuda"); db = torch.empty_like(dg)
    mpt.mpt_bn_bwd_reduce(dev16(y2), dev16(da_o), dev(m32), dev(v32), 1e-5, dg, db, ws)
    dg_o, db_o = norm.bn_bwd_reduce(y2, da_o, m32, v32, 1e-5)
    scale_g = np.abs(da_o.astype(np.float64)).sum(axis=0) * 8                                # |xhat| stays below ~8 here
    assert (np.abs(host(dg) - dg_o) <= 20 * 2.0 ** -24 * scale_g + 1e-12).all()
    assert (np.abs(host(db) - db_o) <= 20 * 2.0 ** -24 * np.abs(da_o.astype(np.float64)).sum(axis=0) + 1e-12).all()
    dg32, db32 = dg_o.astype(np.float32), db_o.astype(np.float32)
    dy = _empty16(P, Kf); mpt.mpt_bn_bwd_apply(dev16(y2), dev16(da_o), dev(m32), dev(v32), dev(gamma), 1e-5, dev(dg32), dev(db32), dy)
    dy_o = norm.bn_bwd_apply(y2, da_o, m32, v32, gamma, 1e-5, dg32, db32)
    assert np.array_equal(fp16.bits(host16(dy)), fp16.bits(dy_o))
    dy4 = dy_o.reshape(Nb, H, W, Kf)
    dx = _empty16(Nb, H, W, C); mpt.mpt_conv3x3_dgrad(dev16(dy4), dev16(w), dx)
    o, sa, s = conv.conv3x3_dgrad(dy4, w, full=True)
    gemm_check(host16(dx), o, sa, s, "block conv dgrad")
    flag = torch.zeros(1, dtype=torch.int32, device="cuda")
    dw = _empty16(Kf, 3, 3, C)
    b = mpt.mpt_conv3x3_workspace_bytes(2, Nb, H, W, C, Kf)
    wsw = torch.empty(max(b, 16) // 4, dtype=torch.float32, device="cuda") if b else None
    mpt.mpt_conv3x3_wgrad(dev16(x), dev16(dy4), dw, flag, wsw)
    o, sa, s = conv.conv3x3_wgrad(x, dy4, full=True)
    gemm_check(host16(dw), o, sa, s, "block conv wgrad")
    assert int(flag.item()) == 0
    # the scaled weight gradient goes through the usual unscale + update
    wm = w.astype(np.float32).reshape(-1); mom = np.zeros_like(wm)
    rw, rm, rh = update.master_update(wm, mom, o.reshape(-1), 1.0 / S, 0.01, 0.9, 0)
    d_w, d_m, d_h = dev(wm.copy()), dev(mom.copy()), dev16(w.reshape(-1).copy())
    mpt.mpt_master_update(d_w, d_m, dev16(o.reshape(-1)), d_h, 1.0 / S, 0.01, 0.9, flag)
    assert np.array_equal(host(d_w).view(np.uint32), rw.view(np.uint32)) and np.array_equal(fp16.bits(host16(d_h)), fp16.bits(rh))
