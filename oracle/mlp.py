"""One mixed-precision training step of a two-layer perceptron, composed from
the oracle's parts in the order of the paper's iteration (Fig. 1 caption and
Sec. 3.1-3.3): FP16 copy -> forward -> scaled loss -> backward-activation and
backward-weight -> unscale + overflow check -> FP32 master update -> FP16 copy.
Test infrastructure only.  The paper prints no numbers for such a step; the
wiring is pinned stage by stage, and end to end, against FP64 autograd of the
same network (tests/test_oracle_mlp.py).
"""
from . import gemm, loss, update


def mlp_step(x16, labels, w1_32, w2_32, w1_16, w2_16, scale, lr):
    """Returns a dict of every intermediate (FP16 containers / FP32 arrays)."""
    inv = 1.0 / float(scale)
    y1, _ = gemm.gemm_fwd(x16, w1_16)
    h1 = loss.relu_fwd(y1)
    logits, _ = gemm.gemm_fwd(h1, w2_16)
    L, dlogits = loss.softmax_xent_scaled(logits, labels, scale)
    dw2, _ = gemm.gemm_wgrad(h1, dlogits)
    dh1, _ = gemm.gemm_dgrad(dlogits, w2_16)
    dy1 = loss.relu_bwd(dh1, y1)
    dw1, _ = gemm.gemm_wgrad(x16, dy1)
    flag = update.overflow_flag(dw1) | update.overflow_flag(dw2)
    w1n, _, w1h = update.master_update(w1_32, None, dw1, inv, lr, 0.0, flag, w1_16)
    w2n, _, w2h = update.master_update(w2_32, None, dw2, inv, lr, 0.0, flag, w2_16)
    return dict(y1=y1, h1=h1, logits=logits, loss=L, dlogits=dlogits, dw2=dw2,
                dh1=dh1, dy1=dy1, dw1=dw1, flag=flag,
                w1_32=w1n, w2_32=w2n, w1_16=w1h, w2_16=w2h)
