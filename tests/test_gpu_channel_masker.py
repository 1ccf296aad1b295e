"""GPU parity of the channel masker (GAP + 2-layer MLP + argmax) and of the chain
masker -> channel-skipping bottleneck, against the CPU oracle."""
import numpy as np
import pytest

from oracle import laud_oracle as O
from paper_2308_15949_amd import inputs as I

pytestmark = pytest.mark.gpu

CASES = [
    # N, H, W, C, D, dtype
    (3, 5, 7, 40, 4, I.F32),       # C/4 = 10 chunk columns: idle threads, ragged slabs
    (4, 7, 7, 2048, 4, I.BF16),    # stage 4: 256 chunk columns
    (6, 14, 14, 1024, 128, I.BF16),  # G = 2 (the paper's granularity) on mid 256
    (2, 56, 56, 256, 64, I.BF16),  # stage 1, G = 1
    (64, 14, 14, 1024, 4, I.BF16),  # config 4, stage 3
    (2, 4, 4, 4104, 8, I.F32),     # more chunk columns than threads
]


@pytest.mark.parametrize("case", CASES)
def test_channel_masker(case):
    import torch as t
    import paper_2308_15949_amd as L
    from paper_2308_15949_amd import device as D_
    N, H, W, C, D, dt = case
    x = I.feature_map(300 + C + N, N, H, W, C, dt)
    wa, ba, wb, bb, hidden = I.channel_masker_weights(301 + D, C, D)
    assert hidden == O.channel_masker_hidden(D)
    ref = O.channel_masker_logits(x, wa, ba, wb, bb)
    xd = D_.to_device(x, dt)
    fx = L.fmap_of(xd)
    dev = lambda a: t.from_numpy(a).cuda()
    cmask = t.full((N, D), 9, dtype=t.uint8, device="cuda")
    lg = t.full((N, 2 * D), float("nan"), dtype=t.float32, device="cuda")
    ws = D_.workspace(L.channel_masker_workspace(fx))
    L.laud_channel_masker(xd, fx, dev(wa), dev(ba), hidden, dev(wb), dev(bb), D, cmask, lg, ws)
    t.cuda.synchronize()
    got = lg.cpu().numpy().reshape(N, D, 2)
    scale = float(np.sqrt(np.mean(ref * ref))) + 1e-6
    assert np.abs(got - ref).max() <= 2e-5 * scale + 1e-6          # float32 sums of H*W*C and C terms
    gm = cmask.cpu().numpy()
    sure = np.abs(ref[..., 0] - ref[..., 1]) > 1e-4 * scale
    assert np.array_equal(gm[sure], O.channel_mask_from_logits(ref)[sure])
    assert sure.mean() > 0.97 and set(np.unique(gm)) <= {0, 1}
    # decisions are exactly the argmax of the logits the GPU itself produced
    assert np.array_equal(gm, (got[..., 0] > got[..., 1]).astype(np.uint8))


def test_channel_masker_feeds_channel_skip_conv():
    import torch as t
    import paper_2308_15949_amd as L
    from paper_2308_15949_amd import device as D_
    N, H, C, m, D, dt = 8, 14, 256, 64, 4, I.BF16
    x = I.feature_map(320, N, H, H, C, dt)
    hb = I.bottleneck_params(321, C, m, C, dt, relu_out=True)
    wa, ba, wb, bb, hidden = I.channel_masker_weights(322, C, D)
    xd = D_.to_device(x, dt)
    fx = L.fmap_of(xd)
    db = D_.DeviceBottleneck(hb)
    dev = lambda a: t.from_numpy(a).cuda()
    cmask = t.zeros((N, D), dtype=t.uint8, device="cuda")
    L.laud_channel_masker(xd, fx, dev(wa), dev(ba), hidden, dev(wb), dev(bb), D, cmask, None,
                          D_.workspace(L.channel_masker_workspace(fx)))
    ws = D_.workspace(L.workspace_size(L.binding.OP_CHANNEL_SKIP, fx, db.desc, D))
    L.laud_channel_skip_conv(xd, fx, db.desc, cmask, D, xd, ws)
    t.cuda.synchronize()
    gm = cmask.cpu().numpy()
    p = O.BottleneckParams(hb.w1, hb.w2, hb.w3, hb.s1, hb.t1, hb.s2, hb.t2, hb.s3, hb.t3, hb.relu_out)
    lr = O.channel_masker_logits(x, wa, ba, wb, bb)
    ref_mask = O.channel_mask_from_logits(lr)
    # no decision of this seeded case lies within float32 rounding of a tie, so the GPU's mask is the oracle's
    assert (np.abs(lr[..., 0] - lr[..., 1]) > 1e-4 * float(np.sqrt(np.mean(lr * lr)))).all()
    assert np.array_equal(gm, ref_mask)
    ref = O.channel_skip_bottleneck(x, p, ref_mask)
    got = D_.to_host(xd).astype(np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    assert np.all(np.abs(got - ref) <= 2e-2 * (np.abs(ref) + rms))
    assert 0 < gm.sum() < gm.size
