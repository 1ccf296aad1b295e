"""Host tests of the latency predictor (Sec. 3.3, App. A): its shape arithmetic against the oracle's
closed forms, its structural properties, and the hardware table the paper prints."""
import dataclasses
import os

import numpy as np
import pytest

from oracle import laud_oracle as O
from paper_2308_15949_amd import predictor as P

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def test_flops_match_the_closed_forms():
    n, hw, c, m = 4, 14, 1024, 256
    macs = sum(O.conv_macs_per_pixel(c, m, c))
    p = P.predict_block(P.MI355X, "static", n=n, hw_px=hw, c_in=c, m=m)
    assert p["flops"] == pytest.approx(2.0 * macs * n * hw * hw)
    # spatial skipping: conv1 on the dilated set, conv2 / conv3 on the active set (Sec. 3.2 FLOP model)
    r, rd = 0.5, 0.75
    p = P.predict_block(P.MI355X, "spatial", n=n, hw_px=hw, c_in=c, m=m, S=2, r=r, r_dil=rd, fused_masker=False,
                        with_masker=False)
    want = O.spatial_flops_ratio(r, rd, c, m, c) * 2.0 * macs * n * hw * hw
    assert p["flops"] == pytest.approx(want, rel=1e-3)
    # channel skipping: r on the two 1x1 convs, r^2 on the 3x3
    p = P.predict_block(P.MI355X, "channel", n=n, hw_px=hw, c_in=c, m=m, r=0.5)
    assert p["flops"] == pytest.approx(O.channel_flops_ratio(0.5, c, m, c) * 2.0 * macs * n * hw * hw)


@pytest.mark.parametrize("S", [1, 2, 4, 7])
@pytest.mark.parametrize("r", [0.2, 0.5, 0.8])
def test_expected_dilated_ratio_against_the_oracle_on_random_masks(S, r):
    g = np.random.default_rng(10 * S + int(10 * r))
    hp = 224 // S   # a large grid: the border's share is small
    mask = (g.random((4, hp, hp)) < r).astype(np.uint8)
    got = O.dilated_ratio(mask, S)
    assert abs(P.expected_dilated_ratio(r, S) - got) < 0.02


def test_structure_of_the_prediction():
    kw = dict(n=128, hw_px=14, c_in=1024, m=256, S=2)
    tot = [P.predict_block(P.MI355X, "spatial", r=r, **kw)["total_s"] for r in (0.0, 0.25, 0.5, 0.75, 1.0)]
    assert all(b >= a for a, b in zip(tot, tot[1:]))           # never faster with more active patches
    # l = l_data + l_computation + l_const, term by term (the paper's equation)
    k = P.predict_block(P.MI355X, "spatial", r=0.5, **kw)["kernels"][2]
    assert k.total == pytest.approx(k.l_off2on + k.l_global2local + k.l_computation + k.l_const)
    # tiles are dealt to PEs in whole numbers: the latency is a staircase in the number of tiles per PE
    assert k.tiles_per_pe == -(-k.tiles // P.MI355X.n_pe)
    # twice the PEs never makes a kernel slower; a faster off-chip memory shortens only l_off2on
    big = dataclasses.replace(P.MI355X, n_pe=512)
    assert P.predict_block(big, "spatial", r=0.5, **kw)["total_s"] <= tot[2]
    fast = dataclasses.replace(P.MI355X, offchip_Bps=16e12)
    k2 = P.predict_block(fast, "spatial", r=0.5, **kw)["kernels"][2]
    assert k2.l_off2on == pytest.approx(k.l_off2on / 2) and k2.l_computation == k.l_computation
    # layer skipping at keep ratio r costs what the static block costs on r*n samples (whole samples, no halo)
    lay = P.predict_block(P.MI355X, "layer", n=128, hw_px=14, c_in=1024, m=256, r=0.5)
    sta = P.predict_block(P.MI355X, "static", n=64, hw_px=14, c_in=1024, m=256)
    assert lay["flops"] == pytest.approx(sta["flops"])
    assert lay["total_s"] == pytest.approx(sta["total_s"], rel=0.05)
    # coarser patches at equal ratio are never slower (less halo for conv1; Sec. 4, latency vs granularity)
    a = P.predict_block(P.MI355X, "spatial", n=128, hw_px=56, c_in=256, m=64, S=1, r=0.5, fused_masker=False)["total_s"]
    b = P.predict_block(P.MI355X, "spatial", n=128, hw_px=56, c_in=256, m=64, S=8, r=0.5, fused_masker=False)["total_s"]
    assert b <= a


def test_hardware_table_of_the_paper():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "hardware_properties.txt")) if l.strip() and l[0] != "#"]
    assert len(rows) == 5
    for name, pe, fp32, mhz, gb in rows:
        hw = P.paper_device(name, int(pe), int(fp32), float(mhz), float(gb))
        # peak FP32 throughput = #PE x #FP32 x 2 x frequency
        assert hw.n_pe * hw.pe_flops("f32") == pytest.approx(int(pe) * int(fp32) * 2 * float(mhz) * 1e6)
    v100 = P.paper_device("V100", 80, 64, 1500, 700)
    assert v100.n_pe * v100.pe_flops("f32") == pytest.approx(15.36e12)   # the V100's 15.4 TFLOP/s FP32


def test_group_convolution_and_se_in_the_prediction():
    kw = dict(n=128, hw_px=14, c_in=320, m=320, S=2, r=0.5, fused_masker=False)
    plain = P.predict_block(P.MI355X, "spatial", **kw)
    grp = P.predict_block(P.MI355X, "spatial", group_width=16, **kw)
    se = P.predict_block(P.MI355X, "spatial", group_width=16, se_width=80, **kw)
    # FLOPs of the 3x3 shrink by m / g; the two 1x1 convs are untouched
    f = lambda p_, name: sum(k.flops for k in p_["kernels"] if name in k.name)
    assert f(grp, "conv2") == pytest.approx(f(plain, "conv2") * 16 / 320)
    assert f(grp, "conv1") == f(plain, "conv1") and f(grp, "conv3") == f(plain, "conv3")
    # the group convolution is never slower than the full one; the SE module adds four kernels and their constants
    assert grp["total_s"] <= plain["total_s"]
    assert len(se["kernels"]) == len(grp["kernels"]) + 4
    assert se["total_s"] >= grp["total_s"] + 4 * P.MI355X.const_s
    # the 3x3's share of FLOPs as the oracle counts them for one group
    rows = 0.5 * 128 * 14 * 14
    assert f(grp, "conv2") == pytest.approx(2.0 * rows * 9 * 16 * 320, rel=1e-3)
