"""Pins for the CPU oracle: everything here checks oracle/laud_oracle.py against something
other than itself -- an independent per-output-element evaluator written with explicit
loops and bounds checks, closed forms, invariants the paper states, library routines for
the special cases that reduce to one, and the one set of values the paper prints."""
import itertools
import os

import numpy as np
import pytest

from oracle import laud_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


# --------------------------------------------------------------------------- #
# independent brute-force evaluator (pure Python floats, no numpy arithmetic)
# --------------------------------------------------------------------------- #
def _rand_params(rng, c_in, m, c_out, relu_out=False):
    return O.BottleneckParams(
        w1=rng.standard_normal((m, c_in)), w2=rng.standard_normal((m, 3, 3, m)) * 0.5,
        w3=rng.standard_normal((c_out, m)),
        s1=1 + 0.3 * rng.standard_normal(m), t1=0.5 * rng.standard_normal(m),
        s2=1 + 0.3 * rng.standard_normal(m), t2=0.5 * rng.standard_normal(m),
        s3=1 + 0.3 * rng.standard_normal(c_out), t3=0.5 * rng.standard_normal(c_out),
        relu_out=relu_out)


def _bf_h1(x, p, n, y, xx, i):
    """conv1 output channel i at pixel (y, xx); ZERO outside the image (the 3x3's padding
    is on its own input, not on x)."""
    H, W, C = len(x[0]), len(x[0][0]), len(x[0][0][0])
    if y < 0 or y >= H or xx < 0 or xx >= W:
        return 0.0
    acc = 0.0
    for c in range(C):
        acc += p["w1"][i][c] * x[n][y][xx][c]
    v = p["s1"][i] * acc + p["t1"][i]
    return v if v > 0.0 else 0.0


def _bf_h2(x, p, n, y, xx, j, cm=None):
    m = len(p["w1"])
    acc = 0.0
    for ky in range(3):
        for kx in range(3):
            for i in range(m):
                h1 = _bf_h1(x, p, n, y + ky - 1, xx + kx - 1, i)
                if cm is not None:
                    h1 *= cm[i]
                acc += p["w2"][j][ky][kx][i] * h1
    v = p["s2"][j] * acc + p["t2"][j]
    v = v if v > 0.0 else 0.0
    if cm is not None:
        v *= cm[j]
    return v


def _bf_out(x, p, n, y, xx, o, relu_out, cm=None):
    m = len(p["w1"])
    acc = 0.0
    for j in range(m):
        acc += p["w3"][o][j] * _bf_h2(x, p, n, y, xx, j, cm)
    v = x[n][y][xx][o] + p["s3"][o] * acc + p["t3"][o]
    if relu_out and v < 0.0:
        v = 0.0
    return v


def _as_lists(p):
    return {k: np.asarray(getattr(p, k), np.float64).tolist()
            for k in ("w1", "w2", "w3", "s1", "t1", "s2", "t2", "s3", "t3")}


def brute_force_dyn(x, p, S, mask):
    xl = np.asarray(x, np.float64).tolist()
    pl = _as_lists(p)
    N, H, W, C = np.shape(x)
    out = np.array(x, np.float64)
    for n in range(N):
        for y in range(H):
            for xx in range(W):
                if mask[n][y // S][xx // S]:
                    for o in range(C):
                        out[n, y, xx, o] = _bf_out(xl, pl, n, y, xx, o, p.relu_out)
    return out


@pytest.mark.parametrize("S", [1, 2, 4])
@pytest.mark.parametrize("relu_out", [False, True])
def test_dyn_block_vs_bruteforce_all_masks(S, relu_out):
    rng = np.random.default_rng(100 + S)
    N, H, W, c_in, m = 1, 4, 4, 4, 2
    x = rng.standard_normal((N, H, W, c_in))
    p = _rand_params(rng, c_in, m, c_in, relu_out)
    hp = H // S
    cells = N * hp * hp
    if cells <= 4:
        masks = list(itertools.product([0, 1], repeat=cells))
    else:  # S = 1: 2^16 masks is too many; all single-cell masks, their complements, and random ones
        eye = [tuple(int(i == j) for i in range(cells)) for j in range(cells)]
        comp = [tuple(1 - v for v in e) for e in eye]
        rnd = [tuple(rng.integers(0, 2, cells).tolist()) for _ in range(8)]
        masks = eye + comp + rnd + [tuple([0] * cells), tuple([1] * cells)]
    # the dense branch does not depend on the mask: evaluate the brute force once, all-active
    full = brute_force_dyn(x, p, S, np.ones((N, hp, hp), int).tolist())
    for bits in masks:
        mk = np.array(bits, np.uint8).reshape(N, hp, hp)
        want = np.where(O.upsample_mask(mk, S).astype(bool)[..., None], full, x)
        got = O.dyn_bottleneck(x, p, S, mk)
        np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_dyn_block_vs_bruteforce_batched_random_masks():
    rng = np.random.default_rng(7)
    N, H, W, c_in, m, S = 2, 6, 4, 3, 2, 2
    x = rng.standard_normal((N, H, W, c_in))
    p = _rand_params(rng, c_in, m, c_in, relu_out=True)
    for _ in range(3):
        mk = rng.integers(0, 2, (N, H // S, W // S)).astype(np.uint8)
        np.testing.assert_allclose(O.dyn_bottleneck(x, p, S, mk),
                                   brute_force_dyn(x, p, S, mk.tolist()), rtol=1e-12, atol=1e-12)


def test_border_padding_is_on_h1_not_on_x():
    """With a non-zero conv1 shift, zero-padding x (instead of h1) would feed relu(t1) != 0 into
    the 3x3 at the border; the brute force pads h1.  A single active corner patch isolates it."""
    rng = np.random.default_rng(3)
    x = rng.standard_normal((1, 4, 4, 3))
    p = _rand_params(rng, 3, 2, 3)
    p.t1 = np.array([0.9, 1.3])  # strictly positive shift
    mk = np.zeros((1, 2, 2), np.uint8)
    mk[0, 0, 0] = 1
    np.testing.assert_allclose(O.dyn_bottleneck(x, p, 2, mk), brute_force_dyn(x, p, 2, mk.tolist()),
                               rtol=1e-12, atol=1e-12)
    # and the wrong reading is measurably different, so the test above has teeth
    xpad = np.zeros((1, 6, 6, 3))
    xpad[:, 1:5, 1:5] = x
    wrong = O.static_bottleneck(xpad, p)[:, 1:5, 1:5]
    assert np.abs(wrong[0, 0, 0] - O.static_bottleneck(x, p)[0, 0, 0]).max() > 1e-3


# --------------------------------------------------------------------------- #
# closed forms
# --------------------------------------------------------------------------- #
def test_conv3x3_box_filter_counts_neighbours():
    """All-ones 3x3 kernel on an all-ones image counts in-bounds neighbours: 4 / 6 / 9."""
    h = np.ones((1, 5, 6, 1))
    out = O.conv3x3(h, np.ones((1, 3, 3, 1)))[0, :, :, 0]
    assert out[0, 0] == out[0, -1] == out[-1, 0] == out[-1, -1] == 4
    assert (out[0, 1:-1] == 6).all() and (out[-1, 1:-1] == 6).all()
    assert (out[1:-1, 0] == 6).all() and (out[1:-1, -1] == 6).all()
    assert (out[1:-1, 1:-1] == 9).all()


@pytest.mark.parametrize("ky,kx", list(itertools.product(range(3), range(3))))
def test_conv3x3_tap_orientation(ky, kx):
    """Cross-correlation: an impulse at (y0,x0) seen through the single tap (ky,kx) lands at
    (y0-(ky-1), x0-(kx-1)); channel routing in -> out as indexed."""
    h = np.zeros((1, 5, 5, 2))
    h[0, 2, 2, 1] = 3.0
    w = np.zeros((3, 3, 3, 2))
    w[2, ky, kx, 1] = 2.0
    out = O.conv3x3(h, w)
    want = np.zeros((1, 5, 5, 3))
    want[0, 2 - (ky - 1), 2 - (kx - 1), 2] = 6.0
    np.testing.assert_array_equal(out, want)


def test_conv1x1_one_hot():
    x = np.zeros((1, 2, 2, 3))
    x[0, 1, 0, 2] = 5.0
    w = np.arange(12, dtype=float).reshape(4, 3)
    out = O.conv1x1(x, w)
    want = np.zeros((1, 2, 2, 4))
    want[0, 1, 0, :] = 5.0 * w[:, 2]
    np.testing.assert_array_equal(out, want)


def test_branch_is_affine_in_s3_t3_and_linear_in_w3():
    rng = np.random.default_rng(11)
    x = rng.standard_normal((1, 4, 4, 4))
    p = _rand_params(rng, 4, 3, 4)
    f0 = O.bottleneck_branch(x, p)
    q = _rand_params(rng, 4, 3, 4)
    q.__dict__.update({k: getattr(p, k) for k in ("w1", "w2", "s1", "t1", "s2", "t2")})
    q.w3, q.s3, q.t3 = 2.0 * p.w3, p.s3, p.t3
    np.testing.assert_allclose(O.bottleneck_branch(x, q) - p.t3, 2.0 * (f0 - p.t3), rtol=1e-12, atol=1e-12)
    q.w3, q.s3, q.t3 = p.w3, 3.0 * p.s3, p.t3 + 1.0
    np.testing.assert_allclose(O.bottleneck_branch(x, q), 3.0 * (f0 - p.t3) + p.t3 + 1.0, rtol=1e-12, atol=1e-12)


# --------------------------------------------------------------------------- #
# library special case: activation ratio 1 is a standard bottleneck
# --------------------------------------------------------------------------- #
@pytest.mark.parametrize("relu_out", [False, True])
def test_ratio_one_equals_torch_conv2d_bottleneck(relu_out):
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(21)
    N, H, W, c_in, m = 2, 8, 12, 16, 8
    x = rng.standard_normal((N, H, W, c_in))
    p = _rand_params(rng, c_in, m, c_in, relu_out)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).double()
    xt = t(x).permute(0, 3, 1, 2)
    ch = lambda v: t(v).view(1, -1, 1, 1)
    h1 = F.relu(F.conv2d(xt, t(p.w1)[:, :, None, None]) * ch(p.s1) + ch(p.t1))
    h2 = F.relu(F.conv2d(h1, t(p.w2).permute(0, 3, 1, 2), padding=1) * ch(p.s2) + ch(p.t2))
    y = xt + F.conv2d(h2, t(p.w3)[:, :, None, None]) * ch(p.s3) + ch(p.t3)
    if relu_out:
        y = F.relu(y)
    want = y.permute(0, 2, 3, 1).numpy()
    got = O.dyn_bottleneck(x, p, 4, np.ones((N, H // 4, W // 4), np.uint8))
    np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-11)
    np.testing.assert_allclose(O.static_bottleneck(x, p), want, rtol=1e-11, atol=1e-11)


# --------------------------------------------------------------------------- #
# invariants of mask-then-select (Sec. 3.1; Fig. 2 caption)
# --------------------------------------------------------------------------- #
def test_ratio_zero_is_identity_and_single_flip_is_local():
    rng = np.random.default_rng(5)
    N, H, W, c, S = 2, 8, 8, 4, 2
    x = rng.standard_normal((N, H, W, c))
    p = _rand_params(rng, c, 2, c, relu_out=True)
    zero = np.zeros((N, H // S, W // S), np.uint8)
    out0 = O.dyn_bottleneck(x, p, S, zero)
    assert np.array_equal(out0, x)
    static = O.static_bottleneck(x, p)
    for (n, py, px) in [(0, 0, 0), (1, 3, 2), (0, 1, 3)]:
        mk = zero.copy()
        mk[n, py, px] = 1
        out = O.dyn_bottleneck(x, p, S, mk)
        changed = np.any(out != x, axis=-1)
        want = np.zeros((N, H, W), bool)
        want[n, py * S:(py + 1) * S, px * S:(px + 1) * S] = True
        assert np.array_equal(changed, want)
        assert np.array_equal(out[want], static[want])


def test_S_equal_H_is_layer_skipping():
    """S = feature resolution turns the spatial block into layer skipping (Sec. 3.2)."""
    rng = np.random.default_rng(6)
    N, H, c = 3, 4, 4
    x = rng.standard_normal((N, H, H, c))
    p = _rand_params(rng, c, 2, c, relu_out=True)
    keep = np.array([1, 0, 1], np.uint8)
    a = O.dyn_bottleneck(x, p, H, keep.reshape(N, 1, 1))
    b = O.layer_skip_bottleneck(x, p, keep)
    assert np.array_equal(a, b)
    assert np.array_equal(b[1], x[1])
    assert np.array_equal(O.layer_skip_bottleneck(x, p, np.ones(N, np.uint8)), O.static_bottleneck(x, p))
    assert np.array_equal(O.layer_skip_bottleneck(x, p, np.zeros(N, np.uint8)), x)
    mk = rng.integers(0, 2, (N, 2, 2)).astype(np.uint8)
    both = O.layer_skip_bottleneck(x, p, keep, 2, mk)
    assert np.array_equal(both, O.dyn_bottleneck(x, p, 2, mk * keep[:, None, None]))
    # one logit per sample when S = H
    assert O.mask_logits(x, H, rng.standard_normal(c), 0.1).shape == (N, 1, 1)


# --------------------------------------------------------------------------- #
# masker (Sec. 3.2; App. B eq.)
# --------------------------------------------------------------------------- #
def test_two_logit_argmax_equals_one_channel_difference():
    rng = np.random.default_rng(8)
    x = rng.standard_normal((3, 8, 8, 16))
    for S in (1, 2, 4, 8):
        w2 = rng.standard_normal((2, 16))
        b2 = rng.standard_normal(2)
        l2 = O.masker_two_logits(x, S, w2, b2)
        one = O.mask_logits(x, S, w2[0] - w2[1], b2[0] - b2[1])
        assert np.abs(one).min() > 1e-9  # no ties in this draw
        assert np.array_equal(O.mask_from_two_logits(l2), O.threshold(one))
        np.testing.assert_allclose(one, l2[..., 0] - l2[..., 1], rtol=1e-12, atol=1e-12)


def test_masker_pool_and_1x1_commute():
    """Pooling and a 1x1 conv are both linear and share the input (App. B), so the masker
    logit equals the S x S mean of the per-pixel projection."""
    rng = np.random.default_rng(9)
    x = rng.standard_normal((2, 8, 12, 6))
    w = rng.standard_normal(6)
    per_pixel = O.conv1x1(x, w[None, :])  # [N,H,W,1]
    for S in (1, 2, 4):
        want = O.pool_patches(per_pixel, S)[..., 0] + 0.25
        np.testing.assert_allclose(O.mask_logits(x, S, w, 0.25), want, rtol=1e-12, atol=1e-12)


def test_mask_logits_hand_example_and_threshold_ties():
    # 1 sample, 2x2 image, 2 channels, S=2: mean over the four pixels, then dot with w, plus bias
    x = np.array([[[[1.0, 10.0], [2.0, 20.0]], [[3.0, 30.0], [6.0, 40.0]]]])
    got = O.mask_logits(x, 2, np.array([2.0, -0.5]), 1.5)
    assert got.shape == (1, 1, 1)
    assert got[0, 0, 0] == pytest.approx(2.0 * 3.0 - 0.5 * 25.0 + 1.5)
    assert O.threshold(np.array([0.0, -0.0, 1e-30, -1e-30, np.nan, np.inf])).tolist() == [0, 0, 1, 0, 0, 1]


def test_valid_granularities_match_the_paper():
    with open(os.path.join(GOLDEN, "valid_S_56.txt")) as f:
        vals = [int(v) for line in f if not line.startswith("#") for v in line.split()]
    x = np.zeros((1, 56, 56, 1))
    ok = []
    for S in range(1, 57):
        try:
            O.pool_patches(x, S)
            ok.append(S)
        except ValueError:
            pass
    assert ok == vals


# --------------------------------------------------------------------------- #
# index generation and gather
# --------------------------------------------------------------------------- #
def test_compact_definition():
    rng = np.random.default_rng(10)
    mk = rng.integers(0, 2, (5, 7, 7)).astype(np.uint8)
    mk[2] = 0
    mk[3] = 1
    idx = O.compact(mk)
    assert idx.dtype == np.int32
    assert np.array_equal(idx, np.flatnonzero(mk.reshape(-1)))
    assert len(idx) == int(mk.sum()) and np.all(np.diff(idx) > 0)
    off = O.sample_offsets(mk)
    assert off[0] == 0 and off[-1] == len(idx) and off[3] - off[2] == 0 and off[4] - off[3] == 49
    for n in range(5):
        seg = idx[off[n]:off[n + 1]]
        assert np.all(seg // 49 == n)
    assert O.compact(np.zeros((2, 3, 3), np.uint8)).size == 0
    # any non-zero byte counts as set
    assert O.compact(np.array([0, 2, 0, 255], np.uint8)).tolist() == [1, 3]


def test_gather_all_active_halo0_is_a_retiling():
    rng = np.random.default_rng(12)
    N, H, W, C, S = 2, 8, 12, 3, 4
    x = rng.standard_normal((N, H, W, C)).astype(np.float32)
    idx = O.compact(np.ones((N, H // S, W // S), np.uint8))
    g = O.gather_patches(x, S, 0, idx)
    want = x.reshape(N, H // S, S, W // S, S, C).transpose(0, 1, 3, 2, 4, 5).reshape(-1, S, S, C)
    assert g.dtype == x.dtype and np.array_equal(g, want)


def test_gather_halo1_matches_padded_slices():
    rng = np.random.default_rng(13)
    N, H, W, C, S = 2, 6, 6, 2, 2
    x = rng.standard_normal((N, H, W, C))
    mk = rng.integers(0, 2, (N, 3, 3)).astype(np.uint8)
    mk[0, 0, 0] = mk[1, 2, 2] = 1  # corners: zero fill on two sides
    idx = O.compact(mk)
    g = O.gather_patches(x, S, 1, idx)
    xp = np.pad(x, ((0, 0), (1, 1), (1, 1), (0, 0)))
    for p, q in enumerate(idx):
        n, r = divmod(int(q), 9)
        py, px = divmod(r, 3)
        assert np.array_equal(g[p], xp[n, py * S:py * S + S + 2, px * S:px * S + S + 2])
    assert np.all(g[0, 0, :, :] == 0) and np.all(g[0, :, 0, :] == 0)


# --------------------------------------------------------------------------- #
# channel skipping (Fig. 2 caption; Sec. 3.2)
# --------------------------------------------------------------------------- #
def test_channel_skip_special_cases_and_independent_formulation():
    rng = np.random.default_rng(14)
    N, H, c, m, D = 4, 5, 6, 8, 4
    x = rng.standard_normal((N, H, H, c))
    p = _rand_params(rng, c, m, c, relu_out=True)
    ones = np.ones((N, D), np.uint8)
    np.testing.assert_allclose(O.channel_skip_bottleneck(x, p, ones), O.static_bottleneck(x, p), rtol=1e-12)
    zeros = np.zeros((N, D), np.uint8)
    np.testing.assert_allclose(O.channel_skip_bottleneck(x, p, zeros), np.maximum(x + p.t3, 0), rtol=1e-12)
    cm = rng.integers(0, 2, (N, D)).astype(np.uint8)
    cm[0] = [1, 0, 0, 1]
    got = O.channel_skip_bottleneck(x, p, cm)
    G = m // D
    for n in range(N):
        # the same block with dropped channels removed from the weights: rows of W1, rows and
        # columns of W2, columns of W3, and the shifts t1, t2 of dropped channels set to zero
        k = np.repeat(cm[n].astype(bool), G)
        q = _rand_params(rng, c, m, c, relu_out=True)
        q.w1 = np.where(k[:, None], p.w1, 0.0)
        q.w2 = np.where(k[:, None, None, None] & k[None, None, None, :], p.w2, 0.0)
        q.w3 = np.where(k[None, :], p.w3, 0.0)
        q.s1, q.s2, q.s3, q.t3 = p.s1, p.s2, p.s3, p.t3
        q.t1 = np.where(k, p.t1, 0.0)
        q.t2 = np.where(k, p.t2, 0.0)
        np.testing.assert_allclose(got[n:n + 1], O.static_bottleneck(x[n:n + 1], q), rtol=1e-11, atol=1e-11)


def test_channel_skip_vs_bruteforce():
    rng = np.random.default_rng(15)
    N, H, c, m, D = 2, 3, 3, 4, 2
    x = rng.standard_normal((N, H, H, c))
    p = _rand_params(rng, c, m, c)
    cm = np.array([[1, 0], [0, 1]], np.uint8)
    got = O.channel_skip_bottleneck(x, p, cm)
    xl, pl = x.tolist(), _as_lists(p)
    for n in range(N):
        cvec = np.repeat(cm[n], m // D).astype(float).tolist()
        for y in range(H):
            for xx in range(H):
                for o in range(c):
                    assert got[n, y, xx, o] == pytest.approx(_bf_out(xl, pl, n, y, xx, o, False, cvec), abs=1e-11)


# --------------------------------------------------------------------------- #
# complexity closed forms (Sec. 3.2 "Computational complexity")
# --------------------------------------------------------------------------- #
def test_flop_ratios_closed_forms():
    for c_in, m in [(256, 64), (512, 128), (1024, 256), (2048, 512)]:
        f1, f2, f3 = O.conv_macs_per_pixel(c_in, m, c_in)
        assert (f1, f2, f3) == (4 * m * m, 9 * m * m, 4 * m * m)
        for r in (0.0, 0.25, 0.6, 1.0):
            assert O.spatial_flops_ratio(r, r, c_in, m, c_in) == pytest.approx(r)
            assert O.spatial_flops_ratio(r, 1.0, c_in, m, c_in) == pytest.approx((4 + 13 * r) / 17)
            assert O.channel_flops_ratio(r, c_in, m, c_in) == pytest.approx((8 * r + 9 * r * r) / 17)
            assert O.channel_flops_ratio(r, c_in, m, c_in) <= r + 1e-15
    # every identity bottleneck of ResNet-50/101 at 224^2 costs the same: 17 m^2 * H*W MACs
    assert {17 * m * m * hw * hw for m, hw in [(64, 56), (128, 28), (256, 14), (512, 7)]} == {218365952}


def test_activation_and_dilated_ratio():
    mk = np.zeros((1, 4, 4), np.uint8)
    assert O.activation_ratio(mk) == 0 and O.dilated_ratio(mk, 2) == 0
    mk[0, 1, 2] = 1
    assert O.activation_ratio(mk) == 1 / 16
    assert O.dilated_ratio(mk, 2) == pytest.approx(16 / 64)   # (S+2)^2 pixels of an 8x8 map
    assert O.dilated_ratio(mk, 1) == pytest.approx(9 / 16)
    mk[:] = 1
    assert O.activation_ratio(mk) == 1 and O.dilated_ratio(mk, 2) == 1
    # brute force on a random mask
    rng = np.random.default_rng(16)
    mk = rng.integers(0, 2, (2, 3, 3)).astype(np.uint8)
    S = 2
    cnt = 0
    for n in range(2):
        for y in range(6):
            for x in range(6):
                hit = False
                for dy in (-1, 0, 1):
                    for dx in (-1, 0, 1):
                        yy, xx = y + dy, x + dx
                        if 0 <= yy < 6 and 0 <= xx < 6 and mk[n, yy // S, xx // S]:
                            hit = True
                cnt += hit
    assert O.dilated_ratio(mk, S) == pytest.approx(cnt / 72)


# --------------------------------------------------------------------------- #
# channel masker (Sec. 3.2 "Masker design")
# --------------------------------------------------------------------------- #
def test_channel_masker_hidden_width_formula():
    # max(floor(D/16), 16): D = C/G for the mid widths 64..512 with G in {1, 2} and for 4 groups
    assert [O.channel_masker_hidden(d) for d in (4, 32, 64, 256, 257, 512, 1024)] == [16, 16, 16, 16, 16, 32, 64]


def test_channel_masker_vs_pure_python_and_hand_example():
    rng = np.random.default_rng(30)
    N, H, W, C, D, hid = 3, 3, 2, 5, 4, 6
    x = rng.standard_normal((N, H, W, C))
    wa, ba = rng.standard_normal((hid, C)), rng.standard_normal(hid)
    wb, bb = rng.standard_normal((2 * D, hid)), rng.standard_normal(2 * D)
    got = O.channel_masker_logits(x, wa, ba, wb, bb)
    assert got.shape == (N, D, 2)
    xl = x.tolist()
    for n in range(N):
        g = [sum(xl[n][y][xx][c] for y in range(H) for xx in range(W)) / (H * W) for c in range(C)]
        h = [max(0.0, sum(wa[j][c] * g[c] for c in range(C)) + ba[j]) for j in range(hid)]
        for o in range(2 * D):
            want = sum(wb[o][j] * h[j] for j in range(hid)) + bb[o]
            assert got[n, o // 2, o % 2] == pytest.approx(want, abs=1e-12)   # row-major [D, 2] view
    # hand example: one pixel, identity first layer, second layer picks h0 - h1 against 0
    x1 = np.array([[[[2.0, -3.0]]]])
    l = O.channel_masker_logits(x1, np.eye(2), np.zeros(2), np.array([[1.0, 0.0], [0.0, 1.0]]), np.zeros(2))
    assert l.tolist() == [[[2.0, 0.0]]]            # relu(-3) = 0
    assert O.channel_mask_from_logits(l).tolist() == [[1]]
    assert O.channel_mask_from_logits(np.array([[[1.0, 1.0], [0.0, 1.0], [np.nan, 0.0]]])).tolist() == [[0, 0, 0]]
    # argmax of two logits == sign of their difference, computed from differenced second-layer weights
    l2 = O.channel_masker_logits(x, wa, ba, wb, bb)
    g = x.mean(axis=(1, 2))
    h = np.maximum(g @ wa.T + ba, 0)
    diff = h @ (wb[0::2] - wb[1::2]).T + (bb[0::2] - bb[1::2])
    assert np.array_equal(O.channel_mask_from_logits(l2), (diff > 0).astype(np.uint8))


# --------------------------------------------------------------------------- #
# static parts of the body: library special cases (torch conv2d / max_pool2d)
# --------------------------------------------------------------------------- #
def test_conv2d_maxpool_stem_and_projection_block_vs_torch():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(40)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).double()
    nchw = lambda a: t(a).permute(0, 3, 1, 2)
    oihw = lambda w: t(w).permute(0, 3, 1, 2)
    back = lambda y: y.permute(0, 2, 3, 1).numpy()
    ch = lambda v: t(v).view(1, -1, 1, 1)
    x = rng.standard_normal((2, 13, 10, 3))
    for k, s_, p_ in ((7, 2, 3), (3, 2, 1), (3, 1, 1), (1, 2, 0)):
        w = rng.standard_normal((5, k, k, 3))
        np.testing.assert_allclose(O.conv2d(x, w, s_, p_), back(F.conv2d(nchw(x), oihw(w), stride=s_, padding=p_)),
                                   rtol=1e-11, atol=1e-11)
    # conv2d with stride 1 pad 1 is the 3x3 the dynamic block uses
    w3 = rng.standard_normal((4, 3, 3, 3))
    np.testing.assert_allclose(O.conv2d(x, w3, 1, 1), O.conv3x3(x, w3), rtol=1e-12, atol=1e-12)
    np.testing.assert_array_equal(O.maxpool3x3_s2(x), back(F.max_pool2d(nchw(x), 3, 2, 1)))
    xn = -np.abs(x) - 1.0   # all-negative input: zero padding would win, -inf padding must not
    np.testing.assert_array_equal(O.maxpool3x3_s2(xn), back(F.max_pool2d(nchw(xn), 3, 2, 1)))
    # stem
    w7, s, tt = rng.standard_normal((6, 7, 7, 3)), 1 + 0.2 * rng.standard_normal(6), rng.standard_normal(6)
    xs = rng.standard_normal((2, 32, 24, 3))
    want = F.max_pool2d(F.relu(F.conv2d(nchw(xs), oihw(w7), stride=2, padding=3) * ch(s) + ch(tt)), 3, 2, 1)
    np.testing.assert_allclose(O.stem(xs, w7, s, tt), back(want), rtol=1e-11, atol=1e-11)
    # projection block, stride 1 and 2
    for stride in (1, 2):
        c_in, m, c_out = 6, 4, 16
        xb = rng.standard_normal((2, 8, 6, c_in))
        p = _rand_params(rng, c_in, m, c_out)
        wsc, ssc, tsc = rng.standard_normal((c_out, c_in)), 1 + 0.2 * rng.standard_normal(c_out), rng.standard_normal(c_out)
        xt = nchw(xb)
        h1 = F.relu(F.conv2d(xt, t(p.w1)[:, :, None, None]) * ch(p.s1) + ch(p.t1))
        h2 = F.relu(F.conv2d(h1, oihw(p.w2), stride=stride, padding=1) * ch(p.s2) + ch(p.t2))
        f = F.conv2d(h2, t(p.w3)[:, :, None, None]) * ch(p.s3) + ch(p.t3)
        sc = F.conv2d(xt, t(wsc)[:, :, None, None], stride=stride) * ch(ssc) + ch(tsc)
        np.testing.assert_allclose(O.projection_bottleneck(xb, p, wsc, ssc, tsc, stride), back(F.relu(f + sc)),
                                   rtol=1e-11, atol=1e-11)


# --------------------------------------------------------------------------- #
# dynamic first block of a stage (mask on the output grid, projection shortcut)
# --------------------------------------------------------------------------- #
def _bf_proj_out(x, p, wsc, ssc, tsc, stride, n, yo, xo, o, active, relu_out):
    """One output element with explicit loops: strided shortcut, plus the branch if the location is active."""
    C, m = len(x[0][0][0]), len(p["w1"])
    acc = 0.0
    for c in range(C):
        acc += wsc[o][c] * x[n][stride * yo][stride * xo][c]
    v = ssc[o] * acc + tsc[o]
    if active:
        f = 0.0
        for j in range(m):
            a2 = 0.0
            for ky in range(3):
                for kx in range(3):
                    for i in range(m):
                        a2 += p["w2"][j][ky][kx][i] * _bf_h1(x, p, n, stride * yo + ky - 1, stride * xo + kx - 1, i)
            h2 = p["s2"][j] * a2 + p["t2"][j]
            f += p["w3"][o][j] * (h2 if h2 > 0.0 else 0.0)
        v += p["s3"][o] * f + p["t3"][o]
    return 0.0 if (relu_out and v < 0.0) else v


@pytest.mark.parametrize("stride,H,W,S", [(2, 4, 4, 1), (2, 4, 4, 2), (1, 2, 2, 1), (2, 5, 3, 1), (2, 8, 4, 2)])
@pytest.mark.parametrize("relu_out", [False, True])
def test_dyn_projection_block_vs_bruteforce_all_masks(stride, H, W, S, relu_out):
    rng = np.random.default_rng(700 + 10 * H + S + stride)
    N, c_in, m, c_out = 1, 3, 2, 4
    x = rng.standard_normal((N, H, W, c_in))
    p = _rand_params(rng, c_in, m, c_out, relu_out)
    wsc, ssc, tsc = rng.standard_normal((c_out, c_in)), 1 + 0.3 * rng.standard_normal(c_out), rng.standard_normal(c_out)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    hp, wp = Ho // S, Wo // S
    xl, pl = x.tolist(), _as_lists(p)
    for bits in itertools.product([0, 1], repeat=hp * wp):
        mask = np.array(bits, np.uint8).reshape(N, hp, wp)
        got = O.dyn_projection_bottleneck(x, p, wsc, ssc, tsc, stride, S, mask)
        assert got.shape == (N, Ho, Wo, c_out)
        for yo in range(Ho):
            for xo in range(Wo):
                for o in range(c_out):
                    want = _bf_proj_out(xl, pl, wsc.tolist(), ssc.tolist(), tsc.tolist(), stride, 0, yo, xo, o,
                                        bool(mask[0, yo // S, xo // S]), relu_out)
                    assert abs(got[0, yo, xo, o] - want) <= 1e-11 * (1 + abs(want))


def test_dyn_projection_block_invariants_and_masker():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(77)
    N, H, W, c_in, m, c_out, stride, S = 2, 12, 8, 6, 4, 8, 2, 2
    x = rng.standard_normal((N, H, W, c_in))
    p = _rand_params(rng, c_in, m, c_out, True)
    wsc, ssc, tsc = rng.standard_normal((c_out, c_in)), 1 + 0.2 * rng.standard_normal(c_out), rng.standard_normal(c_out)
    Ho, Wo = H // stride, W // stride
    ones = np.ones((N, Ho // S, Wo // S), np.uint8)
    # every location active: the static first block (itself pinned against torch above)
    np.testing.assert_allclose(O.dyn_projection_bottleneck(x, p, wsc, ssc, tsc, stride, S, ones),
                               O.projection_bottleneck(x, p, wsc, ssc, tsc, stride), rtol=1e-12, atol=1e-12)
    # nothing active: the activated skip connection alone (library strided 1x1)
    xt = torch.from_numpy(x).permute(0, 3, 1, 2)
    sc = F.conv2d(xt, torch.from_numpy(wsc)[:, :, None, None], stride=stride)
    sc = sc * torch.from_numpy(ssc).view(1, -1, 1, 1) + torch.from_numpy(tsc).view(1, -1, 1, 1)
    np.testing.assert_allclose(O.dyn_projection_bottleneck(x, p, wsc, ssc, tsc, stride, S, 0 * ones),
                               F.relu(sc).permute(0, 2, 3, 1).numpy(), rtol=1e-11, atol=1e-11)
    # one flipped patch changes exactly its S x S output pixels
    mk = (rng.random(ones.shape) < 0.5).astype(np.uint8)
    mk2 = mk.copy()
    mk2[1, 1, 0] ^= 1
    a = O.dyn_projection_bottleneck(x, p, wsc, ssc, tsc, stride, S, mk)
    b = O.dyn_projection_bottleneck(x, p, wsc, ssc, tsc, stride, S, mk2)
    diff = np.any(a != b, axis=-1)
    region = np.zeros_like(diff)
    region[1, S:2 * S, 0:S] = True
    assert not np.any(diff & ~region)
    # masker of a strided block: adaptive average pooling of x to the output patch grid, then the 1x1
    w = rng.standard_normal(c_in)
    pooled = F.adaptive_avg_pool2d(xt, (Ho // S, Wo // S)).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(O.strided_mask_logits(x, stride, S, w, 0.25), pooled @ w + 0.25, rtol=1e-11, atol=1e-11)


# --------------------------------------------------------------------------- #
# group convolution + squeeze-and-excitation block (Sec. 4, RegNetY backbones)
# --------------------------------------------------------------------------- #
def _rand_group_se(rng, c, m, g, se_w, relu_out=False):
    p = _rand_params(rng, c, m, c, relu_out)
    p.w2 = rng.standard_normal((m, 3, 3, g)) * 0.5
    e = O.GroupSE(g, rng.standard_normal((se_w, m)) * 0.7, 0.3 * rng.standard_normal(se_w),
                  rng.standard_normal((m, se_w)) * 0.7, 0.3 * rng.standard_normal(m)) if se_w else O.GroupSE(g)
    return p, e


def _bf_group_se(x, p, e, S, mask):
    """Sparse, loop-by-loop evaluation: h2 only at active pixels (group-restricted taps), the squeeze
    as a running sum over exactly those pixels, then the gate, the last 1x1 and the residual."""
    import math
    xl, pl = np.asarray(x, np.float64).tolist(), _as_lists(p)
    N, H, W, C = np.shape(x)
    m, g = len(pl["w1"]), e.g
    out = np.array(x, np.float64)
    for n in range(N):
        act = [(y, xx) for y in range(H) for xx in range(W) if mask[n][y // S][xx // S]]
        if not act:
            continue
        h2 = {}
        for (y, xx) in act:
            row = []
            for j in range(m):
                acc = 0.0
                for ky in range(3):
                    for kx in range(3):
                        for c in range(g):
                            acc += pl["w2"][j][ky][kx][c] * _bf_h1(xl, pl, n, y + ky - 1, xx + kx - 1, (j // g) * g + c)
                v = pl["s2"][j] * acc + pl["t2"][j]
                row.append(v if v > 0.0 else 0.0)
            h2[(y, xx)] = row
        gate = [1.0] * m
        if e.w_se1 is not None:
            z = [sum(h2[q][j] for q in act) / len(act) for j in range(m)]
            w1, b1, w2, b2 = (np.asarray(a, np.float64).tolist() for a in (e.w_se1, e.b_se1, e.w_se2, e.b_se2))
            hid = [max(sum(w1[k][j] * z[j] for j in range(m)) + b1[k], 0.0) for k in range(len(b1))]
            gate = [1.0 / (1.0 + math.exp(-(sum(w2[j][k] * hid[k] for k in range(len(hid))) + b2[j]))) for j in range(m)]
        for (y, xx) in act:
            for o in range(C):
                f = sum(pl["w3"][o][j] * h2[(y, xx)][j] * gate[j] for j in range(m))
                v = xl[n][y][xx][o] + pl["s3"][o] * f + pl["t3"][o]
                out[n, y, xx, o] = 0.0 if (p.relu_out and v < 0.0) else v
    return out


@pytest.mark.parametrize("S,g,se_w,relu_out", [(1, 2, 3, True), (2, 2, 3, False), (2, 1, 2, True), (4, 4, 0, True),
                                               (2, 4, 2, True)])
def test_group_se_block_vs_bruteforce_all_masks(S, g, se_w, relu_out):
    rng = np.random.default_rng(800 + 10 * S + g)
    N, H, W, c, m = 1, 4, 4, 3, 4
    x = rng.standard_normal((N, H, W, c))
    p, e = _rand_group_se(rng, c, m, g, se_w, relu_out)
    hp = H // S
    masks = list(itertools.product([0, 1], repeat=hp * hp))
    if len(masks) > 64:
        masks = [masks[i] for i in rng.choice(len(masks), 48, replace=False)] + [masks[0], masks[-1]]
    for bits in masks:
        mask = np.array(bits, np.uint8).reshape(N, hp, hp)
        np.testing.assert_allclose(O.dyn_group_se_bottleneck(x, p, e, S, mask), _bf_group_se(x, p, e, S, mask),
                                   rtol=1e-11, atol=1e-11)


def test_group_se_block_batched_bruteforce_and_empty_sample():
    rng = np.random.default_rng(81)
    N, H, W, c, m, g, S = 3, 4, 6, 4, 6, 3, 2
    x = rng.standard_normal((N, H, W, c))
    p, e = _rand_group_se(rng, c, m, g, 2, True)
    mask = (rng.random((N, H // S, W // S)) < 0.5).astype(np.uint8)
    mask[1] = 0  # a sample without any active patch stays untouched (and divides nothing by zero)
    got = O.dyn_group_se_bottleneck(x, p, e, S, mask)
    np.testing.assert_allclose(got, _bf_group_se(x, p, e, S, mask), rtol=1e-11, atol=1e-11)
    assert np.array_equal(got[1], x[1])


def test_group_se_block_all_active_equals_torch_composition():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(82)
    N, H, W, c, m, g, se_w, S = 2, 6, 4, 8, 12, 4, 3, 2
    x = rng.standard_normal((N, H, W, c))
    p, e = _rand_group_se(rng, c, m, g, se_w, True)
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    aff = lambda z, s, b: z * t(s).view(1, -1, 1, 1) + t(b).view(1, -1, 1, 1)
    xt = t(x).permute(0, 3, 1, 2)
    h1 = F.relu(aff(F.conv2d(xt, t(p.w1)[:, :, None, None]), p.s1, p.t1))
    h2 = F.relu(aff(F.conv2d(h1, t(p.w2).permute(0, 3, 1, 2), padding=1, groups=m // g), p.s2, p.t2))
    z = F.adaptive_avg_pool2d(h2, 1)
    gate = torch.sigmoid(F.conv2d(F.relu(F.conv2d(z, t(e.w_se1)[:, :, None, None], t(e.b_se1))),
                                  t(e.w_se2)[:, :, None, None], t(e.b_se2)))
    want = F.relu(xt + aff(F.conv2d(h2 * gate, t(p.w3)[:, :, None, None]), p.s3, p.t3)).permute(0, 2, 3, 1).numpy()
    ones = np.ones((N, H // S, W // S), np.uint8)
    np.testing.assert_allclose(O.dyn_group_se_bottleneck(x, p, e, S, ones), want, rtol=1e-11, atol=1e-11)
    # the group convolution alone against the library's
    hh = rng.standard_normal((N, H, W, m))
    np.testing.assert_allclose(O.group_conv3x3(hh, p.w2, g),
                               F.conv2d(t(hh).permute(0, 3, 1, 2), t(p.w2).permute(0, 3, 1, 2), padding=1,
                                        groups=m // g).permute(0, 2, 3, 1).numpy(), rtol=1e-11, atol=1e-11)
    # layer skipping (S = H = W): kept samples get exactly this static block, the others stay as they are
    Hs = 4
    xs = rng.standard_normal((3, Hs, Hs, c))
    keep = np.array([1, 0, 1], np.uint8).reshape(3, 1, 1)
    full = O.dyn_group_se_bottleneck(xs, p, e, 1, np.ones((3, Hs, Hs), np.uint8))
    got = O.dyn_group_se_bottleneck(xs, p, e, Hs, keep)
    np.testing.assert_allclose(got[[0, 2]], full[[0, 2]], rtol=1e-12, atol=1e-12)
    assert np.array_equal(got[1], xs[1])


def test_group_se_block_reductions_and_locality():
    rng = np.random.default_rng(83)
    N, H, W, c, m, S = 2, 8, 8, 4, 6, 2
    x = rng.standard_normal((N, H, W, c))
    mask = (rng.random((N, H // S, W // S)) < 0.4).astype(np.uint8)
    # one group as wide as the layer and a gate pinned at 1: the plain dynamic bottleneck
    p, e = _rand_group_se(rng, c, m, m, 2, True)
    e.w_se2 = np.zeros_like(e.w_se2)
    e.b_se2 = np.full(m, 50.0)
    np.testing.assert_allclose(O.dyn_group_se_bottleneck(x, p, e, S, mask), O.dyn_bottleneck(x, p, S, mask),
                               rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(O.dyn_group_se_bottleneck(x, p, O.GroupSE(m), S, mask), O.dyn_bottleneck(x, p, S, mask),
                               rtol=0, atol=0)
    # a gate pinned at 1/2 (zero logits) halves the branch input of the last 1x1
    p2, e2 = _rand_group_se(rng, c, m, 3, 2, False)
    e2.w_se2 = np.zeros_like(e2.w_se2)
    e2.b_se2 = np.zeros(m)
    half = O.BottleneckParams(p2.w1, p2.w2, 0.5 * p2.w3, p2.s1, p2.t1, p2.s2, p2.t2, p2.s3, p2.t3, False)
    np.testing.assert_allclose(O.dyn_group_se_bottleneck(x, p2, e2, S, mask),
                               O.dyn_group_se_bottleneck(x, half, O.GroupSE(3), S, mask), rtol=1e-12, atol=1e-12)
    # group-convolution weights embedded block-diagonally in a full 3x3 give the same block
    p3, e3 = _rand_group_se(rng, c, m, 2, 3, True)
    wfull = np.zeros((m, 3, 3, m))
    for o in range(m):
        wfull[o, :, :, (o // 2) * 2:(o // 2) * 2 + 2] = p3.w2[o]
    pf = O.BottleneckParams(p3.w1, wfull, p3.w3, p3.s1, p3.t1, p3.s2, p3.t2, p3.s3, p3.t3, True)
    ef = O.GroupSE(m, e3.w_se1, e3.b_se1, e3.w_se2, e3.b_se2)
    a = O.dyn_group_se_bottleneck(x, p3, e3, S, mask)
    np.testing.assert_allclose(a, O.dyn_group_se_bottleneck(x, pf, ef, S, mask), rtol=1e-12, atol=1e-12)
    # locality of the sparse evaluation: the result depends on x only inside the one-pixel dilation of the
    # active patches (the squeeze included, since it averages over active pixels only)
    up = O.upsample_mask(mask, S).astype(bool)
    pad = np.zeros((N, H + 2, W + 2), bool)
    pad[:, 1:-1, 1:-1] = up
    dil = np.zeros_like(up)
    for dy in range(3):
        for dx in range(3):
            dil |= pad[:, dy:dy + H, dx:dx + W]
    x2 = np.where(dil[..., None], x, x + rng.standard_normal(x.shape))
    b = O.dyn_group_se_bottleneck(x2, p3, e3, S, mask)
    assert np.array_equal(a[up], b[up])


def _bf_group_se_proj(x, p, e, wsc, ssc, tsc, stride, S, mask):
    """Explicit loops: strided shortcut everywhere; at active output pixels the group 3x3 (stride on it) from
    h1 with zero padding, the squeeze over exactly those pixels, gate, last 1x1."""
    import math
    xl, pl = np.asarray(x, np.float64).tolist(), _as_lists(p)
    N, H, W, C = np.shape(x)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    m, g, co = len(pl["w1"]), e.g, len(pl["w3"])
    out = np.zeros((N, Ho, Wo, co))
    for n in range(N):
        act = [(yo, xo) for yo in range(Ho) for xo in range(Wo) if mask[n][yo // S][xo // S]]
        h2 = {}
        for (yo, xo) in act:
            row = []
            for j in range(m):
                acc = 0.0
                for ky in range(3):
                    for kx in range(3):
                        for c in range(g):
                            acc += pl["w2"][j][ky][kx][c] * _bf_h1(xl, pl, n, stride * yo + ky - 1, stride * xo + kx - 1,
                                                                 (j // g) * g + c)
                v = pl["s2"][j] * acc + pl["t2"][j]
                row.append(v if v > 0.0 else 0.0)
            h2[(yo, xo)] = row
        gate = [1.0] * m
        if act and e.w_se1 is not None:
            z = [sum(h2[q][j] for q in act) / len(act) for j in range(m)]
            w1, b1, w2, b2 = (np.asarray(a, np.float64).tolist() for a in (e.w_se1, e.b_se1, e.w_se2, e.b_se2))
            hid = [max(sum(w1[k][j] * z[j] for j in range(m)) + b1[k], 0.0) for k in range(len(b1))]
            gate = [1.0 / (1.0 + math.exp(-(sum(w2[j][k] * hid[k] for k in range(len(hid))) + b2[j]))) for j in range(m)]
        for yo in range(Ho):
            for xo in range(Wo):
                for o in range(co):
                    v = ssc[o] * sum(wsc[o][c] * xl[n][stride * yo][stride * xo][c] for c in range(C)) + tsc[o]
                    if (yo, xo) in h2:
                        f = sum(pl["w3"][o][j] * h2[(yo, xo)][j] * gate[j] for j in range(m))
                        v += pl["s3"][o] * f + pl["t3"][o]
                    out[n, yo, xo, o] = 0.0 if (p.relu_out and v < 0.0) else v
    return out


@pytest.mark.parametrize("stride,H,W,S,g,se_w", [(2, 4, 4, 1, 2, 3), (2, 4, 4, 2, 2, 0), (1, 2, 2, 1, 4, 2), (2, 5, 3, 1, 1, 2),
                                                 (2, 8, 4, 2, 2, 3)])
def test_group_se_projection_block_vs_bruteforce_all_masks(stride, H, W, S, g, se_w):
    rng = np.random.default_rng(900 + 10 * H + S + stride)
    N, c_in, m, c_out = 1, 3, 4, 5
    x = rng.standard_normal((N, H, W, c_in))
    p = _rand_params(rng, c_in, m, c_out, True)
    p.w2 = rng.standard_normal((m, 3, 3, g)) * 0.5
    e = O.GroupSE(g, rng.standard_normal((se_w, m)), 0.3 * rng.standard_normal(se_w), rng.standard_normal((m, se_w)),
                  0.3 * rng.standard_normal(m)) if se_w else O.GroupSE(g)
    wsc, ssc, tsc = rng.standard_normal((c_out, c_in)), 1 + 0.3 * rng.standard_normal(c_out), rng.standard_normal(c_out)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    hp, wp = Ho // S, Wo // S
    for bits in itertools.product([0, 1], repeat=hp * wp):
        mask = np.array(bits, np.uint8).reshape(N, hp, wp)
        got = O.dyn_group_se_projection_bottleneck(x, p, e, wsc, ssc, tsc, stride, S, mask)
        want = _bf_group_se_proj(x, p, e, wsc.tolist(), ssc.tolist(), tsc.tolist(), stride, S, mask)
        np.testing.assert_allclose(got, want, rtol=1e-11, atol=1e-11)


def test_group_se_projection_block_special_cases():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(91)
    N, H, W, c_in, m, c_out, g, se_w, stride, S = 2, 8, 12, 6, 8, 10, 4, 3, 2, 2
    x = rng.standard_normal((N, H, W, c_in))
    p = _rand_params(rng, c_in, m, c_out, True)
    p.w2 = rng.standard_normal((m, 3, 3, g)) * 0.5
    e = O.GroupSE(g, rng.standard_normal((se_w, m)), 0.3 * rng.standard_normal(se_w), rng.standard_normal((m, se_w)),
                  0.3 * rng.standard_normal(m))
    wsc, ssc, tsc = rng.standard_normal((c_out, c_in)), 1 + 0.2 * rng.standard_normal(c_out), rng.standard_normal(c_out)
    Ho, Wo = H // stride, W // stride
    ones = np.ones((N, Ho // S, Wo // S), np.uint8)
    # every location active: the static strided block as a composition of library routines
    t = lambda a: torch.from_numpy(np.asarray(a, np.float64))
    aff = lambda z, s, b: z * t(s).view(1, -1, 1, 1) + t(b).view(1, -1, 1, 1)
    xt = t(x).permute(0, 3, 1, 2)
    h1 = F.relu(aff(F.conv2d(xt, t(p.w1)[:, :, None, None]), p.s1, p.t1))
    h2 = F.relu(aff(F.conv2d(h1, t(p.w2).permute(0, 3, 1, 2), stride=stride, padding=1, groups=m // g), p.s2, p.t2))
    gate = torch.sigmoid(F.conv2d(F.relu(F.conv2d(F.adaptive_avg_pool2d(h2, 1), t(e.w_se1)[:, :, None, None], t(e.b_se1))),
                                  t(e.w_se2)[:, :, None, None], t(e.b_se2)))
    sc = aff(F.conv2d(xt, t(wsc)[:, :, None, None], stride=stride), ssc, tsc)
    want = F.relu(sc + aff(F.conv2d(h2 * gate, t(p.w3)[:, :, None, None]), p.s3, p.t3)).permute(0, 2, 3, 1).numpy()
    np.testing.assert_allclose(O.dyn_group_se_projection_bottleneck(x, p, e, wsc, ssc, tsc, stride, S, ones), want,
                               rtol=1e-11, atol=1e-11)
    # one group as wide as the layer and no SE module: the plain dynamic first block
    mk = (rng.random(ones.shape) < 0.5).astype(np.uint8)
    pf = _rand_params(rng, c_in, m, c_out, True)
    np.testing.assert_allclose(O.dyn_group_se_projection_bottleneck(x, pf, O.GroupSE(m), wsc, ssc, tsc, stride, S, mk),
                               O.dyn_projection_bottleneck(x, pf, wsc, ssc, tsc, stride, S, mk), rtol=1e-12, atol=1e-12)
    # stride 1: the group convolution with a stride reduces to the one without
    hh = rng.standard_normal((N, H, W, m))
    np.testing.assert_allclose(O.group_conv2d(hh, p.w2, g, 1), O.group_conv3x3(hh, p.w2, g), rtol=1e-12, atol=1e-12)
    # nothing active: the activated shortcut alone
    np.testing.assert_allclose(O.dyn_group_se_projection_bottleneck(x, p, e, wsc, ssc, tsc, stride, S, 0 * ones),
                               F.relu(sc).permute(0, 2, 3, 1).numpy(), rtol=1e-11, atol=1e-11)


def test_stem3x3_vs_torch_and_hand_case():
    torch = pytest.importorskip("torch")
    F = torch.nn.functional
    rng = np.random.default_rng(95)
    for (H, W) in ((8, 8), (9, 7)):
        x = rng.standard_normal((2, H, W, 3))
        w = rng.standard_normal((5, 3, 3, 3))
        s, b = 1 + 0.2 * rng.standard_normal(5), rng.standard_normal(5)
        y = F.conv2d(torch.from_numpy(x).permute(0, 3, 1, 2), torch.from_numpy(w).permute(0, 3, 1, 2), stride=2, padding=1)
        want = F.relu(y * torch.from_numpy(s).view(1, -1, 1, 1) + torch.from_numpy(b).view(1, -1, 1, 1)).permute(0, 2, 3, 1)
        np.testing.assert_allclose(O.stem3x3(x, w, s, b), want.numpy(), rtol=1e-12, atol=1e-12)
    # an all-ones 4x4 image under an all-ones kernel: the corner window holds 2x2 pixels, the others 3x2 / 2x3 / 3x3
    one = O.stem3x3(np.ones((1, 4, 4, 3)), np.ones((1, 3, 3, 3)), np.ones(1), np.zeros(1))[0, :, :, 0]
    assert np.array_equal(one, 3.0 * np.array([[4, 6], [6, 9]]))
