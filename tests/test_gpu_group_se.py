"""GPU parity of laud_dyn_group_se_bottleneck (group-convolution 3x3 + squeeze-and-excitation, the block of
the RegNetY backbones) against the CPU oracle, element by element on the same seeded inputs; tolerance
|gpu - ref| <= tol * (|ref| + rms(ref)), tol = 1e-4 (fp32) or 2e-2 (bf16); inactive pixels bit for bit."""
import numpy as np
import pytest

from oracle import laud_oracle as O
from paper_2308_15949_amd import inputs as I
from test_gpu_parity import G, TOL, assert_close, oracle_params  # noqa: F401  (G is a fixture)

pytestmark = pytest.mark.gpu


def run_group_se(G, x, hb, g, se, S, mask, inplace):
    t, L, D = G.torch, G.L, G.D
    xd = D.to_device(x, hb.dtype)
    fx = L.fmap_of(xd)
    db = D.DeviceBottleneck(hb)
    de = D.DeviceGroupSE(g, se)
    npatch = mask.size
    idx = t.zeros(npatch, dtype=t.int32, device="cuda")
    cnt = t.zeros(1, dtype=t.int32, device="cuda")
    L.laud_layer_skip_compact(t.from_numpy(np.ascontiguousarray(mask.reshape(-1))).cuda(), npatch, idx, cnt,
                              D.workspace(L.workspace_size(L.binding.OP_COMPACT, fx, None, npatch)))
    ws = D.workspace(L.workspace_size(L.binding.OP_DYN_BOTTLENECK, fx, db.desc, S))
    ws.fill_(0xFF)  # NaN patterns: anything read before it is written shows up
    out = xd if inplace else t.full_like(xd, 123.0)
    L.laud_dyn_group_se_bottleneck(xd, fx, db.desc, de.desc, S, idx, cnt, out, ws)
    t.cuda.synchronize()
    return D.to_host(out)


def check_group_se(got, x, hb, g, se, S, mask):
    e = O.GroupSE(g, *se) if se is not None else O.GroupSE(g)
    ref = O.dyn_group_se_bottleneck(x, oracle_params(hb), e, S, mask)
    up = O.upsample_mask(mask, S).astype(bool)
    assert np.array_equal(got[~up], x[~up])
    assert_close(got[up], ref[up], TOL[hb.dtype], "active pixels")


CASES = [
    # N, H, W, C, g, se_width, S, dtype, relu_out, ratio
    (2, 8, 8, 32, 8, 8, 2, I.F32, True, 0.5),
    (2, 8, 8, 32, 8, 0, 2, I.F32, False, 0.5),      # group convolution only
    (3, 12, 8, 48, 16, 12, 4, I.F32, True, 0.5),    # 48 channels: one ragged 64-channel window
    (2, 14, 14, 144, 16, 16, 2, I.BF16, True, 0.5),  # RegNetY-800MF stage 2 width: windows 64 + 64 + 16
    (4, 14, 14, 320, 16, 80, 2, I.BF16, True, 0.5),  # RegNetY-800MF stage 3
    (3, 7, 7, 784, 16, 80, 1, I.BF16, True, 0.5),    # RegNetY-800MF stage 4
    (2, 56, 56, 64, 16, 8, 4, I.BF16, True, 0.4),    # RegNetY-800MF stage 1
    (2, 28, 28, 104, 8, 12, 4, I.BF16, True, 0.6),   # RegNetY-400MF stage 2 (group width 8)
    (3, 14, 14, 208, 8, 26, 7, I.BF16, False, 0.5),  # RegNetY-400MF stage 3 at S = 7
    (2, 7, 7, 440, 8, 52, 1, I.F32, True, 0.5),      # RegNetY-400MF stage 4, fp32
    (2, 12, 12, 128, 32, 32, 3, I.BF16, True, 0.5),
    (2, 12, 12, 128, 64, 16, 2, I.F32, True, 0.5),
    (2, 8, 8, 64, 64, 16, 2, I.BF16, True, 0.5),     # one group as wide as the layer
    (40, 14, 14, 320, 16, 80, 2, I.BF16, True, 0.5),  # many row tiles
]


@pytest.mark.parametrize("case", CASES)
@pytest.mark.parametrize("inplace", [True, False])
def test_group_se_block_bernoulli(G, case, inplace):
    N, H, W, C, g, se_w, S, dt, relu_out, r = case
    x = I.feature_map(3000 + C + H, N, H, W, C, dt)
    hb = I.bottleneck_params(3100 + C, C, C, C, dt, relu_out, group_width=g)
    se = I.se_weights(3200 + C, C, se_w) if se_w else None
    mask = I.bernoulli_mask(9 + H + S + C, (N, H // S, W // S), r)
    got = run_group_se(G, x, hb, g, se, S, mask, inplace)
    check_group_se(got, x, hb, g, se, S, mask)


@pytest.mark.parametrize("dt", [I.F32, I.BF16])
@pytest.mark.parametrize("kind", ["ones", "zeros", "one_sample_empty", "single_patch", "layer_skip"])
def test_group_se_block_special_masks(G, dt, kind):
    N, H, W, C, g, se_w, S = 3, 8, 8, 80, 16, 20, 2
    if kind == "layer_skip":
        S = H
    x = I.feature_map(52, N, H, W, C, dt)
    hb = I.bottleneck_params(53, C, C, C, dt, relu_out=True, group_width=g)
    hb.t1 = np.abs(hb.t1) + 0.5  # positive conv1 shift: padding must be on h1, not on x
    se = I.se_weights(54, C, se_w)
    mk = np.zeros((N, H // S, W // S), np.uint8)
    if kind == "ones":
        mk[:] = 1
    elif kind == "one_sample_empty":
        mk[0] = I.bernoulli_mask(1, mk[0].shape, 0.5)
        mk[2] = 1
    elif kind == "single_patch":
        mk[1, 1, 2] = 1
    elif kind == "layer_skip":
        mk[0] = 1
        mk[2] = 1
    for inplace in (True, False):
        got = run_group_se(G, x, hb, g, se, S, mk, inplace)
        check_group_se(got, x, hb, g, se, S, mk)
        if kind == "zeros":
            assert np.array_equal(got, x)


def test_group_se_gate_pinned_matches_plain_block_kernels(G):
    """One group as wide as the layer and no SE module: the same result as laud_dyn_bottleneck, bit for bit
    (same arithmetic, same order: one 64-channel window is the whole reduction)."""
    t, L, D = G.torch, G.L, G.D
    from test_gpu_parity import run_dyn
    N, H, W, C, S, dt = 2, 8, 8, 64, 2, I.BF16
    x = I.feature_map(61, N, H, W, C, dt)
    hb = I.bottleneck_params(62, C, C, C, dt, True, group_width=C)
    mask = I.bernoulli_mask(63, (N, H // S, W // S), 0.5)
    a = run_group_se(G, x, hb, C, None, S, mask, False)
    b = run_dyn(G, x, hb, S, mask, False)
    assert np.array_equal(a, b)


def test_group_se_block_rejects_bad_arguments(G):
    t, L, D = G.torch, G.L, G.D
    N, H, W, C, S, dt = 1, 4, 4, 48, 2, I.F32
    x = I.feature_map(71, N, H, W, C, dt)
    hb = I.bottleneck_params(72, C, C, C, dt, True, group_width=8)
    xd = D.to_device(x, dt)
    fx = L.fmap_of(xd)
    db = D.DeviceBottleneck(hb)
    idx = t.zeros(4, dtype=t.int32, device="cuda")
    cnt = t.zeros(1, dtype=t.int32, device="cuda")
    ws = D.workspace(L.workspace_size(L.binding.OP_DYN_BOTTLENECK, fx, db.desc, S))
    for gw, want in [(0, L.binding.ERR_INVALID_ARG), (7, L.binding.ERR_INVALID_ARG), (5, L.binding.ERR_INVALID_ARG),
                     (24, L.binding.ERR_UNSUPPORTED), (12, L.binding.ERR_UNSUPPORTED)]:
        with pytest.raises(L.LaudError) as ei:
            L.laud_dyn_group_se_bottleneck(xd, fx, db.desc, L.make_group_se(gw), S, idx, cnt, xd, ws)
        assert ei.value.status == want, gw
    with pytest.raises(L.LaudError) as ei:
        L.laud_dyn_group_se_bottleneck(xd, fx, db.desc, None, S, idx, cnt, xd, ws)
    assert ei.value.status == L.binding.ERR_INVALID_ARG
    bad = L.GroupSE(8, 4, None, None, None, None)  # SE width without weights
    with pytest.raises(L.LaudError) as ei:
        L.laud_dyn_group_se_bottleneck(xd, fx, db.desc, bad, S, idx, cnt, xd, ws)
    assert ei.value.status == L.binding.ERR_INVALID_ARG
    t.cuda.synchronize()


# ------------------------------------------------------------------------------------------
# first block of a stage: stride on the group 3x3, projection shortcut, mask on the output grid
# ------------------------------------------------------------------------------------------
PROJ_CASES = [
    # N, H, W, c_in, c_out (= mid), g, se_width, stride, S, dtype, mask kind
    (2, 12, 8, 16, 32, 8, 4, 2, 1, I.F32, "bern"),
    (2, 12, 8, 16, 32, 8, 0, 2, 2, I.F32, "bern"),            # group convolution only
    (3, 9, 7, 40, 48, 16, 8, 2, 1, I.F32, "bern"),            # odd input size: Ho = 5, Wo = 4
    (2, 16, 16, 32, 64, 16, 8, 2, 4, I.BF16, "ones"),         # every location active: the static first block
    (2, 16, 16, 32, 64, 16, 8, 2, 4, I.BF16, "zeros"),
    (2, 16, 16, 32, 64, 16, 8, 1, 2, I.BF16, "one_sample_empty"),
    (2, 112, 112, 32, 64, 16, 8, 2, 4, I.BF16, "bern"),       # RegNetY-800MF: first block of stage 1
    (2, 56, 56, 64, 144, 16, 16, 2, 4, I.BF16, "bern"),       # ... stage 2
    (2, 28, 28, 144, 320, 16, 36, 2, 2, I.BF16, "bern"),      # ... stage 3
    (3, 14, 14, 320, 784, 16, 80, 2, 1, I.BF16, "bern"),      # ... stage 4
    (3, 14, 14, 320, 784, 16, 80, 2, 7, I.BF16, "bern"),      # ... as a layer gate (S = output size)
    (2, 28, 28, 104, 208, 8, 26, 2, 2, I.BF16, "ones"),       # RegNetY-400MF stage 3 (group width 8, SE width 26)
]


@pytest.mark.parametrize("case", PROJ_CASES)
def test_group_se_projection_block(G, case):
    t, L, D = G.torch, G.L, G.D
    N, H, W, ci, co, g, se_w, stride, S, dt, kind = case
    x = I.feature_map(3300 + ci + S, N, H, W, ci, dt)
    hb = I.bottleneck_params(3310 + ci, ci, co, co, dt, relu_out=True, s3_gain=0.5, group_width=g)
    hb.t1 = (np.abs(hb.t1) + 0.25).astype(np.float32)   # positive conv1 shift: the 3x3's padding must be on h1
    se = I.se_weights(3320 + ci, co, se_w) if se_w else None
    gs = np.random.default_rng(3330 + ci)
    wsc = I.round_to(gs.standard_normal((co, ci), dtype=np.float32) * np.float32(np.sqrt(2.0 / ci)), dt)
    ssc = (0.5 * (1 + 0.1 * gs.standard_normal(co))).astype(np.float32)
    tsc = (0.1 * gs.standard_normal(co)).astype(np.float32)
    Ho, Wo = (H - 1) // stride + 1, (W - 1) // stride + 1
    shape = (N, Ho // S, Wo // S)
    if kind == "bern":
        mask = I.bernoulli_mask(3340 + S + H, shape, 0.5)
    elif kind == "ones":
        mask = np.ones(shape, np.uint8)
    elif kind == "zeros":
        mask = np.zeros(shape, np.uint8)
    else:
        mask = I.bernoulli_mask(3341, shape, 0.5)
        mask[0] = 0
    e = O.GroupSE(g, *se) if se is not None else O.GroupSE(g)
    ref = O.dyn_group_se_projection_bottleneck(x, oracle_params(hb), e, wsc, ssc, tsc, stride, S, mask)
    xd = D.to_device(x, dt)
    fx = L.fmap_of(xd)
    db = D.DeviceBottleneck(hb)
    de = D.DeviceGroupSE(g, se)
    npatch = mask.size
    idx = t.zeros(npatch, dtype=t.int32, device="cuda")
    cnt = t.zeros(1, dtype=t.int32, device="cuda")
    L.laud_layer_skip_compact(t.from_numpy(np.ascontiguousarray(mask.reshape(-1))).cuda(), npatch, idx, cnt,
                              D.workspace(L.workspace_size(L.binding.OP_COMPACT, fx, None, npatch)))
    out = t.full(ref.shape, 7.0, dtype=xd.dtype, device="cuda")
    ws = D.workspace(L.dyn_projection_workspace(fx, db.desc, stride))
    ws.fill_(0xFF)  # NaN patterns: anything read before it is written shows up
    print(f"group/SE projection case {case}", flush=True)
    L.laud_dyn_group_se_projection_bottleneck(xd, fx, db.desc, de.desc, D.to_device(wsc, dt), t.from_numpy(ssc).cuda(),
                                              t.from_numpy(tsc).cuda(), stride, S, idx, cnt, out, ws)
    t.cuda.synchronize()
    assert np.array_equal(D.to_host(xd), x)   # the input is left alone
    assert_close(D.to_host(out), ref, TOL[dt], "group/SE first block")


@pytest.mark.parametrize("stage", [1, 3, 4])
def test_group_se_block_full_batch_sampled(G, stage):
    """The bench shapes (RegNetY-800MF stage blocks, batch 128, bf16, masker-calibrated ratio 0.5 replaced by a
    seeded Bernoulli mask): the whole batch runs on the GPU, the oracle checks a few samples (samples are
    independent: mask, squeeze and gate are per sample)."""
    cfg = I.REGNETY["800MF"]
    N, C, hw, g, S = 128, cfg["stages"][stage]["c"], cfg["stages"][stage]["hw"], cfg["g"], I.STAGES[stage]["S"]
    x8 = I.feature_map(3400 + stage, 8, hw, hw, C, I.BF16)
    x = np.concatenate([x8] * (N // 8), axis=0)
    hb = I.bottleneck_params(3410 + stage, C, C, C, I.BF16, True, s3_gain=0.25, group_width=g)
    se = I.se_weights(3420 + stage, C, C // 4)
    mask = I.bernoulli_mask(3430 + stage, (N, hw // S, hw // S), 0.5)
    mask[5] = 0      # a sample without active patches in the middle of the batch
    mask[6] = 1
    got = run_group_se(G, x, hb, g, se, S, mask, True)
    for n in (0, 5, 6, 37, 127):
        check_group_se(got[n:n + 1], x[n:n + 1], hb, g, se, S, mask[n:n + 1])
