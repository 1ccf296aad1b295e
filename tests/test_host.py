"""CPU-only checks: the C-ABI library loads and exports what include/laud.h declares, argument
validation returns the documented codes before anything is launched, and the seeded input
generators behave (bf16 rounding against torch's conversion, bias placement, mask ratios)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2308_15949_amd as L
from paper_2308_15949_amd import binding as B
from paper_2308_15949_amd import inputs as I

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2308_15949_amd import build
        build.build(verbose=False)
    return L.load()


def test_header_symbols_are_exported(lib):
    with open(os.path.join(ROOT, "include", "laud.h")) as f:
        text = re.sub(r"/\*.*?\*/", "", f.read(), flags=re.S)
    declared = sorted(set(re.findall(r"\b(laud_[a-z0-9_]+)\s*\(", text)))
    assert declared == sorted(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert L.abi_version() == 4
    assert L.status_string(0) == "LAUD_OK"
    for code in (-1, -2, -3, -4):
        assert L.status_string(code).startswith("LAUD_ERR_")


def test_struct_layout_matches_header():
    assert C.sizeof(B.Fmap) == 20
    # 3 ints (+4 pad), 9 pointers, 1 int (+4 pad), 1 pointer
    assert C.sizeof(B.Bottleneck) == 16 + 72 + 8 + 8
    assert C.sizeof(B.GroupSE) == 8 + 32


FAKE = 0x10000  # never dereferenced: validation happens on the host before any launch


def _bn(c_in=64, m=16, c_out=64):
    return B.Bottleneck(c_in, m, c_out, *([FAKE] * 9), 0)


def test_workspace_sizes(lib):
    fx = B.Fmap(128, 14, 14, 1024, B.BF16)
    p = _bn(1024, 256, 1024)
    npix = 128 * 14 * 14
    dyn = L.workspace_size(B.OP_DYN_BOTTLENECK, fx, p, 2)
    packed = L.packed_weights_size(p, B.BF16)   # room for the per-call copy of the re-ordered weights
    assert packed == 256 * 1024 * 2 + (256 * 9 * 256 + 1024 * 256) * 2
    assert dyn >= 2 * npix * 256 * 2 + npix * 4 + packed and dyn < 2 * npix * 256 * 2 + npix * 4 + packed + 8192  # + small counters
    assert L.packed_weights_size(p, B.F32) == 0 and L.packed_weights_size(_bn(256, 64, 256), B.BF16) == 0
    cs = L.workspace_size(B.OP_CHANNEL_SKIP, fx, p, 4)   # h1 + h2, the sample order of the fused-kernel path, packed weights
    assert 2 * npix * 256 * 2 + packed <= cs < 2 * npix * 256 * 2 + packed + 8192
    assert L.workspace_size(B.OP_MASK_GEN, fx, None, 2) == 256
    assert L.workspace_size(B.OP_COMPACT, fx, None, 300001) >= 4 * 74
    assert L.workspace_size(B.OP_GATHER, fx, None, 2) == 0
    assert L.workspace_size(B.OP_MASK_GEN, fx, None, 3) == 0      # 3 does not divide 14
    assert L.workspace_size(99, fx, None, 2) == 0


def test_argument_validation_returns_codes_without_launching(lib):
    vp = C.c_void_p
    fx = B.Fmap(2, 8, 8, 64, B.F32)
    p = _bn()
    st = None
    # mask_gen
    f = lib.laud_mask_gen
    assert f(None, fx, 2, vp(FAKE), 0.0, None, vp(FAKE), vp(FAKE), vp(FAKE), None, None, None, 0, st) == B.ERR_INVALID_ARG
    assert f(vp(FAKE), fx, 3, vp(FAKE), 0.0, None, vp(FAKE), vp(FAKE), vp(FAKE), None, None, None, 0, st) == B.ERR_INVALID_ARG
    assert f(vp(FAKE), B.Fmap(2, 8, 8, 60, 0), 2, vp(FAKE), 0.0, None, vp(FAKE), vp(FAKE), vp(FAKE), None, None, None, 0, st) == B.ERR_UNSUPPORTED
    assert f(vp(FAKE), B.Fmap(2, 8, 8, 64, 7), 2, vp(FAKE), 0.0, None, vp(FAKE), vp(FAKE), vp(FAKE), None, None, None, 0, st) == B.ERR_INVALID_ARG
    big = B.Fmap(200, 56, 56, 64, 0)  # 200*196 patches > one compaction block: needs a workspace
    assert f(vp(FAKE), big, 4, vp(FAKE), 0.0, None, vp(FAKE), vp(FAKE), vp(FAKE), None, None, None, 0, st) == B.ERR_WORKSPACE
    # compact
    g = lib.laud_layer_skip_compact
    assert g(None, 5, vp(FAKE), vp(FAKE), None, 0, st) == B.ERR_INVALID_ARG
    assert g(vp(FAKE), -1, vp(FAKE), vp(FAKE), None, 0, st) == B.ERR_INVALID_ARG
    assert g(vp(FAKE), 100000, vp(FAKE), vp(FAKE), None, 0, st) == B.ERR_WORKSPACE
    # gather
    h = lib.laud_gather_patches
    assert h(vp(FAKE), fx, 2, 2, vp(FAKE), vp(FAKE), vp(FAKE), st) == B.ERR_INVALID_ARG
    assert h(vp(FAKE), fx, 5, 1, vp(FAKE), vp(FAKE), vp(FAKE), st) == B.ERR_INVALID_ARG
    assert h(vp(FAKE), fx, 2, 1, None, vp(FAKE), vp(FAKE), st) == B.ERR_INVALID_ARG
    # dyn bottleneck
    d = lib.laud_dyn_bottleneck
    need = L.workspace_size(B.OP_DYN_BOTTLENECK, fx, p, 2)
    assert d(vp(FAKE), fx, C.byref(p), 2, vp(FAKE), vp(FAKE), vp(FAKE), None, 0, st) == B.ERR_WORKSPACE
    assert d(vp(FAKE), fx, C.byref(p), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), need - 1, st) == B.ERR_WORKSPACE
    assert d(vp(FAKE), fx, C.byref(p), 3, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), need, st) == B.ERR_INVALID_ARG
    assert d(vp(FAKE), fx, None, 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), need, st) == B.ERR_INVALID_ARG
    assert d(vp(FAKE), fx, C.byref(_bn(32, 16, 32)), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), need, st) == B.ERR_INVALID_ARG  # C mismatch
    assert d(vp(FAKE), fx, C.byref(_bn(64, 16, 128)), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), need, st) == B.ERR_UNSUPPORTED
    assert d(vp(FAKE), fx, C.byref(_bn(64, 12, 64)), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), need, st) == B.ERR_UNSUPPORTED
    assert d(vp(FAKE), fx, C.byref(p), 2, vp(FAKE), vp(FAKE), vp(FAKE + 64), vp(FAKE), need, st) == B.ERR_INVALID_ARG  # partial overlap
    nullw = B.Bottleneck(64, 16, 64, 0, *([FAKE] * 8), 0)
    assert d(vp(FAKE), fx, C.byref(nullw), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), need, st) == B.ERR_INVALID_ARG
    # fused masker variant
    fm = lib.laud_masker_dyn_bottleneck
    assert fm(vp(FAKE), fx, C.byref(p), 2, None, 0.0, None, vp(FAKE), vp(FAKE), vp(FAKE), None, None, vp(FAKE), vp(FAKE), need, st) == B.ERR_INVALID_ARG
    assert fm(vp(FAKE), fx, C.byref(p), 2, vp(FAKE), 0.0, None, vp(FAKE), vp(FAKE), vp(FAKE), None, None, vp(FAKE), vp(FAKE), need - 1, st) == B.ERR_WORKSPACE
    assert fm(vp(FAKE), fx, C.byref(p), 3, vp(FAKE), 0.0, None, vp(FAKE), vp(FAKE), vp(FAKE), None, None, vp(FAKE), vp(FAKE), need, st) == B.ERR_INVALID_ARG
    # unfused schedule, static block, stem
    uf = lib.laud_dyn_bottleneck_unfused
    needu = lib.laud_dyn_bottleneck_unfused_workspace(fx, C.byref(p), 2)
    assert needu > need
    assert uf(vp(FAKE), fx, C.byref(p), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needu - 1, st) == B.ERR_WORKSPACE
    assert uf(vp(FAKE), fx, C.byref(p), 3, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needu, st) == B.ERR_INVALID_ARG
    sb = lib.laud_static_bottleneck
    pw = _bn(64, 16, 128)
    needs = lib.laud_static_bottleneck_workspace(fx, C.byref(pw), 2)
    assert needs >= 2 * 64 * 16 * 4 + 2 * 16 * 16 * 4
    assert sb(vp(FAKE), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 2, vp(FAKE + (1 << 20)), vp(FAKE), needs - 1, st) == B.ERR_WORKSPACE
    assert sb(vp(FAKE), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 3, vp(FAKE + (1 << 20)), vp(FAKE), needs, st) == B.ERR_INVALID_ARG
    assert sb(vp(FAKE), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 2, vp(FAKE), vp(FAKE), needs, st) == B.ERR_INVALID_ARG  # out == x
    assert sb(vp(FAKE), fx, C.byref(pw), None, vp(FAKE), vp(FAKE), 2, vp(FAKE + (1 << 20)), vp(FAKE), needs, st) == B.ERR_INVALID_ARG
    # dynamic first block of a stage (fx is 2 x 8 x 8 x 64: output 4 x 4 at stride 2)
    dp = lib.laud_dyn_projection_bottleneck
    needp = lib.laud_dyn_projection_workspace(fx, C.byref(pw), 2)
    assert needp >= 2 * 64 * 4 + 2 * 64 * 16 * 4 + 2 * 16 * 16 * 4
    assert lib.laud_dyn_projection_workspace(fx, C.byref(pw), 3) == 0
    far = vp(FAKE + (1 << 20))
    assert dp(vp(FAKE), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 2, 2, vp(FAKE), vp(FAKE), far, vp(FAKE), needp - 1, st) == B.ERR_WORKSPACE
    assert dp(vp(FAKE), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 2, 3, vp(FAKE), vp(FAKE), far, vp(FAKE), needp, st) == B.ERR_INVALID_ARG  # 3 does not divide 4
    assert dp(vp(FAKE), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 3, 2, vp(FAKE), vp(FAKE), far, vp(FAKE), needp, st) == B.ERR_INVALID_ARG  # stride
    assert dp(vp(FAKE), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 2, 2, None, vp(FAKE), far, vp(FAKE), needp, st) == B.ERR_INVALID_ARG       # no index list
    assert dp(vp(FAKE), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 2, 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needp, st) == B.ERR_INVALID_ARG  # out == x
    assert dp(vp(FAKE), fx, C.byref(_bn(64, 12, 128)), vp(FAKE), vp(FAKE), vp(FAKE), 2, 2, vp(FAKE), vp(FAKE), far, vp(FAKE), needp, st) == B.ERR_UNSUPPORTED
    # group-convolution / SE variant of the dynamic block
    gs = lib.laud_dyn_group_se_bottleneck
    pg = _bn(64, 64, 64)
    needg = L.workspace_size(B.OP_DYN_BOTTLENECK, fx, pg, 2)
    ge = lambda g, w=0, ptr=FAKE: C.byref(B.GroupSE(g, w, ptr, ptr, ptr, ptr))
    assert gs(vp(FAKE), fx, C.byref(pg), None, 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needg, st) == B.ERR_INVALID_ARG
    assert gs(vp(FAKE), fx, C.byref(pg), ge(0), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needg, st) == B.ERR_INVALID_ARG
    assert gs(vp(FAKE), fx, C.byref(pg), ge(24), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needg, st) == B.ERR_INVALID_ARG  # 24 does not divide 64
    assert gs(vp(FAKE), fx, C.byref(pg), ge(4), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needg, st) == B.ERR_UNSUPPORTED
    assert gs(vp(FAKE), fx, C.byref(pg), ge(16, 8, None), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needg, st) == B.ERR_INVALID_ARG
    assert gs(vp(FAKE), fx, C.byref(pg), ge(16, 2048), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needg, st) == B.ERR_UNSUPPORTED
    assert gs(vp(FAKE), fx, C.byref(pg), ge(16, -1), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needg, st) == B.ERR_INVALID_ARG
    assert gs(vp(FAKE), fx, C.byref(pg), ge(16, 8), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needg - 1, st) == B.ERR_WORKSPACE
    assert gs(vp(FAKE), fx, C.byref(pg), ge(16, 8), 3, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), needg, st) == B.ERR_INVALID_ARG  # 3 does not divide 8
    gp = lib.laud_dyn_group_se_projection_bottleneck
    pq = _bn(64, 128, 128)
    needq = lib.laud_dyn_projection_workspace(fx, C.byref(pq), 2)
    far = vp(FAKE + (1 << 20))
    assert gp(vp(FAKE), fx, C.byref(pq), None, vp(FAKE), vp(FAKE), vp(FAKE), 2, 2, vp(FAKE), vp(FAKE), far, vp(FAKE), needq, st) == B.ERR_INVALID_ARG
    assert gp(vp(FAKE), fx, C.byref(pq), ge(24), vp(FAKE), vp(FAKE), vp(FAKE), 2, 2, vp(FAKE), vp(FAKE), far, vp(FAKE), needq, st) == B.ERR_INVALID_ARG
    assert gp(vp(FAKE), fx, C.byref(pq), ge(4), vp(FAKE), vp(FAKE), vp(FAKE), 2, 2, vp(FAKE), vp(FAKE), far, vp(FAKE), needq, st) == B.ERR_UNSUPPORTED
    assert gp(vp(FAKE), fx, C.byref(pq), ge(16, 8), vp(FAKE), vp(FAKE), vp(FAKE), 2, 2, vp(FAKE), vp(FAKE), far, vp(FAKE), needq - 1, st) == B.ERR_WORKSPACE
    assert gp(vp(FAKE), fx, C.byref(pq), ge(16, 8), vp(FAKE), vp(FAKE), vp(FAKE), 2, 3, vp(FAKE), vp(FAKE), far, vp(FAKE), needq, st) == B.ERR_INVALID_ARG
    assert gp(vp(FAKE), fx, C.byref(pq), ge(16, 8), None, vp(FAKE), vp(FAKE), 2, 2, vp(FAKE), vp(FAKE), far, vp(FAKE), needq, st) == B.ERR_INVALID_ARG
    s3 = lib.laud_stem3x3
    assert s3(vp(FAKE), 2, 64, 64, 1, vp(FAKE), vp(FAKE), vp(FAKE), 36, vp(FAKE), st) == B.ERR_UNSUPPORTED
    assert s3(vp(FAKE), 2, 64, 64, 1, vp(FAKE), vp(FAKE), vp(FAKE), 512, vp(FAKE), st) == B.ERR_UNSUPPORTED
    assert s3(vp(FAKE), 2, 64, 64, 7, vp(FAKE), vp(FAKE), vp(FAKE), 32, vp(FAKE), st) == B.ERR_INVALID_ARG
    assert s3(vp(FAKE), 2, 0, 64, 1, vp(FAKE), vp(FAKE), vp(FAKE), 32, vp(FAKE), st) == B.ERR_INVALID_ARG
    assert s3(None, 2, 64, 64, 1, vp(FAKE), vp(FAKE), vp(FAKE), 32, vp(FAKE), st) == B.ERR_INVALID_ARG
    sm = lib.laud_stem
    nst = lib.laud_stem_workspace(2, 64, 64, 64, 1)
    assert nst >= 2 * 32 * 32 * (152 + 64) * 2
    assert sm(vp(FAKE), 2, 64, 64, 1, vp(FAKE), vp(FAKE), vp(FAKE), 64, vp(FAKE), vp(FAKE), nst - 1, st) == B.ERR_WORKSPACE
    assert sm(vp(FAKE), 2, 64, 64, 1, vp(FAKE), vp(FAKE), vp(FAKE), 60, vp(FAKE), vp(FAKE), 1 << 30, st) == B.ERR_UNSUPPORTED
    assert sm(vp(FAKE), 2, 64, 64, 5, vp(FAKE), vp(FAKE), vp(FAKE), 64, vp(FAKE), vp(FAKE), nst, st) == B.ERR_INVALID_ARG
    # channel masker
    km = lib.laud_channel_masker
    wsk = lib.laud_channel_masker_workspace(fx)
    assert wsk >= 2 * 64 * 4
    assert km(vp(FAKE), fx, None, vp(FAKE), 16, vp(FAKE), vp(FAKE), 4, vp(FAKE), None, vp(FAKE), wsk, st) == B.ERR_INVALID_ARG
    assert km(vp(FAKE), fx, vp(FAKE), vp(FAKE), 0, vp(FAKE), vp(FAKE), 4, vp(FAKE), None, vp(FAKE), wsk, st) == B.ERR_INVALID_ARG
    assert km(vp(FAKE), fx, vp(FAKE), vp(FAKE), 16, vp(FAKE), vp(FAKE), 4, vp(FAKE), None, vp(FAKE), wsk - 1, st) == B.ERR_WORKSPACE
    assert km(vp(FAKE), B.Fmap(2, 8, 8, 60, 0), vp(FAKE), vp(FAKE), 16, vp(FAKE), vp(FAKE), 4, vp(FAKE), None, vp(FAKE), wsk, st) == B.ERR_UNSUPPORTED
    # channel skip
    c = lib.laud_channel_skip_conv
    needc = L.workspace_size(B.OP_CHANNEL_SKIP, fx, p, 4)
    assert c(vp(FAKE), fx, C.byref(p), vp(FAKE), 3, vp(FAKE), vp(FAKE), needc, st) == B.ERR_INVALID_ARG  # 3 does not divide 16
    assert c(vp(FAKE), fx, C.byref(p), None, 4, vp(FAKE), vp(FAKE), needc, st) == B.ERR_INVALID_ARG
    assert c(vp(FAKE), fx, C.byref(p), vp(FAKE), 4, vp(FAKE), vp(FAKE), needc - 1, st) == B.ERR_WORKSPACE


def test_binding_raises_typed_error(lib):
    with pytest.raises(L.LaudError) as e:
        B._check(B.ERR_WORKSPACE, "laud_dyn_bottleneck")
    assert e.value.status == B.ERR_WORKSPACE and "workspace" in str(e.value)


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/liblaud.so")
    with pytest.raises(RuntimeError, match="no CPU fallback"):
        B.load()


# ----- input generators --------------------------------------------------------------------
def test_bf16_rounding_matches_torch():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(0)
    a = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 10.0 ** rng.integers(-20, 20, 20000),
                        np.array([0.0, -0.0, np.inf, -np.inf, 1.0, 1.00390625, 1.01171875, 3.4e38], np.float32)])
    want = torch.from_numpy(a).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16)
    assert np.array_equal(I.bf16_bits(a), want)
    assert np.array_equal(I.bf16_bits_to_f32(I.bf16_bits(a)), torch.from_numpy(a).to(torch.bfloat16).float().numpy())
    assert I.bf16_bits(np.array([np.nan], np.float32))[0] == 0x7FC0
    r = I.round_to(a[:100], I.BF16)
    assert np.array_equal(I.round_to(r, I.BF16), r)  # idempotent


def test_bias_for_ratio_hits_the_target_in_a_gap():
    rng = np.random.default_rng(1)
    lg = rng.standard_normal(6272)
    for r in (0.25, 0.5, 0.75):
        b, half = I.bias_for_ratio(lg, r)
        n_on = int((lg + b > 0).sum())
        assert abs(n_on - round(r * lg.size)) <= 16
        assert np.abs(lg + b).min() == pytest.approx(half)
    b, _ = I.bias_for_ratio(lg, 1.0)
    assert (lg + b > 0).all()
    b, _ = I.bias_for_ratio(lg, 0.0)
    assert not (lg + b > 0).any()


def test_masks_and_params_are_seeded_and_shaped():
    m1 = I.coherent_mask(3, 4, 7, 7, 0.5)
    assert m1.shape == (4, 7, 7) and np.all(m1.reshape(4, -1).sum(1) == 24)
    assert np.array_equal(m1, I.coherent_mask(3, 4, 7, 7, 0.5))
    assert I.coherent_mask(3, 2, 7, 7, 0.0).sum() == 0 and I.coherent_mask(3, 2, 7, 7, 1.0).sum() == 98
    hb = I.bottleneck_params(10, 64, 16, 64, I.BF16)
    assert hb.w1.shape == (16, 64) and hb.w2.shape == (16, 3, 3, 16) and hb.w3.shape == (64, 16)
    assert np.array_equal(I.round_to(hb.w2, I.BF16), hb.w2)
    assert abs(float(hb.w2.std()) - np.sqrt(2.0 / (9 * 16))) < 0.02
    assert I.seed_for(2, 5, 3) == 2035


def test_operands_beyond_the_32_bit_offset_range_are_refused(lib):
    """The kernels address one operand with 32-bit byte offsets (upper half reserved for 'reads as zero'): a
    feature map or scratch activation of 2 GiB or more is refused on the host, before anything is launched."""
    vp = C.c_void_p
    big = B.Fmap(4096, 56, 56, 256, B.BF16)          # 6.6 GB of bf16
    p = _bn(256, 64, 256)
    d = lib.laud_dyn_bottleneck
    assert d(vp(FAKE), big, C.byref(p), 4, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), 1 << 40, None) == B.ERR_UNSUPPORTED
    ok = B.Fmap(1024, 56, 56, 256, B.BF16)           # 1.6 GB: inside the range (fails later, on the workspace)
    assert d(vp(FAKE), ok, C.byref(p), 4, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), 16, None) == B.ERR_WORKSPACE
    f32 = B.Fmap(1024, 56, 56, 256, B.F32)           # the same shape in float32: 3.3 GB
    assert d(vp(FAKE), f32, C.byref(p), 4, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), 1 << 40, None) == B.ERR_UNSUPPORTED
    cs = lib.laud_channel_skip_conv
    assert cs(vp(FAKE), big, C.byref(p), vp(FAKE), 4, vp(FAKE), vp(FAKE), 1 << 40, None) == B.ERR_UNSUPPORTED


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU benchmark: --gpus N with N > 1 exits with a message before touching any GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)


def test_alignment_overlap_and_operand_range_are_checked_on_the_host(lib):
    """16-byte loads/stores need aligned bases; partial overlap of x and out is rejected on every block path;
    the 3x3's descriptor shift counts towards the 2 GiB operand limit."""
    vp = C.c_void_p
    fx = B.Fmap(2, 8, 8, 64, B.F32)
    p = _bn()
    st = None
    need = L.workspace_size(B.OP_DYN_BOTTLENECK, fx, p, 2)
    d = lib.laud_dyn_bottleneck
    assert d(vp(FAKE + 8), fx, C.byref(p), 2, vp(FAKE), vp(FAKE), vp(FAKE + 8), vp(FAKE), need, st) == B.ERR_UNSUPPORTED
    assert d(vp(FAKE), fx, C.byref(p), 2, vp(FAKE), vp(FAKE), vp(FAKE + (1 << 20) + 4), vp(FAKE), need, st) == B.ERR_UNSUPPORTED
    pm = _bn()
    pm.w2 = FAKE + 2
    assert d(vp(FAKE), fx, C.byref(pm), 2, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), need, st) == B.ERR_UNSUPPORTED
    # static / dynamic projection blocks: out [2,4,4,128] f32 = 16 KiB, x [2,8,8,64] f32 = 32 KiB
    pw = _bn(64, 16, 128)
    sb = lib.laud_static_bottleneck
    needs = lib.laud_static_bottleneck_workspace(fx, C.byref(pw), 2)
    far = vp(FAKE + (1 << 20))
    assert sb(vp(FAKE), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 2, vp(FAKE + 1024), vp(FAKE), needs, st) == B.ERR_INVALID_ARG  # out inside x
    assert sb(vp(FAKE + 1024), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 2, vp(FAKE), vp(FAKE), needs, st) == B.ERR_INVALID_ARG  # x starts inside out
    assert sb(vp(FAKE), fx, C.byref(pw), vp(FAKE + 4), vp(FAKE), vp(FAKE), 2, far, vp(FAKE), needs, st) == B.ERR_UNSUPPORTED       # shortcut weights misaligned
    dp = lib.laud_dyn_projection_bottleneck
    needp = lib.laud_dyn_projection_workspace(fx, C.byref(pw), 2)
    assert dp(vp(FAKE), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 2, 2, vp(FAKE), vp(FAKE), vp(FAKE + 2048), vp(FAKE), needp, st) == B.ERR_INVALID_ARG
    assert dp(vp(FAKE + 8), fx, C.byref(pw), vp(FAKE), vp(FAKE), vp(FAKE), 2, 2, vp(FAKE), vp(FAKE), far, vp(FAKE), needp, st) == B.ERR_UNSUPPORTED
    # a very wide map: N*H*W*C*2 bytes alone fits below the limit, with twice the (W+1)-pixel tap shift it does not
    wide = B.Fmap(1, 2, 130000, 4096, B.BF16)
    pwide = _bn(4096, 64, 4096)
    assert 2 * 130000 * 4096 * 2 < 0x7f000000 < 2 * 130000 * 4096 * 2 + 2 * 130001 * 4096 * 2
    assert d(vp(FAKE), wide, C.byref(pwide), 1, vp(FAKE), vp(FAKE), vp(FAKE), vp(FAKE), 1 << 40, st) == B.ERR_UNSUPPORTED


def test_no_environment_variable_is_read():
    """The launch path is a function of its arguments alone."""
    for name in os.listdir(os.path.join(ROOT, "paper_2308_15949_amd", "csrc")):
        if name.endswith((".hip", ".h")):
            with open(os.path.join(ROOT, "paper_2308_15949_amd", "csrc", name)) as f:
                assert "getenv" not in f.read(), name


def test_bench_reads_traffic_from_the_committed_counter_summary():
    """roofline.traffic comes from profiles/: the summary of the FETCH_SIZE / WRITE_SIZE runs carries one
    machine-readable line per kernel, and bench.py finds the dominant kernel's."""
    import importlib.util
    spec = importlib.util.spec_from_file_location("bench_mod", os.path.join(ROOT, "bench.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    v = mod.traffic_from_profile("k_tail")
    assert v is not None and 4e7 < v < 2e8   # tens of MB per launch at batch 128, ratio 0.5
    assert mod.traffic_from_profile("k_head") is not None
    assert mod.traffic_from_profile("no_such_kernel") is None
