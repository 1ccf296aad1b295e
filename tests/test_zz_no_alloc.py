"""The allocation-free entry point (laud_dyn_bottleneck_noalloc) against laud_dyn_bottleneck: same inputs, same
index list, results bit for bit equal (the two share their kernels; only where the scratch activations live
differs), on two calls in a row, the second with a smaller input, and both also within the oracle's tolerance.
Also: a shape beyond the fixed scratch array is refused with LAUD_ERR_SCRATCH_LIMIT before any launch."""
import numpy as np
import pytest

from oracle import laud_oracle as O
from paper_2308_15949_amd import inputs as I

pytestmark = pytest.mark.gpu

TOL = {I.F32: 1e-4, I.BF16: 2e-2}


def _case(t, L, D, seed, N, H, C, m, S, dt, ratio):
    x = I.feature_map(seed, N, H, H, C, dt)
    hb = I.bottleneck_params(seed + 1, C, m, C, dt, relu_out=True)
    mask = I.bernoulli_mask(seed + 2, (N, H // S, H // S), ratio)
    ref_idx = O.compact(mask)
    xd = D.to_device(x, dt)
    fx = L.fmap_of(xd)
    db = D.DeviceBottleneck(hb)
    idx = t.zeros(mask.size, dtype=t.int32, device="cuda")
    idx[: len(ref_idx)] = t.from_numpy(ref_idx.astype(np.int32)).cuda()
    cnt = t.tensor([len(ref_idx)], dtype=t.int32, device="cuda")
    # existing entry point, caller workspace, out of place
    ws = D.workspace(L.workspace_size(L.binding.OP_DYN_BOTTLENECK, fx, db.desc, S))
    out_ws = t.full_like(xd, 7.0)
    L.laud_dyn_bottleneck(xd, fx, db.desc, S, idx, cnt, out_ws, ws)
    # allocation-free entry point
    out_na = t.full_like(xd, -3.0)
    L.laud_dyn_bottleneck_noalloc(xd, fx, db.desc, S, idx, cnt, out_na)
    t.cuda.synchronize()
    a, b = D.to_host(out_ws), D.to_host(out_na)
    assert np.array_equal(a.view(np.uint32), b.view(np.uint32)), "no-alloc result differs from laud_dyn_bottleneck"
    p = O.BottleneckParams(hb.w1, hb.w2, hb.w3, hb.s1, hb.t1, hb.s2, hb.t2, hb.s3, hb.t3, hb.relu_out)
    ref = O.dyn_bottleneck(x, p, S, mask)
    rms = float(np.sqrt(np.mean(ref * ref)))
    err = np.abs(b.astype(np.float64) - ref)
    assert np.all(err <= TOL[dt] * (np.abs(ref) + rms)), f"max err {err.max():.3e}"
    # in place as well
    L.laud_dyn_bottleneck_noalloc(xd, fx, db.desc, S, idx, cnt, xd)
    t.cuda.synchronize()
    assert np.array_equal(D.to_host(xd).view(np.uint32), a.view(np.uint32))


def test_noalloc_matches_workspace_entry_point_on_two_calls_the_second_smaller():
    import torch as t
    import paper_2308_15949_amd as L
    from paper_2308_15949_amd import device as D
    L.load()
    L.laud_init()
    # first call: batch 6 of a 28 x 28 x 128 bf16 map (several row tiles, ragged tail); second: one 14 x 14 x 64
    # float32 image -- smaller in every dimension, so stale contents of the shared scratch array lie beyond and
    # inside what the second call uses
    _case(t, L, D, 4100, 6, 28, 128, 32, 4, I.BF16, 0.5)
    _case(t, L, D, 4200, 1, 14, 64, 16, 2, I.F32, 0.4)


def test_noalloc_refuses_shapes_beyond_its_scratch_array():
    import ctypes as C
    import torch as t
    import paper_2308_15949_amd as L
    B = L.binding
    lib = L.load()
    fx = B.Fmap(128, 14, 14, 1024, B.BF16)
    fake = 0x10000
    p = B.Bottleneck(1024, 256, 1024, *([fake] * 9), 0)
    assert L.workspace_size(B.OP_DYN_BOTTLENECK, fx, p, 2) > B.NOALLOC_SCRATCH_BYTES
    vp = C.c_void_p
    rc = lib.laud_dyn_bottleneck_noalloc(vp(fake), fx, C.byref(p), 2, vp(fake), vp(fake), vp(fake), None)
    assert rc == B.ERR_SCRATCH_LIMIT
    assert "SCRATCH_LIMIT" in L.status_string(rc)
