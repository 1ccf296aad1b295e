"""Thin ctypes binding of liblaud.so: argument marshalling only.

Every function below has the name and the meaning of the C entry point declared in
include/laud.h; tensors are torch CUDA tensors used purely as device memory, the
stream is torch's current stream.  There is no CPU fallback: if the library has not
been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "liblaud.so")

F32, BF16 = 0, 1
OP_MASK_GEN, OP_COMPACT, OP_GATHER, OP_DYN_BOTTLENECK, OP_CHANNEL_SKIP = range(5)
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE, ERR_HIP, ERR_SCRATCH_LIMIT = 0, -1, -2, -3, -4, -5
NOALLOC_SCRATCH_BYTES = 16 << 20

EXPORTS = ["laud_status_string", "laud_abi_version", "laud_workspace_size", "laud_mask_gen",
           "laud_layer_skip_compact", "laud_gather_patches", "laud_dyn_bottleneck",
           "laud_channel_skip_conv", "laud_masker_dyn_bottleneck", "laud_channel_masker", "laud_channel_masker_workspace", "laud_dyn_bottleneck_unfused",
           "laud_dyn_bottleneck_unfused_workspace", "laud_static_bottleneck", "laud_static_bottleneck_workspace",
           "laud_stem", "laud_stem3x3", "laud_stem_workspace", "laud_dyn_projection_bottleneck", "laud_dyn_projection_workspace",
           "laud_dyn_group_se_bottleneck", "laud_dyn_group_se_projection_bottleneck", "laud_stage_timing_enable", "laud_stage_timing_read", "laud_stage_name",
           "laud_init", "laud_dyn_bottleneck_noalloc", "laud_probe_mfma", "laud_probe_copy", "laud_probe_read",
           "laud_packed_weights_size", "laud_pack_weights"]
STAGE_COUNT = 13


class Fmap(C.Structure):
    _fields_ = [("N", C.c_int32), ("H", C.c_int32), ("W", C.c_int32), ("C", C.c_int32), ("dtype", C.c_int32)]


class Bottleneck(C.Structure):
    _fields_ = [("c_in", C.c_int32), ("c_mid", C.c_int32), ("c_out", C.c_int32),
                ("w1", C.c_void_p), ("w2", C.c_void_p), ("w3", C.c_void_p),
                ("s1", C.c_void_p), ("t1", C.c_void_p), ("s2", C.c_void_p), ("t2", C.c_void_p),
                ("s3", C.c_void_p), ("t3", C.c_void_p), ("relu_out", C.c_int32), ("packed", C.c_void_p)]


class GroupSE(C.Structure):
    _fields_ = [("group_width", C.c_int32), ("se_width", C.c_int32), ("w_se1", C.c_void_p), ("b_se1", C.c_void_p),
                ("w_se2", C.c_void_p), ("b_se2", C.c_void_p)]


class LaudError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)}")


_lib = None


def load() -> C.CDLL:
    """Loads liblaud.so (once).  Raises if it has not been built: there is no fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2308_15949_amd.build` "
                           "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    vp, i32, sz = C.c_void_p, C.c_int, C.c_size_t
    lib.laud_status_string.restype = C.c_char_p
    lib.laud_status_string.argtypes = [i32]
    lib.laud_abi_version.restype = i32
    lib.laud_abi_version.argtypes = []
    lib.laud_workspace_size.restype = sz
    lib.laud_workspace_size.argtypes = [i32, Fmap, C.POINTER(Bottleneck), i32]
    lib.laud_mask_gen.restype = i32
    lib.laud_mask_gen.argtypes = [vp, Fmap, i32, vp, C.c_float, vp, vp, vp, vp, vp, vp, vp, sz, vp]
    lib.laud_layer_skip_compact.restype = i32
    lib.laud_layer_skip_compact.argtypes = [vp, i32, vp, vp, vp, sz, vp]
    lib.laud_gather_patches.restype = i32
    lib.laud_gather_patches.argtypes = [vp, Fmap, i32, i32, vp, vp, vp, vp]
    lib.laud_dyn_bottleneck.restype = i32
    lib.laud_dyn_bottleneck.argtypes = [vp, Fmap, C.POINTER(Bottleneck), i32, vp, vp, vp, vp, sz, vp]
    lib.laud_probe_mfma.restype = i32
    lib.laud_probe_mfma.argtypes = [i32, i32, i32, C.POINTER(C.c_double), vp, vp]
    lib.laud_probe_read.restype = i32
    lib.laud_probe_read.argtypes = [vp, sz, vp, vp]
    lib.laud_probe_copy.restype = i32
    lib.laud_probe_copy.argtypes = [vp, vp, sz, vp]
    lib.laud_packed_weights_size.restype = sz
    lib.laud_packed_weights_size.argtypes = [C.POINTER(Bottleneck), i32]
    lib.laud_pack_weights.restype = i32
    lib.laud_pack_weights.argtypes = [C.POINTER(Bottleneck), i32, vp, vp]
    lib.laud_init.restype = i32
    lib.laud_init.argtypes = []
    lib.laud_dyn_bottleneck_noalloc.restype = i32
    lib.laud_dyn_bottleneck_noalloc.argtypes = [vp, Fmap, C.POINTER(Bottleneck), i32, vp, vp, vp, vp]
    lib.laud_dyn_group_se_bottleneck.restype = i32
    lib.laud_dyn_group_se_bottleneck.argtypes = [vp, Fmap, C.POINTER(Bottleneck), C.POINTER(GroupSE), i32, vp, vp, vp, vp,
                                                 sz, vp]
    lib.laud_channel_skip_conv.restype = i32
    lib.laud_channel_skip_conv.argtypes = [vp, Fmap, C.POINTER(Bottleneck), vp, i32, vp, vp, sz, vp]
    lib.laud_masker_dyn_bottleneck.restype = i32
    lib.laud_masker_dyn_bottleneck.argtypes = [vp, Fmap, C.POINTER(Bottleneck), i32, vp, C.c_float, vp, vp, vp, vp,
                                               vp, vp, vp, vp, sz, vp]
    lib.laud_dyn_bottleneck_unfused_workspace.restype = sz
    lib.laud_dyn_bottleneck_unfused_workspace.argtypes = [Fmap, C.POINTER(Bottleneck), i32]
    lib.laud_dyn_bottleneck_unfused.restype = i32
    lib.laud_dyn_bottleneck_unfused.argtypes = [vp, Fmap, C.POINTER(Bottleneck), i32, vp, vp, vp, vp, sz, vp]
    lib.laud_static_bottleneck_workspace.restype = sz
    lib.laud_static_bottleneck_workspace.argtypes = [Fmap, C.POINTER(Bottleneck), i32]
    lib.laud_static_bottleneck.restype = i32
    lib.laud_static_bottleneck.argtypes = [vp, Fmap, C.POINTER(Bottleneck), vp, vp, vp, i32, vp, vp, sz, vp]
    lib.laud_dyn_projection_workspace.restype = sz
    lib.laud_dyn_projection_workspace.argtypes = [Fmap, C.POINTER(Bottleneck), i32]
    lib.laud_dyn_projection_bottleneck.restype = i32
    lib.laud_dyn_projection_bottleneck.argtypes = [vp, Fmap, C.POINTER(Bottleneck), vp, vp, vp, i32, i32, vp, vp, vp, vp,
                                                   sz, vp]
    lib.laud_dyn_group_se_projection_bottleneck.restype = i32
    lib.laud_dyn_group_se_projection_bottleneck.argtypes = [vp, Fmap, C.POINTER(Bottleneck), C.POINTER(GroupSE), vp, vp, vp,
                                                            i32, i32, vp, vp, vp, vp, sz, vp]
    lib.laud_stem_workspace.restype = sz
    lib.laud_stem_workspace.argtypes = [i32, i32, i32, i32, i32]
    lib.laud_stem.restype = i32
    lib.laud_stem.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, i32, vp, vp, sz, vp]
    lib.laud_stem3x3.restype = i32
    lib.laud_stem3x3.argtypes = [vp, i32, i32, i32, i32, vp, vp, vp, i32, vp, vp]
    lib.laud_channel_masker_workspace.restype = sz
    lib.laud_channel_masker_workspace.argtypes = [Fmap]
    lib.laud_channel_masker.restype = i32
    lib.laud_channel_masker.argtypes = [vp, Fmap, vp, vp, i32, vp, vp, i32, vp, vp, vp, sz, vp]
    lib.laud_stage_timing_enable.restype = i32
    lib.laud_stage_timing_enable.argtypes = [i32]
    lib.laud_stage_timing_read.restype = i32
    lib.laud_stage_timing_read.argtypes = [C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    lib.laud_stage_name.restype = C.c_char_p
    lib.laud_stage_name.argtypes = [i32]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load().laud_status_string(int(status)).decode()


def abi_version() -> int:
    return int(load().laud_abi_version())


# ----- marshalling helpers ---------------------------------------------------------------
def _ptr(t):
    """Device (or raw integer) pointer of a tensor; None -> NULL."""
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream():
    import torch
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _check(status: int, where: str) -> None:
    if status != OK:
        raise LaudError(status, where)


def fmap_of(x, dtype: int | None = None) -> Fmap:
    """Fmap of an [N,H,W,C] tensor (float32 or bfloat16)."""
    import torch
    if dtype is None:
        dtype = BF16 if x.dtype == torch.bfloat16 else F32
    n, h, w, c = x.shape
    return Fmap(int(n), int(h), int(w), int(c), int(dtype))


def make_bottleneck(w1, w2, w3, s1, t1, s2, t2, s3, t3, relu_out: bool) -> Bottleneck:
    """Bottleneck descriptor over device tensors w1 [m,Cin], w2 [m,3,3,m], w3 [Cout,m] and
    float32 affine vectors.  The caller keeps the tensors alive."""
    return Bottleneck(int(w1.shape[1]), int(w1.shape[0]), int(w3.shape[0]),
                      w1.data_ptr(), w2.data_ptr(), w3.data_ptr(),
                      s1.data_ptr(), t1.data_ptr(), s2.data_ptr(), t2.data_ptr(),
                      s3.data_ptr(), t3.data_ptr(), 1 if relu_out else 0)


def packed_weights_size(p: Bottleneck, dtype: int) -> int:
    return int(load().laud_packed_weights_size(C.byref(p), int(dtype)))


def laud_pack_weights(p: Bottleneck, dtype: int, packed) -> None:
    """Re-orders the block's weights into `packed` (device memory of packed_weights_size bytes); the caller then sets
    p.packed = packed.data_ptr() and keeps the tensor alive."""
    _check(load().laud_pack_weights(C.byref(p), int(dtype), _ptr(packed), _stream()), "laud_pack_weights")


def workspace_size(op: int, fx: Fmap, p: Bottleneck | None, s_or_d: int) -> int:
    return int(load().laud_workspace_size(int(op), fx, C.byref(p) if p is not None else None, int(s_or_d)))


def _ws_args(ws):
    if ws is None:
        return None, 0
    return _ptr(ws), int(ws.numel() * ws.element_size())


# ----- entry points (same names as the C ABI) ---------------------------------------------
def laud_mask_gen(x, fx: Fmap, S: int, w, bias: float, keep, mask, idx, count, sample_offsets, logits, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_mask_gen(_ptr(x), fx, int(S), _ptr(w), float(bias), _ptr(keep), _ptr(mask), _ptr(idx),
                                _ptr(count), _ptr(sample_offsets), _ptr(logits), wp, wb, _stream()),
           "laud_mask_gen")


def laud_layer_skip_compact(keep, n: int, idx, count, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_layer_skip_compact(_ptr(keep), int(n), _ptr(idx), _ptr(count), wp, wb, _stream()),
           "laud_layer_skip_compact")


def laud_gather_patches(x, fx: Fmap, S: int, halo: int, idx, count, out) -> None:
    _check(load().laud_gather_patches(_ptr(x), fx, int(S), int(halo), _ptr(idx), _ptr(count), _ptr(out), _stream()),
           "laud_gather_patches")


def laud_dyn_bottleneck(x, fx: Fmap, p: Bottleneck, S: int, idx, count, out, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_dyn_bottleneck(_ptr(x), fx, C.byref(p), int(S), _ptr(idx), _ptr(count), _ptr(out),
                                      wp, wb, _stream()), "laud_dyn_bottleneck")


def laud_probe_mfma(dtype: int, iters: int, blocks: int, sink) -> float:
    """Enqueues the bare MFMA loop; returns the FLOPs of the launch."""
    fl = C.c_double(0.0)
    _check(load().laud_probe_mfma(int(dtype), int(iters), int(blocks), C.byref(fl), _ptr(sink), _stream()), "laud_probe_mfma")
    return float(fl.value)


def laud_probe_copy(src, dst, nbytes: int) -> None:
    _check(load().laud_probe_copy(_ptr(src), _ptr(dst), int(nbytes), _stream()), "laud_probe_copy")


def laud_probe_read(src, nbytes: int, sink) -> None:
    _check(load().laud_probe_read(_ptr(src), int(nbytes), _ptr(sink), _stream()), "laud_probe_read")


def laud_init() -> None:
    _check(load().laud_init(), "laud_init")


def laud_dyn_bottleneck_noalloc(x, fx: Fmap, p: Bottleneck, S: int, idx, count, out) -> None:
    _check(load().laud_dyn_bottleneck_noalloc(_ptr(x), fx, C.byref(p), int(S), _ptr(idx), _ptr(count), _ptr(out),
                                              _stream()), "laud_dyn_bottleneck_noalloc")


def make_group_se(group_width: int, w_se1=None, b_se1=None, w_se2=None, b_se2=None) -> GroupSE:
    """Descriptor of the group-convolution / SE extension over float32 device tensors (w_se1 [se_width, c_mid],
    w_se2 [c_mid, se_width]); without tensors: group convolution only.  The caller keeps the tensors alive."""
    if w_se1 is None:
        return GroupSE(int(group_width), 0, None, None, None, None)
    return GroupSE(int(group_width), int(w_se1.shape[0]), w_se1.data_ptr(), b_se1.data_ptr(), w_se2.data_ptr(),
                   b_se2.data_ptr())


def laud_dyn_group_se_bottleneck(x, fx: Fmap, p: Bottleneck, e: GroupSE, S: int, idx, count, out, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_dyn_group_se_bottleneck(_ptr(x), fx, C.byref(p), C.byref(e) if e is not None else None, int(S),
                                               _ptr(idx), _ptr(count), _ptr(out), wp, wb, _stream()),
           "laud_dyn_group_se_bottleneck")


def laud_channel_skip_conv(x, fx: Fmap, p: Bottleneck, cmask, D: int, out, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_channel_skip_conv(_ptr(x), fx, C.byref(p), _ptr(cmask), int(D), _ptr(out),
                                         wp, wb, _stream()), "laud_channel_skip_conv")


def laud_masker_dyn_bottleneck(x, fx: Fmap, p: Bottleneck, S: int, w, bias: float, keep, mask, idx, count,
                               sample_offsets, logits, out, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_masker_dyn_bottleneck(_ptr(x), fx, C.byref(p), int(S), _ptr(w), float(bias), _ptr(keep),
                                             _ptr(mask), _ptr(idx), _ptr(count), _ptr(sample_offsets), _ptr(logits),
                                             _ptr(out), wp, wb, _stream()), "laud_masker_dyn_bottleneck")


def dyn_bottleneck_unfused_workspace(fx: Fmap, p: Bottleneck, S: int) -> int:
    return int(load().laud_dyn_bottleneck_unfused_workspace(fx, C.byref(p), int(S)))


def laud_dyn_bottleneck_unfused(x, fx: Fmap, p: Bottleneck, S: int, idx, count, out, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_dyn_bottleneck_unfused(_ptr(x), fx, C.byref(p), int(S), _ptr(idx), _ptr(count), _ptr(out),
                                              wp, wb, _stream()), "laud_dyn_bottleneck_unfused")


def static_bottleneck_workspace(fx: Fmap, p: Bottleneck, stride: int) -> int:
    return int(load().laud_static_bottleneck_workspace(fx, C.byref(p), int(stride)))


def laud_static_bottleneck(x, fx: Fmap, p: Bottleneck, w_sc, s_sc, t_sc, stride: int, out, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_static_bottleneck(_ptr(x), fx, C.byref(p), _ptr(w_sc), _ptr(s_sc), _ptr(t_sc), int(stride),
                                         _ptr(out), wp, wb, _stream()), "laud_static_bottleneck")


def dyn_projection_workspace(fx: Fmap, p: Bottleneck, stride: int) -> int:
    return int(load().laud_dyn_projection_workspace(fx, C.byref(p), int(stride)))


def laud_dyn_projection_bottleneck(x, fx: Fmap, p: Bottleneck, w_sc, s_sc, t_sc, stride: int, S: int, idx, count,
                                   out, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_dyn_projection_bottleneck(_ptr(x), fx, C.byref(p), _ptr(w_sc), _ptr(s_sc), _ptr(t_sc),
                                                 int(stride), int(S), _ptr(idx), _ptr(count), _ptr(out), wp, wb,
                                                 _stream()), "laud_dyn_projection_bottleneck")


def laud_dyn_group_se_projection_bottleneck(x, fx: Fmap, p: Bottleneck, e: GroupSE, w_sc, s_sc, t_sc, stride: int, S: int,
                                            idx, count, out, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_dyn_group_se_projection_bottleneck(_ptr(x), fx, C.byref(p), C.byref(e) if e is not None else None,
                                                          _ptr(w_sc), _ptr(s_sc), _ptr(t_sc), int(stride), int(S),
                                                          _ptr(idx), _ptr(count), _ptr(out), wp, wb, _stream()),
           "laud_dyn_group_se_projection_bottleneck")


def stem_workspace(n: int, hin: int, win: int, c_out: int, dtype: int) -> int:
    return int(load().laud_stem_workspace(int(n), int(hin), int(win), int(c_out), int(dtype)))


def laud_stem(x, n: int, hin: int, win: int, dtype: int, w7, s, t, c_out: int, out, ws) -> None:
    wp, wb = _ws_args(ws)
    _check(load().laud_stem(_ptr(x), int(n), int(hin), int(win), int(dtype), _ptr(w7), _ptr(s), _ptr(t), int(c_out),
                            _ptr(out), wp, wb, _stream()), "laud_stem")


def laud_stem3x3(x, n: int, hin: int, win: int, dtype: int, w3, s, t, c_out: int, out) -> None:
    _check(load().laud_stem3x3(_ptr(x), int(n), int(hin), int(win), int(dtype), _ptr(w3), _ptr(s), _ptr(t), int(c_out),
                               _ptr(out), _stream()), "laud_stem3x3")


def channel_masker_workspace(fx: Fmap) -> int:
    return int(load().laud_channel_masker_workspace(fx))


def laud_channel_masker(x, fx: Fmap, wa, ba, hidden: int, wb, bb, D: int, cmask, logits2, ws) -> None:
    wp, wb_ = _ws_args(ws)
    _check(load().laud_channel_masker(_ptr(x), fx, _ptr(wa), _ptr(ba), int(hidden), _ptr(wb), _ptr(bb), int(D),
                                      _ptr(cmask), _ptr(logits2), wp, wb_, _stream()), "laud_channel_masker")


def laud_stage_timing_enable(on: bool) -> None:
    _check(load().laud_stage_timing_enable(1 if on else 0), "laud_stage_timing_enable")


def laud_stage_timing_read() -> dict[str, tuple[float, int]]:
    """{stage name: (total milliseconds, launches)} for the stages that ran since enabling."""
    ms = (C.c_double * STAGE_COUNT)()
    n = (C.c_int64 * STAGE_COUNT)()
    _check(load().laud_stage_timing_read(ms, n), "laud_stage_timing_read")
    return {load().laud_stage_name(i).decode(): (float(ms[i]), int(n[i])) for i in range(STAGE_COUNT) if n[i]}
