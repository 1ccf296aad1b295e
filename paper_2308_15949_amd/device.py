"""Device-memory plumbing for the tests, the benchmark and the smoke check: host numpy arrays
(already rounded to the storage type) -> torch CUDA tensors, and back.  No arithmetic."""
from __future__ import annotations

import numpy as np

from . import binding as B
from .inputs import BF16, HostBottleneck


def to_device(a: np.ndarray, dtype: int, device: str = "cuda:0"):
    """float32 host array -> device tensor of the storage type (exact for pre-rounded values)."""
    import torch
    t = torch.from_numpy(np.ascontiguousarray(a, dtype=np.float32)).to(device)
    return t.to(torch.bfloat16).contiguous() if dtype == BF16 else t.contiguous()


def to_host(t) -> np.ndarray:
    """Device tensor (bf16/f32/int/uint8) -> numpy; bf16 widened to float32 exactly."""
    import torch
    if t.dtype == torch.bfloat16:
        t = t.float()
    return t.detach().cpu().numpy()


class DeviceBottleneck:
    """Holds the device tensors of one bottleneck and the C descriptor that points at them."""

    def __init__(self, hb: HostBottleneck, device: str = "cuda:0", prepack: bool = True):
        import torch
        self.hb = hb
        self.w1 = to_device(hb.w1, hb.dtype, device)
        self.w2 = to_device(hb.w2, hb.dtype, device)
        self.w3 = to_device(hb.w3, hb.dtype, device)
        f = lambda v: torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(device)
        self.s1, self.t1, self.s2, self.t2, self.s3, self.t3 = map(f, (hb.s1, hb.t1, hb.s2, hb.t2, hb.s3, hb.t3))
        self.desc = B.make_bottleneck(self.w1, self.w2, self.w3, self.s1, self.t1, self.s2, self.t2,
                                      self.s3, self.t3, hb.relu_out)
        # weights in the kernels' streaming order, made once (as when a model is loaded); prepack=False leaves the
        # re-ordering to every call
        self.packed = None
        plain = tuple(hb.w2.shape) == (hb.c_mid, 3, 3, hb.c_mid)   # (a group convolution's w2 has another shape)
        nb = B.packed_weights_size(self.desc, hb.dtype) if prepack and plain else 0
        if nb:
            self.packed = torch.empty(nb, dtype=torch.uint8, device=device)
            B.laud_pack_weights(self.desc, hb.dtype, self.packed)
            self.desc.packed = self.packed.data_ptr()


class DeviceGroupSE:
    """Device tensors of the SE module (if any) and the C descriptor of the group-conv / SE extension."""

    def __init__(self, group_width: int, se=None, device: str = "cuda:0"):
        import torch
        self.t = None
        if se is not None:
            self.t = [torch.from_numpy(np.ascontiguousarray(v, dtype=np.float32)).to(device) for v in se]
            self.desc = B.make_group_se(group_width, *self.t)
        else:
            self.desc = B.make_group_se(group_width)


def workspace(nbytes: int, device: str = "cuda:0"):
    import torch
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)
