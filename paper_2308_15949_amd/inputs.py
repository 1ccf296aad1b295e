"""Seeded synthetic inputs shared by the tests, the benchmark and the smoke check.

This module draws random tensors and rounds them to the storage type; it holds none
of the method's arithmetic (no convolution, no masker, no compaction), so the CPU
oracle and the HIP path can both be fed from it without sharing code.

Workload shapes follow the ResNet-50/101 bottleneck stages at 224x224 input and the
batch sizes of the paper's server-GPU experiments (Sec. 4: batch 128); values are
N(0,1) activations, Kaiming-normal (fan-in) weights and a non-trivial per-channel
affine standing for the folded BN, so that padding and shift mistakes are visible.
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

F32 = 0
BF16 = 1


# ----- storage-type rounding ------------------------------------------------ #
def bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bfloat16 bit patterns (uint16), round-to-nearest-even; NaN kept quiet."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    rounded = ((u.astype(np.uint64) + 0x7FFF + ((u >> 16) & 1)) >> 16).astype(np.uint16)
    nan = np.isnan(a)
    if nan.any():
        rounded = np.where(nan, np.uint16(0x7FC0), rounded)
    return rounded


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to(a: np.ndarray, dtype: int) -> np.ndarray:
    """The float32 array holding exactly the values the storage type can represent."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return bf16_bits_to_f32(bf16_bits(a)) if dtype == BF16 else a


# ----- tensors -------------------------------------------------------------- #
def feature_map(seed: int, n: int, h: int, w: int, c: int, dtype: int, nonneg: bool = False) -> np.ndarray:
    """x ~ N(0,1) as [N,H,W,C] float32 already rounded to `dtype`."""
    x = np.random.default_rng(seed).standard_normal((n, h, w, c), dtype=np.float32)
    if nonneg:
        x = np.abs(x)
    return round_to(x, dtype)


@dataclass
class HostBottleneck:
    """Host-side float32 copies (already rounded to the storage type) of one bottleneck."""
    c_in: int
    c_mid: int
    c_out: int
    w1: np.ndarray  # [m, C_in]
    w2: np.ndarray  # [m, 3, 3, m]  (out, ky, kx, in)
    w3: np.ndarray  # [C_out, m]
    s1: np.ndarray
    t1: np.ndarray
    s2: np.ndarray
    t2: np.ndarray
    s3: np.ndarray
    t3: np.ndarray
    relu_out: bool
    dtype: int


def bottleneck_params(seed: int, c_in: int, m: int, c_out: int, dtype: int,
                      relu_out: bool = False, s3_gain: float = 1.0, group_width: int | None = None) -> HostBottleneck:
    """Kaiming-normal weights (std = sqrt(2/fan_in)); affine s = 1 + 0.1 N(0,1),
    t = 0.1 N(0,1) in float32 (the affine is never rounded to bf16).  With group_width g the 3x3 is
    a group convolution: w2 [m, 3, 3, g], fan-in 9g."""
    g2 = m if group_width is None else group_width
    def w(k, shape, fan_in):
        g = np.random.default_rng(seed + k)
        return round_to(g.standard_normal(shape, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in)), dtype)

    ga = np.random.default_rng(seed + 4)
    aff = lambda ch, gain=1.0: (
        (gain * (1.0 + 0.1 * ga.standard_normal(ch))).astype(np.float32),
        (0.1 * ga.standard_normal(ch)).astype(np.float32),
    )
    s1, t1 = aff(m)
    s2, t2 = aff(m)
    s3, t3 = aff(c_out, s3_gain)
    return HostBottleneck(c_in, m, c_out,
                          w(1, (m, c_in), c_in), w(2, (m, 3, 3, g2), 9 * g2), w(3, (c_out, m), m),
                          s1, t1, s2, t2, s3, t3, relu_out, dtype)


def masker_weights(seed: int, c: int) -> np.ndarray:
    """One-channel spatial-masker weights ~ N(0, 1/C), float32."""
    return (np.random.default_rng(seed).standard_normal(c) / np.sqrt(c)).astype(np.float32)


# ----- masks ---------------------------------------------------------------- #
def bernoulli_mask(seed: int, shape: tuple[int, ...], p: float) -> np.ndarray:
    """Independent Bernoulli(p) decisions as uint8."""
    return (np.random.default_rng(seed).random(shape) < p).astype(np.uint8)


def coherent_mask(seed: int, n: int, hp: int, wp: int, r: float) -> np.ndarray:
    """Spatially coherent mask: a box-blurred N(0,1) field on the patch grid thresholded
    per sample at its (1-r) quantile, so active patches form contiguous regions like the
    object regions learned maskers select (Sec. 4, visualisation)."""
    g = np.random.default_rng(seed).standard_normal((n, hp + 2, wp + 2))
    f = np.zeros((n, hp, wp))
    for dy in range(3):
        for dx in range(3):
            f += g[:, dy:dy + hp, dx:dx + wp]
    k = int(round(r * hp * wp))
    out = np.zeros((n, hp * wp), np.uint8)
    if k > 0:
        order = np.argsort(-f.reshape(n, -1), axis=1, kind="stable")
        np.put_along_axis(out, order[:, :k], 1, axis=1)
    return out.reshape(n, hp, wp)


def bias_for_ratio(logits: np.ndarray, r: float, window: int = 16) -> tuple[float, float]:
    """Bias b such that (logits + b > 0) has close to r*size active entries, placed at the
    middle of the widest gap between adjacent sorted logits within `window` order
    statistics of the (1-r) quantile, so that rounding differences between two
    evaluations of the logits cannot flip a decision.  Returns (bias, half_gap).
    r >= 1 puts the threshold one standard deviation below the minimum; r <= 0 one above
    the maximum."""
    v = np.sort(np.asarray(logits, np.float64).reshape(-1))
    n = v.size
    sd = float(v.std()) or 1.0
    if r >= 1.0:
        return float(-(v[0] - sd)), sd
    if r <= 0.0:
        return float(-(v[-1] + sd)), sd
    k = int(round((1.0 - r) * n))  # threshold between v[k-1] and v[k]
    lo = max(1, k - window)
    hi = min(n - 1, k + window)
    gaps = v[lo:hi + 1] - v[lo - 1:hi]
    j = int(np.argmax(gaps)) + lo
    thr = 0.5 * (v[j - 1] + v[j])
    return float(-thr), float(0.5 * (v[j] - v[j - 1]))


# ----- named workloads ------------------------------------------------------ #
# (c_in, mid, H=W, S) of the identity bottlenecks of each ResNet-50/101 stage at 224^2,
# with the per-stage spatial granularity 4-4-2-1 used for LAUD-ResNet (Sec. 4).
STAGES = {
    1: dict(c_in=256, m=64, hw=56, S=4),
    2: dict(c_in=512, m=128, hw=28, S=4),
    3: dict(c_in=1024, m=256, hw=14, S=2),
    4: dict(c_in=2048, m=512, hw=7, S=1),
}


def seed_for(config: int, k: int, block: int = 0) -> int:
    """seed = 1000*config + 10*block + k; k: 0 x, 1..3 weights, 4 affine, 5 mask / masker
    weights, 6 channel masks, 7 layer gates."""
    return 1000 * config + 10 * block + k


def channel_masker_weights(seed: int, c: int, d: int, hidden: int | None = None):
    """Channel-masker MLP weights (float32): wa [hidden, C] ~ N(0, 2/C), ba ~ 0.1 N(0,1),
    wb [2D, hidden] ~ N(0, 1/hidden), bb ~ 0.1 N(0,1); hidden defaults to max(D // 16, 16)
    (Sec. 3.2 "Masker design")."""
    hidden = max(d // 16, 16) if hidden is None else hidden
    g = np.random.default_rng(seed)
    wa = (g.standard_normal((hidden, c)) * np.sqrt(2.0 / c)).astype(np.float32)
    ba = (0.1 * g.standard_normal(hidden)).astype(np.float32)
    wb = (g.standard_normal((2 * d, hidden)) / np.sqrt(hidden)).astype(np.float32)
    bb = (0.1 * g.standard_normal(2 * d)).astype(np.float32)
    return wa, ba, wb, bb, hidden


def se_weights(seed: int, c: int, se_width: int):
    """Squeeze-and-excitation weights (float32): w1 [se_width, C] ~ N(0, 2/C), b1 ~ 0.1 N(0,1),
    w2 [C, se_width] ~ N(0, 4/se_width) (so that the gates spread over (0,1)), b2 ~ 0.5 N(0,1)."""
    g = np.random.default_rng(seed)
    w1 = (g.standard_normal((se_width, c)) * np.sqrt(2.0 / c)).astype(np.float32)
    b1 = (0.1 * g.standard_normal(se_width)).astype(np.float32)
    w2 = (g.standard_normal((c, se_width)) * np.sqrt(4.0 / se_width)).astype(np.float32)
    b2 = (0.5 * g.standard_normal(c)).astype(np.float32)
    return w1, b1, w2, b2


# Identity blocks of the RegNetY-800MF stages at 224^2 (widths 64-144-320-784, group width 16, bottleneck
# ratio 1; the SE module's hidden width is a quarter of the block's input width) and of RegNetY-400MF
# (48-104-208-440, group width 8), the two lightweight backbones of Sec. 4.
REGNETY = {
    "800MF": dict(g=16, stages={1: dict(c=64, hw=56), 2: dict(c=144, hw=28), 3: dict(c=320, hw=14), 4: dict(c=784, hw=7)}),
    "400MF": dict(g=8, stages={1: dict(c=48, hw=56), 2: dict(c=104, hw=28), 3: dict(c=208, hw=14), 4: dict(c=440, hw=7)}),
}
