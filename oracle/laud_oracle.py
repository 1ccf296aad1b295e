"""CPU oracle for the LAUDNet dynamic-bottleneck hot path.  TEST INFRASTRUCTURE ONLY.

Plain numpy, float64 throughout, no blocking, no fusion, no reordering: every
function is the definition the paper gives, written out so that it can be
checked against the paper by eye.  Only the test-suite, the smoke check and the
``cpu_baseline`` leg of the benchmark may import this module; the product path
(the HIP library and its Python binding) never does, and this module imports
nothing from the product.

Tensor conventions (index order only; nothing here depends on memory layout):
    feature map x      [N, H, W, C]           (Sec. 3.1: x in R^{H x W x C}, batched)
    W1                 [m, C_in]              1x1 conv, out-channel major
    W2                 [m, 3, 3, m]           3x3 conv, [out, ky, kx, in], stride 1, zero pad 1
    W3                 [C_out, m]             1x1 conv
    s_k, t_k           per-channel affine that stands for the folded BN (Sec. 3.4,
                       general optimisations: BN and activation fused into the convs)
    coarse mask        [N, H/S, W/S] of {0,1} (Sec. 3.2, dynamic granularity)
    channel mask       [N, D] of {0,1}, D = m/G groups of G channels (Sec. 3.2)
    layer gate         [N] of {0,1}           (Sec. 3.1, dynamic layer skipping)

Pins (tests/test_oracle_pins.py): an independent per-output-element brute-force
evaluator on tiny inputs with every coarse mask enumerated; closed forms (box
filter neighbour counts 4/6/9, one-hot inputs); the library special case
(activation ratio 1 == a standard bottleneck == torch.nn.functional.conv2d
composition); the invariants ratio 1 == static block and ratio 0 == identity;
the two-logit argmax == one-channel difference > 0 identity of App. B; the
pool/1x1-conv commutation of App. B; the FLOP-ratio closed forms of Sec. 3.2;
the group-convolution + SE block against torch's grouped conv2d / pooling composition (all
active), a per-element brute force over every mask, and its reduction to dyn_bottleneck (the
strided first-block form likewise: brute force, torch composition, reduction to dyn_projection_bottleneck).
No function in this file is "parity unpinned".
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np


# --------------------------------------------------------------------------- #
# parameters
# --------------------------------------------------------------------------- #
@dataclass
class BottleneckParams:
    """Folded parameters of one residual bottleneck (Fig. 2; Sec. 3.4)."""

    w1: np.ndarray  # [m, C_in]
    w2: np.ndarray  # [m, 3, 3, m]
    w3: np.ndarray  # [C_out, m]
    s1: np.ndarray
    t1: np.ndarray
    s2: np.ndarray
    t2: np.ndarray
    s3: np.ndarray
    t3: np.ndarray
    relu_out: bool = False  # ReLU after the residual add (on computed pixels only)

    def as_f64(self) -> "BottleneckParams":
        f = lambda a: np.asarray(a, dtype=np.float64)
        return BottleneckParams(f(self.w1), f(self.w2), f(self.w3), f(self.s1), f(self.t1),
                                f(self.s2), f(self.t2), f(self.s3), f(self.t3), bool(self.relu_out))


# --------------------------------------------------------------------------- #
# dense building blocks (definitions)
# --------------------------------------------------------------------------- #
def conv1x1(x: np.ndarray, w: np.ndarray) -> np.ndarray:
    """out[n,y,x,o] = sum_c w[o,c] * x[n,y,x,c]."""
    return np.matmul(np.asarray(x, np.float64), np.asarray(w, np.float64).T)


def conv3x3(h: np.ndarray, w: np.ndarray) -> np.ndarray:
    """Stride-1, zero-pad-1 cross-correlation:
    out[n,y,x,o] = sum_{ky,kx,c} w[o,ky,kx,c] * hpad[n, y+ky, x+kx, c],
    where hpad is h with one ring of zeros (so tap (1,1) is the centre)."""
    h = np.asarray(h, np.float64)
    w = np.asarray(w, np.float64)
    n, hh, ww, c = h.shape
    hpad = np.zeros((n, hh + 2, ww + 2, c), np.float64)
    hpad[:, 1:hh + 1, 1:ww + 1, :] = h
    out = np.zeros((n, hh, ww, w.shape[0]), np.float64)
    for ky in range(3):
        for kx in range(3):
            out += np.matmul(hpad[:, ky:ky + hh, kx:kx + ww, :], w[:, ky, kx, :].T)
    return out


def affine(z: np.ndarray, s: np.ndarray, t: np.ndarray) -> np.ndarray:
    return z * np.asarray(s, np.float64) + np.asarray(t, np.float64)


def relu(z: np.ndarray) -> np.ndarray:
    return np.maximum(z, 0.0)


def bottleneck_branch(x: np.ndarray, p: BottleneckParams) -> np.ndarray:
    """Residual branch F(x) of the bottleneck on EVERY pixel (Fig. 2(a)):
    1x1 -> affine -> ReLU -> 3x3 -> affine -> ReLU -> 1x1 -> affine."""
    p = p.as_f64()
    h1 = relu(affine(conv1x1(x, p.w1), p.s1, p.t1))
    h2 = relu(affine(conv3x3(h1, p.w2), p.s2, p.t2))
    return affine(conv1x1(h2, p.w3), p.s3, p.t3)


def static_bottleneck(x: np.ndarray, p: BottleneckParams) -> np.ndarray:
    """out = act(x + F(x)) on every pixel; act = ReLU iff p.relu_out."""
    y = np.asarray(x, np.float64) + bottleneck_branch(x, p)
    return relu(y) if p.relu_out else y


# --------------------------------------------------------------------------- #
# spatial masker (Sec. 3.2 "Masker design"; App. B, operator fusion item 1)
# --------------------------------------------------------------------------- #
def pool_patches(x: np.ndarray, S: int) -> np.ndarray:
    """Adaptive average pool of x to [N, H/S, W/S, C]; S must divide H and W, so every
    output cell is the plain mean of one S x S patch."""
    x = np.asarray(x, np.float64)
    n, h, w, c = x.shape
    if h % S or w % S:
        raise ValueError("S must divide H and W")
    return x.reshape(n, h // S, S, w // S, S, c).mean(axis=(2, 4))


def masker_two_logits(x: np.ndarray, S: int, w2: np.ndarray, b2: np.ndarray) -> np.ndarray:
    """The masker as Sec. 3.2 states it: pool, then a 1x1 conv to TWO logits per patch.
    w2 [2, C], b2 [2] -> logits [N, H/S, W/S, 2]."""
    return np.matmul(pool_patches(x, S), np.asarray(w2, np.float64).T) + np.asarray(b2, np.float64)


def mask_from_two_logits(l2: np.ndarray) -> np.ndarray:
    """Inference decision: a patch is active iff logit channel 0 strictly exceeds channel 1
    (App. B: [x*W]_0 > [x*W]_1)."""
    return (l2[..., 0] > l2[..., 1]).astype(np.uint8)


def mask_logits(x: np.ndarray, S: int, w: np.ndarray, bias: float) -> np.ndarray:
    """One-channel masker of App. B: logit = bias + sum_c w[c] * mean_{SxS}(x[..., c]),
    with w = W_0 - W_1 (and bias = b_0 - b_1)."""
    return np.matmul(pool_patches(x, S), np.asarray(w, np.float64)) + float(bias)


def threshold(logits: np.ndarray) -> np.ndarray:
    """Active iff logit > 0, strictly; a logit of exactly 0 and a NaN are inactive."""
    return (np.asarray(logits) > 0).astype(np.uint8)


def upsample_mask(mask_coarse: np.ndarray, S: int) -> np.ndarray:
    """Each coarse element governs one S x S patch (Sec. 3.2): M_up[n,y,x] = M[n, y//S, x//S]."""
    return np.repeat(np.repeat(np.asarray(mask_coarse), S, axis=1), S, axis=2)


# --------------------------------------------------------------------------- #
# channel masker (Sec. 3.2 "Masker design"; Fig. 3(b))
# --------------------------------------------------------------------------- #
def channel_masker_hidden(D: int) -> int:
    """Hidden width of the channel masker's MLP: max(floor(D/16), 16)."""
    return max(D // 16, 16)


def channel_masker_logits(x: np.ndarray, wa: np.ndarray, ba: np.ndarray, wb: np.ndarray, bb: np.ndarray) -> np.ndarray:
    """Global average pooling over H x W, then a 2-layer MLP (ReLU between the layers; the paper does
    not name the non-linearity) producing 2D logits per sample, viewed as [N, D, 2] (row-major
    reshape of the 2D vector, as the paper reshapes the 2C vector to C x 2).
    wa [hidden, C], ba [hidden], wb [2D, hidden], bb [2D]."""
    g = np.asarray(x, np.float64).mean(axis=(1, 2))                       # [N, C]
    h = relu(np.matmul(g, np.asarray(wa, np.float64).T) + np.asarray(ba, np.float64))
    l2 = np.matmul(h, np.asarray(wb, np.float64).T) + np.asarray(bb, np.float64)  # [N, 2D]
    return l2.reshape(l2.shape[0], -1, 2)


def channel_mask_from_logits(l2: np.ndarray) -> np.ndarray:
    """Group d of a sample is kept iff its logit 0 strictly exceeds its logit 1 (argmax at inference,
    ties and NaN drop the group, as for the spatial masker)."""
    return (l2[..., 0] > l2[..., 1]).astype(np.uint8)


# --------------------------------------------------------------------------- #
# index generation / gather (App. B, operator fusion item 2; Sec. 3.1 step 1)
# --------------------------------------------------------------------------- #
def compact(mask: np.ndarray) -> np.ndarray:
    """Indices of the non-zero entries of the flattened mask, ascending (int32).
    For a coarse mask [N,Hp,Wp] the flat index is (n*Hp + py)*Wp + px."""
    flat = np.asarray(mask).reshape(-1)
    return np.array([i for i in range(flat.size) if flat[i] != 0], dtype=np.int32)


def sample_offsets(mask_coarse: np.ndarray) -> np.ndarray:
    """offsets[n] = number of active patches in samples 0..n-1 ([N+1] int32): the
    patch <-> sample correspondence that batching needs (Sec. 3.4, batching inference)."""
    per = np.asarray(mask_coarse).reshape(mask_coarse.shape[0], -1).astype(bool).sum(axis=1)
    return np.concatenate([[0], np.cumsum(per)]).astype(np.int32)


def gather_patches(x: np.ndarray, S: int, halo: int, idx: np.ndarray) -> np.ndarray:
    """g[p, dy, dx, :] = x[n, py*S - halo + dy, px*S - halo + dx, :] when that pixel lies
    inside the image, else 0; (n, py, px) decoded from idx[p].  halo = 1 gives the
    neighbours a 3x3 kernel needs (Sec. 3.1 step 1).  Same dtype as x (a pure copy)."""
    x = np.asarray(x)
    n, h, w, c = x.shape
    hp, wp = h // S, w // S
    e = S + 2 * halo
    g = np.zeros((len(idx), e, e, c), x.dtype)
    for p, q in enumerate(np.asarray(idx).tolist()):
        b, r = divmod(q, hp * wp)
        py, px = divmod(r, wp)
        for dy in range(e):
            for dx in range(e):
                yy, xx = py * S - halo + dy, px * S - halo + dx
                if 0 <= yy < h and 0 <= xx < w:
                    g[p, dy, dx, :] = x[b, yy, xx, :]
    return g


# --------------------------------------------------------------------------- #
# the three dynamic paradigms (Sec. 3.1, Sec. 3.2, Fig. 2)
# --------------------------------------------------------------------------- #
def dyn_bottleneck(x: np.ndarray, p: BottleneckParams, S: int, mask_coarse: np.ndarray) -> np.ndarray:
    """Spatially adaptive block.  The spatial mask is applied on the block's final
    output and unselected positions keep the skip-connection value (Fig. 2 caption;
    Sec. 3.1): compute the branch everywhere, then
        out = M_up ? act(x + F(x)) : x."""
    x64 = np.asarray(x, np.float64)
    full = static_bottleneck(x64, p)
    m_up = upsample_mask(mask_coarse, S).astype(bool)[..., None]
    return np.where(m_up, full, x64)


def channel_skip_bottleneck(x: np.ndarray, p: BottleneckParams, cmask: np.ndarray) -> np.ndarray:
    """Channel skipping (Fig. 2 caption; Sec. 3.2): the per-sample channel mask, one
    decision per group of G = m/D consecutive channels, multiplies the input AND the
    output of the 3x3 conv, i.e. the outputs of the first two (conv, affine, ReLU)
    layers.  No spatial mask: out = act(x + F_c(x)) on every pixel."""
    p = p.as_f64()
    x64 = np.asarray(x, np.float64)
    cmask = np.asarray(cmask)
    m = p.w1.shape[0]
    d = cmask.shape[1]
    if m % d:
        raise ValueError("D must divide the mid width")
    mc = np.repeat(cmask.astype(np.float64), m // d, axis=1)[:, None, None, :]  # [N,1,1,m]
    h1 = relu(affine(conv1x1(x64, p.w1), p.s1, p.t1)) * mc
    h2 = relu(affine(conv3x3(h1, p.w2), p.s2, p.t2)) * mc
    y = x64 + affine(conv1x1(h2, p.w3), p.s3, p.t3)
    return relu(y) if p.relu_out else y


def layer_skip_bottleneck(x: np.ndarray, p: BottleneckParams, keep: np.ndarray,
                          S: int | None = None, mask_coarse: np.ndarray | None = None) -> np.ndarray:
    """Layer skipping (Sec. 3.1): a scalar gate per sample; gate 1 executes the whole
    block, gate 0 leaves the sample untouched.  With a spatial mask as well, the two
    decisions are AND-ed (a skipped sample has no active patch)."""
    x64 = np.asarray(x, np.float64)
    keep = np.asarray(keep).astype(bool)
    if mask_coarse is None:
        full = static_bottleneck(x64, p)
    else:
        full = dyn_bottleneck(x64, p, S, mask_coarse)
    return np.where(keep[:, None, None, None], full, x64)


# --------------------------------------------------------------------------- #
# group convolution + squeeze-and-excitation blocks (Sec. 4: the RegNetY backbones; Sec. 3.2: the
# design is meant to carry over to arbitrary bottleneck ratios and group convolutions)
# --------------------------------------------------------------------------- #
@dataclass
class GroupSE:
    """What a RegNetY-style bottleneck adds to BottleneckParams: the 3x3 is a group convolution
    with g channels per group (w2 is then [m, 3, 3, g]: output channel o reads the input channels
    (o // g) * g ... (o // g) * g + g - 1), and a squeeze-and-excitation module sits between the 3x3
    (after its affine and ReLU) and the last 1x1.  se_width 0 (w_se1 None) means no SE module."""
    g: int
    w_se1: np.ndarray | None = None  # [se_width, m]
    b_se1: np.ndarray | None = None  # [se_width]
    w_se2: np.ndarray | None = None  # [m, se_width]
    b_se2: np.ndarray | None = None  # [m]


def group_conv3x3(h: np.ndarray, w: np.ndarray, g: int) -> np.ndarray:
    """Stride-1, zero-pad-1 group cross-correlation with g channels per group (as many in as out):
    out[n,y,x,o] = sum_{ky,kx,c<g} w[o,ky,kx,c] * hpad[n, y+ky, x+kx, (o//g)*g + c]."""
    h = np.asarray(h, np.float64)
    w = np.asarray(w, np.float64)
    m = w.shape[0]
    if m % g or h.shape[-1] != m or w.shape[-1] != g:
        raise ValueError("group width must divide the channel count")
    out = np.zeros(h.shape[:3] + (m,), np.float64)
    for k in range(m // g):
        out[..., k * g:(k + 1) * g] = conv3x3(h[..., k * g:(k + 1) * g], w[k * g:(k + 1) * g])
    return out


def se_scale(h2: np.ndarray, m_up: np.ndarray, e: GroupSE) -> np.ndarray:
    """Squeeze-and-excitation gate per sample and channel, [N, m].  The paper does not say what the
    squeeze averages over when only some locations are computed; the reading taken here: the mean over
    the sample's COMPUTED (active) pixels, the only ones whose h2 exists in a sparse evaluation.  With
    every pixel active this is the ordinary global average.  z = mean, gate = sigmoid(W2 relu(W1 z + b1)
    + b2).  A sample without an active pixel gets gate 1 (its branch is never added)."""
    h2 = np.asarray(h2, np.float64)
    n, _, _, m = h2.shape
    gate = np.ones((n, m), np.float64)
    for b in range(n):
        act = np.asarray(m_up[b]).astype(bool)
        cnt = int(act.sum())
        if cnt == 0:
            continue
        z = h2[b][act].sum(axis=0) / cnt
        hid = relu(np.matmul(np.asarray(e.w_se1, np.float64), z) + np.asarray(e.b_se1, np.float64))
        a = np.matmul(np.asarray(e.w_se2, np.float64), hid) + np.asarray(e.b_se2, np.float64)
        gate[b] = 1.0 / (1.0 + np.exp(-a))
    return gate


def dyn_group_se_bottleneck(x: np.ndarray, p: BottleneckParams, e: GroupSE, S: int,
                            mask_coarse: np.ndarray) -> np.ndarray:
    """Spatially adaptive bottleneck whose 3x3 is a group convolution and which may carry an SE module
    (the block of the RegNetY backbones, Sec. 4).  Dense-then-mask like dyn_bottleneck:
        h1 = relu(affine(1x1(x))), h2 = relu(affine(group3x3(h1))) on every pixel,
        gate = se_scale(h2, M_up) per sample,  f = affine(1x1(h2 * gate)),
        out = M_up ? act(x + f) : x."""
    q = p.as_f64()
    x64 = np.asarray(x, np.float64)
    m_up = upsample_mask(mask_coarse, S).astype(bool)
    h1 = relu(affine(conv1x1(x64, q.w1), q.s1, q.t1))
    h2 = relu(affine(group_conv3x3(h1, q.w2, e.g), q.s2, q.t2))
    if e.w_se1 is not None:
        h2 = h2 * se_scale(h2, m_up, e)[:, None, None, :]
    y = x64 + affine(conv1x1(h2, q.w3), q.s3, q.t3)
    if q.relu_out:
        y = relu(y)
    return np.where(m_up[..., None], y, x64)


# --------------------------------------------------------------------------- #
# complexity accounting (Sec. 3.2 "Computational complexity")
# --------------------------------------------------------------------------- #
def conv_macs_per_pixel(c_in: int, m: int, c_out: int) -> tuple[int, int, int]:
    """Multiply-accumulates per output pixel of the three convs: F1, F2, F3."""
    return c_in * m, 9 * m * m, m * c_out


def activation_ratio(mask_coarse: np.ndarray) -> float:
    """r^s = sum(M) / (H*W); identical on the coarse grid since every element stands
    for S*S pixels."""
    mk = np.asarray(mask_coarse).astype(bool)
    return float(mk.sum()) / float(mk.size)


def dilated_ratio(mask_coarse: np.ndarray, S: int) -> float:
    """r^s_dil: fraction of pixels of the 3x3-dilated full-resolution mask, i.e. the
    pixels whose conv1 output some active pixel's 3x3 window touches."""
    up = upsample_mask(mask_coarse, S).astype(bool)
    n, h, w = up.shape
    pad = np.zeros((n, h + 2, w + 2), bool)
    pad[:, 1:-1, 1:-1] = up
    dil = np.zeros_like(up)
    for dy in range(3):
        for dx in range(3):
            dil |= pad[:, dy:dy + h, dx:dx + w]
    return float(dil.sum()) / float(dil.size)


def spatial_flops_ratio(r: float, r_dil: float, c_in: int, m: int, c_out: int) -> float:
    """(r_dil*F1 + r*F2 + r*F3) / (F1 + F2 + F3)."""
    f1, f2, f3 = conv_macs_per_pixel(c_in, m, c_out)
    return (r_dil * f1 + r * f2 + r * f3) / (f1 + f2 + f3)


def channel_flops_ratio(rc: float, c_in: int, m: int, c_out: int) -> float:
    """(r*F1 + r^2*F2 + r*F3) / (F1 + F2 + F3)."""
    f1, f2, f3 = conv_macs_per_pixel(c_in, m, c_out)
    return (rc * f1 + rc * rc * f2 + rc * f3) / (f1 + f2 + f3)


# --------------------------------------------------------------------------- #
# static parts of the ResNet body (the whole-body workload): stem and projection blocks
# --------------------------------------------------------------------------- #
def conv2d(x: np.ndarray, w: np.ndarray, stride: int, pad: int) -> np.ndarray:
    """General cross-correlation, NHWC: out[n,yo,xo,o] = sum_{ky,kx,c} w[o,ky,kx,c] *
    xpad[n, yo*stride + ky, xo*stride + kx, c], xpad = x with `pad` rings of zeros;
    output size floor((H + 2*pad - k)/stride) + 1."""
    x = np.asarray(x, np.float64)
    w = np.asarray(w, np.float64)
    n, h, wd, c = x.shape
    co, kh, kw, _ = w.shape
    ho = (h + 2 * pad - kh) // stride + 1
    wo = (wd + 2 * pad - kw) // stride + 1
    xp = np.zeros((n, h + 2 * pad, wd + 2 * pad, c), np.float64)
    xp[:, pad:pad + h, pad:pad + wd, :] = x
    out = np.zeros((n, ho, wo, co), np.float64)
    for ky in range(kh):
        for kx in range(kw):
            win = xp[:, ky:ky + (ho - 1) * stride + 1:stride, kx:kx + (wo - 1) * stride + 1:stride, :]
            out += np.matmul(win, w[:, ky, kx, :].T)
    return out


def maxpool3x3_s2(x: np.ndarray) -> np.ndarray:
    """3x3 max pooling, stride 2, padding 1 (padding never wins: -inf)."""
    x = np.asarray(x, np.float64)
    n, h, wd, c = x.shape
    ho, wo = (h + 2 - 3) // 2 + 1, (wd + 2 - 3) // 2 + 1
    xp = np.full((n, h + 2, wd + 2, c), -np.inf)
    xp[:, 1:h + 1, 1:wd + 1, :] = x
    out = np.full((n, ho, wo, c), -np.inf)
    for ky in range(3):
        for kx in range(3):
            out = np.maximum(out, xp[:, ky:ky + (ho - 1) * 2 + 1:2, kx:kx + (wo - 1) * 2 + 1:2, :])
    return out


def stem(x: np.ndarray, w7: np.ndarray, s: np.ndarray, t: np.ndarray) -> np.ndarray:
    """ResNet stem: 7x7 stride-2 pad-3 conv, affine (folded BN), ReLU, 3x3 stride-2 max pool."""
    return maxpool3x3_s2(relu(affine(conv2d(x, w7, 2, 3), s, t)))


def projection_bottleneck(x: np.ndarray, p: BottleneckParams, w_sc: np.ndarray, s_sc: np.ndarray,
                          t_sc: np.ndarray, stride: int) -> np.ndarray:
    """First block of a stage (always executed, no mask): the stride sits on the 3x3 (as in the
    torchvision models the paper initialises from) and the shortcut is a strided 1x1 conv with its
    own affine; out = relu(branch + shortcut)."""
    p = p.as_f64()
    h1 = relu(affine(conv1x1(x, p.w1), p.s1, p.t1))
    h2 = relu(affine(conv2d(h1, p.w2, stride, 1), p.s2, p.t2))
    f = affine(conv1x1(h2, p.w3), p.s3, p.t3)
    sc = affine(conv2d(x, np.asarray(w_sc, np.float64)[:, None, None, :], stride, 0), s_sc, t_sc)
    return relu(f + sc)


def dyn_projection_bottleneck(x: np.ndarray, p: BottleneckParams, w_sc: np.ndarray, s_sc: np.ndarray,
                              t_sc: np.ndarray, stride: int, S: int, mask_coarse: np.ndarray) -> np.ndarray:
    """Dynamic first block of a stage: the spatial mask lives on the OUTPUT grid (the mask decides at which
    output locations the convolutions run, Sec. 3.1), in patches of S x S output pixels; locations that are
    not selected take the value of the skip connection (Sec. 3.1), which in this block is the strided
    1x1 projection with its own affine:  out = act(shortcut(x) + M * branch(x)).  Dense-then-mask."""
    q = p.as_f64()
    h1 = relu(affine(conv1x1(x, q.w1), q.s1, q.t1))
    h2 = relu(affine(conv2d(h1, q.w2, stride, 1), q.s2, q.t2))
    f = affine(conv1x1(h2, q.w3), q.s3, q.t3)
    sc = affine(conv2d(x, np.asarray(w_sc, np.float64)[:, None, None, :], stride, 0), s_sc, t_sc)
    up = upsample_mask(mask_coarse, S).astype(np.float64)[..., None]
    out = sc + up * f
    return relu(out) if q.relu_out else out


def strided_mask_logits(x: np.ndarray, stride: int, S: int, w: np.ndarray, bias: float) -> np.ndarray:
    """Masker of a strided block (Sec. 3.2 "Masker design"): the input is pooled adaptively to the
    patch grid of the OUTPUT (Ho/S x Wo/S); with H = stride*Ho that is a mean over windows of
    stride*S input pixels, followed by the one-channel 1x1 conv."""
    return mask_logits(x, stride * S, w, bias)


def group_conv2d(h: np.ndarray, w: np.ndarray, g: int, stride: int) -> np.ndarray:
    """3x3 group cross-correlation with zero padding 1 and a spatial stride, g channels per group:
    out[n,yo,xo,o] = sum_{ky,kx,c<g} w[o,ky,kx,c] * hpad[n, yo*stride + ky, xo*stride + kx, (o//g)*g + c]."""
    h = np.asarray(h, np.float64)
    w = np.asarray(w, np.float64)
    m = w.shape[0]
    if m % g or h.shape[-1] != m or w.shape[-1] != g:
        raise ValueError("group width must divide the channel count")
    return np.concatenate([conv2d(h[..., k * g:(k + 1) * g], w[k * g:(k + 1) * g], stride, 1) for k in range(m // g)],
                          axis=-1)


def dyn_group_se_projection_bottleneck(x: np.ndarray, p: BottleneckParams, e: GroupSE, w_sc: np.ndarray,
                                       s_sc: np.ndarray, t_sc: np.ndarray, stride: int, S: int,
                                       mask_coarse: np.ndarray) -> np.ndarray:
    """First block of a stage of the group-convolution / SE backbones (Sec. 4): as dyn_projection_bottleneck
    (mask on the output grid, unselected locations keep the strided projection shortcut), with the stride on
    the group 3x3 and the SE gate of se_scale taken over the sample's active OUTPUT pixels:
        out = act(shortcut(x) + M_up * affine(1x1(h2 * gate))),  h2 = relu(affine(group3x3_stride(h1))).
    With every location active this is the static first block."""
    q = p.as_f64()
    h1 = relu(affine(conv1x1(x, q.w1), q.s1, q.t1))
    h2 = relu(affine(group_conv2d(h1, q.w2, e.g, stride), q.s2, q.t2))
    m_up = upsample_mask(mask_coarse, S).astype(bool)
    if e.w_se1 is not None:
        h2 = h2 * se_scale(h2, m_up, e)[:, None, None, :]
    f = affine(conv1x1(h2, q.w3), q.s3, q.t3)
    sc = affine(conv2d(x, np.asarray(w_sc, np.float64)[:, None, None, :], stride, 0), s_sc, t_sc)
    out = sc + m_up[..., None].astype(np.float64) * f
    return relu(out) if q.relu_out else out


def stem3x3(x: np.ndarray, w3: np.ndarray, s: np.ndarray, t: np.ndarray) -> np.ndarray:
    """Stem of the RegNet backbones (Sec. 4): 3x3 stride-2 pad-1 conv from the image, affine (folded BN), ReLU;
    no pooling.  x [N,H,W,3], w3 [c_out,3,3,3] -> [N, (H-1)//2+1, (W-1)//2+1, c_out]."""
    return relu(affine(conv2d(x, w3, 2, 1), s, t))
