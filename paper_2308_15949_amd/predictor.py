"""Latency predictor for the dynamic bottleneck, re-parameterised for MI355X (Sec. 3.3 "Latency
predictor", App. A "Latency prediction model").

The paper models a device as processing engines (PEs) with three memory levels and predicts a block's
latency as data movement + computation + a constant: an operator's output is cut into tiles, tiles are
dealt to the PEs, a PE moves the inputs of each of its tiles once from on-chip global memory to its
local memory (bandwidth x efficiency), the off-chip traffic runs at the full off-chip bandwidth, and
the computation time follows from the FLOPs of a tile and the PE's peak throughput; the tile shape
is searched over a candidate set.

Here the PE is a compute unit (256 of them), its local memory the LDS, the on-chip global memory the
L2 / Infinity Cache, peak throughput the MFMA rate of the arithmetic type, and the tile candidates
are the ones the library's kernels are built for.  Host arithmetic only; nothing here touches the GPU.
The three free constants (local-memory efficiency, per-kernel and per-tile constants) were set once from
measured latencies of the LDS-staged kernels (the granularity curves of the four stages at ratio 0.5, batch 128,
bf16); every other number is a datasheet figure or follows from shapes.  The 256-wide bf16 blocks run on
register-weight kernels (128 x 256 tiles for the first 1x1; 3x3 and last 1x1 as one kernel whose tile moves both
weight tensors once): they are modelled with their own tile shapes and the nominal local-memory rate, which is
what their contiguous requests were measured to reach.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field


@dataclass(frozen=True)
class Hardware:
    """Hardware properties H of the model (App. A, table of hardware properties, extended by the
    local-memory path that the text describes)."""
    name: str
    n_pe: int                    # processing engines
    clock_hz: float
    flop_per_clk_pe: dict        # peak FLOP per clock per PE by arithmetic type ("bf16", "f32")
    offchip_Bps: float           # off-chip memory bandwidth
    local_B_per_clk: float       # on-chip global -> local memory, bytes per clock per PE (nominal)
    local_efficiency: float      # fraction of it a gathered, tiled access stream reaches
    offchip_efficiency: float    # fraction of the off-chip bandwidth a short streaming kernel reaches
    const_s: float               # per-kernel constant (launch + first/last dependent memory round trips)
    tile_const_s: float = 0.0    # per tile a PE works through: the part of a tile's prologue / epilogue nothing hides
    stream_efficiency: float = 1.0  # the same fraction for kernels that read pre-ordered weights straight into registers
                                    # and rows straight into local memory (contiguous 1 KB requests: the nominal rate)
    tiles: tuple = field(default=((64, 64), (64, 128), (128, 128)))

    def local_Bps(self, streamed: bool = False) -> float:
        return self.local_B_per_clk * self.clock_hz * (self.stream_efficiency if streamed else self.local_efficiency)

    def pe_flops(self, dtype: str) -> float:
        return self.flop_per_clk_pe[dtype] * self.clock_hz


# 256 CUs at 2.4 GHz; dense MFMA 2.5 PFLOP/s bf16 and 157.3 TFLOP/s fp32 over the chip; HBM3E 8 TB/s;
# 64 B/clk nominal L2 -> CU path.  local_efficiency, const_s and tile_const_s are the fitted constants.
MI355X = Hardware("MI355X", 256, 2.4e9, {"bf16": 4096.0, "f32": 256.0}, 8.0e12, 64.0, 0.65, 0.40, 4.0e-6, 0.75e-6)


def paper_device(name: str, n_pe: int, n_fp32: int, mhz: float, gbps: float) -> Hardware:
    """A device given the way the paper's hardware table gives it: #PE, FP32 units per PE,
    frequency and off-chip bandwidth (one FMA = 2 FLOP per unit per clock)."""
    return Hardware(name, n_pe, mhz * 1e6, {"f32": 2.0 * n_fp32, "bf16": 2.0 * n_fp32}, gbps * 1e9, 128.0, 0.5, 0.8,
                    5.0e-6)


@dataclass
class KernelPrediction:
    name: str
    tile: tuple
    tiles: int
    tiles_per_pe: int
    flops: float
    offchip_bytes: float
    l_off2on: float
    l_global2local: float
    l_computation: float
    l_const: float

    @property
    def total(self) -> float:
        return self.l_off2on + self.l_global2local + self.l_computation + self.l_const


def _gemm(hw: Hardware, name: str, rows: int, cols: int, k: int, taps: int, eb: int, dtype: str,
          a_offchip_bytes: float, residual: bool, tile=None, streamed: bool = False) -> KernelPrediction:
    """One tiled implicit GEMM [rows x (taps*k)] x [(taps*k) x cols] (App. A: shape definition, mapping
    of output tiles to PEs, latency estimation).  a_offchip_bytes: distinct activation bytes that come
    from off-chip memory; weights and outputs are added here."""
    best = None
    for bm, bn in ([tile] if tile else hw.tiles):
        n_tiles = math.ceil(rows / bm) * math.ceil(cols / bn) if rows > 0 else 0
        per_pe = math.ceil(n_tiles / hw.n_pe)
        # a PE moves the inputs of a tile once: activation and weight slices of the whole reduction,
        # the residual chunk it adds, and the tile it writes back
        tile_bytes = taps * k * (bm + bn) * eb + bm * bn * eb * (2 if residual else 1)
        tile_flops = 2.0 * bm * bn * k * taps
        off = a_offchip_bytes + taps * k * cols * eb + rows * cols * eb * (2 if residual else 1)
        kp = KernelPrediction(name, (bm, bn), n_tiles, per_pe, 2.0 * rows * cols * k * taps, off,
                              off / hw.offchip_Bps if rows > 0 else 0.0,
                              per_pe * tile_bytes / hw.local_Bps(streamed),
                              per_pe * tile_flops / hw.pe_flops(dtype),
                              hw.const_s + per_pe * hw.tile_const_s)
        if best is None or kp.total < best.total:
            best = kp
    return best


def _fused_tail(hw: Hardware, rows: int, m: int, c_out: int, eb: int, dtype: str, a_offchip_bytes: float) -> KernelPrediction:
    """3x3 -> last 1x1 -> residual add as ONE kernel (what the library runs for 256-wide bf16 blocks): a tile is bm
    pixels x all channels of both convolutions, h2 stays in local memory, and a PE moves both weight tensors once
    per tile whatever its height; the tile height is searched over the kernel's candidates (App. A: tile shape
    search), as the kernel itself does on the device."""
    w_bytes = (9 * m * m + m * c_out) * eb
    flops = 2.0 * rows * (9 * m * m + m * c_out)
    off = a_offchip_bytes + w_bytes + 2.0 * rows * c_out * eb
    best = None
    for bm in (32, 64, 96):
        n_tiles = math.ceil(rows / bm) if rows > 0 else 0
        per_pe = math.ceil(n_tiles / hw.n_pe)
        tile_bytes = w_bytes + bm * 9 * m * eb + 2 * bm * c_out * eb
        tile_flops = 2.0 * bm * (9 * m * m + m * c_out)
        kp = KernelPrediction("conv2 + conv3 + scatter-add (one kernel)", (bm, c_out), n_tiles, per_pe, flops, off,
                              off / hw.offchip_Bps if rows > 0 else 0.0, per_pe * tile_bytes / hw.local_Bps(True),
                              per_pe * tile_flops / hw.pe_flops(dtype), hw.const_s + per_pe * hw.tile_const_s)
        if best is None or kp.total < best.total:
            best = kp
    return best


def fused_shapes(c_in: int, m: int, dtype: str, group_width, se_width: int) -> bool:
    """Blocks the library runs on its register-weight kernels (first 1x1 with 128 x 256 tiles; 3x3 and last 1x1 fused)."""
    return dtype == "bf16" and m == 256 and c_in == 1024 and group_width is None and se_width == 0


def _stream(hw: Hardware, name: str, nbytes: float) -> KernelPrediction:
    """A kernel that only streams off-chip data (masker, pooling, compaction)."""
    return KernelPrediction(name, (0, 0), 0, 0, 0.0, nbytes, nbytes / (hw.offchip_Bps * hw.offchip_efficiency), 0.0, 0.0,
                            hw.const_s)


def expected_dilated_ratio(r: float, S: int) -> float:
    """Expected fraction of pixels inside the one-pixel dilation of the active patches (the set
    conv1 covers, Sec. 3.2) for independent Bernoulli(r) patches, image borders ignored: a pixel in
    the interior of its patch depends on 1 patch, on an edge on 2, in a corner on 4 (S = 1: on 9)."""
    q = 1.0 - r
    if S == 1:
        return 1.0 - q ** 9
    corner, edge, inner = 4, 4 * (S - 2), (S - 2) ** 2
    return (corner * (1 - q ** 4) + edge * (1 - q ** 2) + inner * (1 - q)) / (S * S)


def predict_block(hw: Hardware, paradigm: str, *, n: int, hw_px: int, c_in: int, m: int, dtype: str = "bf16",
                  S: int = 1, r: float = 1.0, r_dil: float | None = None, fused_masker: bool = True,
                  with_masker: bool = True, group_width: int | None = None, se_width: int = 0) -> dict:
    """Latency of one identity bottleneck (c_in -> m -> m -> c_in) on a batch of n feature maps of
    hw_px x hw_px pixels: l = G(H, P, D, S, r) of Sec. 3.3.

    paradigm "spatial": activation ratio r over S x S patches (r_dil: ratio of the dilated set, default
    the Bernoulli expectation); "channel": r is the kept fraction of the m mid channels; "layer": r is
    the kept fraction of samples (S = feature size); "static": the plain block.
    group_width g turns the 3x3 into a group convolution (spatial / layer / static paradigms): FLOPs count the g
    input channels a kernel really reads; the time is that of the 64-channel window the kernel multiplies.
    se_width adds the SE module between the 3x3 and the last 1x1: four small kernels that stream the active
    rows (read for the mean, read and written for the gate) and the two fully connected layers.
    Returns {"kernels": [KernelPrediction...], "total_s": ..., "flops": ...}."""
    eb = 2 if dtype == "bf16" else 4
    npix = n * hw_px * hw_px
    ks = []
    if paradigm == "static":
        paradigm, r, with_masker = "spatial", 1.0, False
    if paradigm == "layer":
        S, r_dil, paradigm = hw_px, r, "spatial"
        fused_masker = False
        with_masker = False
    if paradigm == "spatial":
        if r_dil is None:
            r_dil = expected_dilated_ratio(r, S)
        fused = fused_shapes(c_in, m, dtype, group_width, se_width)
        tile1 = (128, 256) if fused else None
        if with_masker and fused_masker:
            rows1, a_off = npix, float(npix * c_in * eb)
            ks.append(_gemm(hw, "conv1 (every pixel) + masker projection", rows1, m, c_in, 1, eb, dtype, a_off, False, tile=tile1, streamed=fused))
            ks.append(_stream(hw, "pool + threshold + index list", npix * 4.0))
        else:
            if with_masker:
                ks.append(_stream(hw, "masker", float(npix * c_in * eb)))
                ks.append(_stream(hw, "index list", float(npix // (S * S))))
            rows1 = int(round(r_dil * npix))
            ks.append(_gemm(hw, "conv1 (dilated active set)", rows1, m, c_in, 1, eb, dtype, float(rows1 * c_in * eb), False, tile=tile1, streamed=fused))
        rows = int(round(r * npix))
        if fused:
            ks.append(_fused_tail(hw, rows, m, c_in, eb, dtype, float(min(r_dil, 1.0) * npix * m * eb)))
            return {"kernels": ks, "total_s": sum(k.total for k in ks), "flops": sum(k.flops for k in ks)}
        if group_width is None:
            ks.append(_gemm(hw, "conv2 (active patches)", rows, m, m, 9, eb, dtype, float(min(r_dil, 1.0) * npix * m * eb), False))
        else:
            # one 64-channel output tile reduces over its own 64 input channels: the executed reduction length
            kwin = min(64, m)
            k2 = _gemm(hw, "group conv2 (active patches)", rows, m, kwin, 9, eb, dtype, float(min(r_dil, 1.0) * npix * m * eb),
                       False, tile=(64, 64))
            k2.flops = 2.0 * rows * m * group_width * 9
            ks.append(k2)
        if se_width > 0:
            ks.append(_stream(hw, "SE squeeze", float(rows * m * eb)))
            fc = KernelPrediction("SE fc1", (0, 0), 0, 0, 2.0 * n * m * se_width, 4.0 * m * se_width, 0.0, 0.0, 0.0, hw.const_s)
            ks.append(fc)
            ks.append(KernelPrediction("SE fc2", (0, 0), 0, 0, 2.0 * n * m * se_width, 4.0 * m * se_width, 0.0, 0.0, 0.0, hw.const_s))
            ks.append(_stream(hw, "SE gate", float(2 * rows * m * eb)))
        ks.append(_gemm(hw, "conv3 + scatter-add", rows, c_in, m, 1, eb, dtype, float(rows * m * eb), True))
    elif paradigm == "channel":
        mk = max(int(round(r * m)), 0)
        ks.append(_gemm(hw, "conv1 (kept kernels)", npix, mk, c_in, 1, eb, dtype, float(npix * c_in * eb), False))
        ks.append(_gemm(hw, "conv2 (kept in/out)", npix, mk, mk, 9, eb, dtype, float(npix * mk * eb), False))
        ks.append(_gemm(hw, "conv3 (kept inputs) + add", npix, c_in, mk, 1, eb, dtype, float(npix * mk * eb), True))
    else:
        raise ValueError(paradigm)
    return {"kernels": ks, "total_s": sum(k.total for k in ks), "flops": sum(k.flops for k in ks)}
