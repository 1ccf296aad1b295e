// Channel masker (Sec. 3.2 "Masker design", Fig. 3(b)): global average pooling over H x W, a 2-layer
// MLP with hidden width max(floor(D/16), 16), 2D logits viewed as [D][2], argmax at inference.
//
//   k_gap_partial   HBM-bound: every block sums one slab of a sample's pixels for all C channels
//                   (16-byte loads, float32 sums) and writes one partial row; no atomics, so the
//                   result does not depend on scheduling.
//   k_channel_mlp   one block per sample: adds the partial rows in slab order, divides by H*W, runs
//                   the two small layers (float32) and writes the D keep/drop decisions.
#include "laud_common.h"

namespace laud {

constexpr int kGapThreads = 256;

template <typename ET>
__global__ __launch_bounds__(kGapThreads) void k_gap_partial(const ET* __restrict__ x, int HW, int C, int slabs,
                                                             float* __restrict__ partial) {
  constexpr int EPC = elem<ET>::per16;
  __shared__ float red[kGapThreads * 8];
  const int n = blockIdx.x / slabs, slab = blockIdx.x % slabs;
  const int cpr = C / EPC;  // 16-byte chunks per pixel
  const int p0 = (int)((long long)HW * slab / slabs), p1 = (int)((long long)HW * (slab + 1) / slabs);
  // The block covers `cw` chunk columns at a time with `lanes` pixels in flight per column:
  // consecutive threads read consecutive chunks of one pixel (coalesced).
  const int cw = cpr < kGapThreads ? cpr : kGapThreads;
  const int lanes = kGapThreads / cw;
  const int cvi = threadIdx.x % cw, pl = threadIdx.x / cw;
  for (int cv0 = 0; cv0 < cpr; cv0 += cw) {
    const int cv = cv0 + cvi;
    const bool active = cv < cpr && pl < lanes;
    float acc[EPC];
#pragma unroll
    for (int e = 0; e < EPC; ++e) acc[e] = 0.f;
    if (active) {
      const ET* col = x + (size_t)n * HW * C + (size_t)cv * EPC;
      int p = p0 + pl;
      // four pixels' chunks in flight per thread before any is added (same order of additions as one by one)
      for (; p + 3 * lanes < p1; p += 4 * lanes) {
        uint4 raw[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) raw[u] = *reinterpret_cast<const uint4*>(col + (size_t)(p + u * lanes) * C);
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          ET v[EPC];
          __builtin_memcpy(v, &raw[u], 16);
#pragma unroll
          for (int e = 0; e < EPC; ++e) acc[e] += elem<ET>::load(&v[e]);
        }
      }
      for (; p < p1; p += lanes) {
        const uint4 raw = *reinterpret_cast<const uint4*>(col + (size_t)p * C);
        ET v[EPC];
        __builtin_memcpy(v, &raw, 16);
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[e] += elem<ET>::load(&v[e]);
      }
    }
#pragma unroll
    for (int e = 0; e < EPC; ++e) red[threadIdx.x * EPC + e] = acc[e];
    __syncthreads();
    if (active && pl == 0) {  // the pixel lanes of a chunk column are added in lane order
      float* out = partial + ((size_t)n * slabs + slab) * C + (size_t)cv * EPC;
#pragma unroll
      for (int e = 0; e < EPC; ++e) {
        float s = 0.f;
        for (int l = 0; l < lanes; ++l) s += red[(l * cw + cvi) * EPC + e];
        out[e] = s;
      }
    }
    __syncthreads();
  }
}

constexpr int kMlpThreads = 1024;  // 16 waves: one hidden unit per wave in a single round for the usual 16 units
__global__ __launch_bounds__(kMlpThreads) void k_channel_mlp(const float* __restrict__ partial, int slabs, int HW, int C,
                                                     const float* __restrict__ wa, const float* __restrict__ ba,
                                                     int hidden, const float* __restrict__ wb,
                                                     const float* __restrict__ bb, int D,
                                                     uint8_t* __restrict__ cmask, float* __restrict__ logits2) {
  extern __shared__ __align__(16) float sm[];  // g[C], h[hidden], l[2D]
  float* g = sm;
  float* h = g + C;
  float* l = h + hidden;
  const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float inv = 1.0f / (float)HW;
  for (int c = tid; c < C; c += kMlpThreads) {
    float s = 0.f;
    const float* pc = partial + (size_t)n * slabs * C + c;
    int k = 0;
    for (; k + 8 <= slabs; k += 8) {  // eight partial rows requested together, added in slab order
      float v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = pc[(size_t)(k + u) * C];
#pragma unroll
      for (int u = 0; u < 8; ++u) s += v[u];
    }
    for (; k < slabs; ++k) s += pc[(size_t)k * C];
    g[c] = s * inv;
  }
  __syncthreads();
  for (int j = wave; j < hidden; j += kMlpThreads / kWave) {  // one wave per hidden unit
    // the weight row is read in 16-byte pieces, four of them requested before any is used: the row comes
    // from L2 and a dependent load per element would cost a round trip each
    const float4* wr = reinterpret_cast<const float4*>(wa + (size_t)j * C);
    const float4* gv = reinterpret_cast<const float4*>(g);
    const int nv = C / 4;
    float acc = 0.f;
    int c = lane;
    for (; c + 3 * kWave < nv; c += 4 * kWave) {
      float4 w4[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) w4[u] = wr[c + u * kWave];
#pragma unroll
      for (int u = 0; u < 4; ++u) {
        const float4 g4 = gv[c + u * kWave];
        acc += w4[u].x * g4.x + w4[u].y * g4.y + w4[u].z * g4.z + w4[u].w * g4.w;
      }
    }
    for (; c < nv; c += kWave) {
      const float4 w4 = wr[c], g4 = gv[c];
      acc += w4.x * g4.x + w4.y * g4.y + w4.z * g4.z + w4.w * g4.w;
    }
    acc = wave_sum(acc);
    if (lane == 0) h[j] = fmaxf(acc + ba[j], 0.f);
  }
  __syncthreads();
  for (int o = tid; o < 2 * D; o += kMlpThreads) {
    float acc = bb[o];
    for (int j = 0; j < hidden; ++j) acc += wb[(size_t)o * hidden + j] * h[j];
    l[o] = acc;
    if (logits2) logits2[(size_t)n * 2 * D + o] = acc;
  }
  __syncthreads();
  for (int d = tid; d < D; d += kMlpThreads) cmask[(size_t)n * D + d] = (l[2 * d] > l[2 * d + 1]) ? 1 : 0;  // false for NaN
}

// Slabs per sample: about sixteen pixels per block (the partial sums are float32, so every slab writes
// twice a pixel's bytes: few pixels per slab would write more than the kernel reads), more slabs only
// while the grid is short of a thousand blocks and a slab keeps at least four pixels.
static int gap_slabs(int N, int HW) {
  int s = HW / 16;
  if (s < 1) s = 1;
  if (s > 64) s = 64;
  while ((long long)N * s < 1024 && s * 2 <= HW / 4 && s * 2 <= 64) s *= 2;
  return s;
}

}  // namespace laud

using namespace laud;

extern "C" size_t laud_channel_masker_workspace(laud_fmap fx) {
  if (!valid_fmap(fx)) return 0;
  return align_up((size_t)fx.N * gap_slabs(fx.N, fx.H * fx.W) * fx.C * sizeof(float), 256);
}

extern "C" int laud_channel_masker(const void* x, laud_fmap fx, const float* wa, const float* ba, int hidden,
                                   const float* wb, const float* bb, int D, uint8_t* cmask, float* logits2, void* ws,
                                   size_t ws_bytes, void* stream) {
  if (!x || !wa || !ba || !wb || !bb || !cmask || !valid_fmap(fx) || hidden <= 0 || D <= 0) return LAUD_ERR_INVALID_ARG;
  if (fx.C % 8 || fx.C > 256 * 8 * 4) return LAUD_ERR_UNSUPPORTED;
  if ((size_t)(fx.C + hidden + 2 * D) * sizeof(float) > 60000) return LAUD_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < laud_channel_masker_workspace(fx)) return LAUD_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  const int HW = fx.H * fx.W, slabs = gap_slabs(fx.N, HW);
  float* partial = (float*)ws;
  if (fx.dtype == LAUD_BF16)
    hipLaunchKernelGGL((k_gap_partial<bf16_t>), dim3(fx.N * slabs), dim3(kGapThreads), 0, st, (const bf16_t*)x, HW,
                       fx.C, slabs, partial);
  else
    hipLaunchKernelGGL((k_gap_partial<float>), dim3(fx.N * slabs), dim3(kGapThreads), 0, st, (const float*)x, HW,
                       fx.C, slabs, partial);
  if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;
  hipLaunchKernelGGL(k_channel_mlp, dim3(fx.N), dim3(kMlpThreads), (size_t)(fx.C + hidden + 2 * D) * sizeof(float), st,
                     partial, slabs, HW, fx.C, wa, ba, hidden, wb, bb, D, cmask, logits2);
  return check_launch();
}
