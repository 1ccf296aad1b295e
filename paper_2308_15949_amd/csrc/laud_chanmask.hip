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
      for (int p = p0 + pl; p < p1; p += lanes) {
        const uint4 raw = *reinterpret_cast<const uint4*>(x + ((size_t)n * HW + p) * C + (size_t)cv * EPC);
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

__global__ __launch_bounds__(256) void k_channel_mlp(const float* __restrict__ partial, int slabs, int HW, int C,
                                                     const float* __restrict__ wa, const float* __restrict__ ba,
                                                     int hidden, const float* __restrict__ wb,
                                                     const float* __restrict__ bb, int D,
                                                     uint8_t* __restrict__ cmask, float* __restrict__ logits2) {
  extern __shared__ float sm[];  // g[C], h[hidden], l[2D]
  float* g = sm;
  float* h = g + C;
  float* l = h + hidden;
  const int n = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const float inv = 1.0f / (float)HW;
  for (int c = tid; c < C; c += 256) {
    float s = 0.f;
    for (int k = 0; k < slabs; ++k) s += partial[((size_t)n * slabs + k) * C + c];
    g[c] = s * inv;
  }
  __syncthreads();
  for (int j = wave; j < hidden; j += 4) {  // one wave per hidden unit
    float acc = 0.f;
    for (int c = lane; c < C; c += kWave) acc += wa[(size_t)j * C + c] * g[c];
    acc = wave_sum(acc);
    if (lane == 0) h[j] = fmaxf(acc + ba[j], 0.f);
  }
  __syncthreads();
  for (int o = tid; o < 2 * D; o += 256) {
    float acc = bb[o];
    for (int j = 0; j < hidden; ++j) acc += wb[(size_t)o * hidden + j] * h[j];
    l[o] = acc;
    if (logits2) logits2[(size_t)n * 2 * D + o] = acc;
  }
  __syncthreads();
  for (int d = tid; d < D; d += 256) cmask[(size_t)n * D + d] = (l[2 * d] > l[2 * d + 1]) ? 1 : 0;  // false for NaN
}

static int gap_slabs(int N, int HW) {
  int s = (2048 + N - 1) / N;  // aim at a couple of thousand blocks
  if (s > HW) s = HW;
  if (s < 1) s = 1;
  if (s > 64) s = 64;
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
  hipLaunchKernelGGL(k_channel_mlp, dim3(fx.N), dim3(256), (size_t)(fx.C + hidden + 2 * D) * sizeof(float), st,
                     partial, slabs, HW, fx.C, wa, ba, hidden, wb, bb, D, cmask, logits2);
  return check_launch();
}
