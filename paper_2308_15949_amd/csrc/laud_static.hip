// Static stem of the ResNet body (BASELINE config 3): 7x7 stride-2 conv on the 3-channel image with
// folded-BN affine and ReLU, then 3x3 stride-2 max pooling.  Both are outside the dynamic hot path
// (they run once per image and are not masked); they are plain direct kernels, written for
// correctness and reasonable memory behaviour, not tuned.
#include "laud_common.h"

namespace laud {

constexpr int kStemK = 7 * 7 * 3;  // reduction length of the stem conv

// Block = 32 output pixels x (c_out / 8) channel groups (256 threads at c_out = 64).  The weights sit
// in LDS as float32 [k][c_out]; every thread accumulates 8 output channels of one pixel.
template <typename ET>
__global__ __launch_bounds__(256) void k_stem_conv(const ET* __restrict__ x, int N, int Hin, int Win,
                                                   const ET* __restrict__ w7, const float* __restrict__ s,
                                                   const float* __restrict__ t, int c_out, int Ho, int Wo,
                                                   ET* __restrict__ out) {
  extern __shared__ float s_w[];  // [kStemK][c_out]
  const int groups = c_out / 8;
  for (int i = threadIdx.x; i < kStemK * c_out; i += blockDim.x) {
    const int o = i / kStemK, k = i - o * kStemK;  // source layout [c_out][7][7][3]
    s_w[k * c_out + o] = elem<ET>::load(w7 + i);
  }
  __syncthreads();
  const int g = threadIdx.x % groups, pl = threadIdx.x / groups;
  const int ppb = blockDim.x / groups;
  const long long pix = (long long)blockIdx.x * ppb + pl;
  if (pl >= ppb || pix >= (long long)N * Ho * Wo) return;
  const int n = (int)(pix / (Ho * Wo)), r = (int)(pix - (long long)n * Ho * Wo);
  const int yo = r / Wo, xo = r - yo * Wo;
  float acc[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) acc[e] = 0.f;
  for (int ky = 0; ky < 7; ++ky) {
    const int yy = yo * 2 - 3 + ky;
    if (yy < 0 || yy >= Hin) continue;
    for (int kx = 0; kx < 7; ++kx) {
      const int xx = xo * 2 - 3 + kx;
      if (xx < 0 || xx >= Win) continue;
      const ET* px = x + (((size_t)n * Hin + yy) * Win + xx) * 3;
#pragma unroll
      for (int c = 0; c < 3; ++c) {
        const float v = elem<ET>::load(px + c);
        const float* wk = s_w + ((ky * 7 + kx) * 3 + c) * c_out + g * 8;
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] += v * wk[e];
      }
    }
  }
  ET* po = out + (size_t)pix * c_out + g * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) elem<ET>::store(po + e, fmaxf(acc[e] * s[g * 8 + e] + t[g * 8 + e], 0.f));
}

// One thread per (output pixel, 8 channels).
template <typename ET>
__global__ __launch_bounds__(256) void k_maxpool3x3s2(const ET* __restrict__ in, int N, int H, int W, int C, int Ho,
                                                      int Wo, ET* __restrict__ out) {
  const int groups = C / 8;
  const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
  if (id >= (long long)N * Ho * Wo * groups) return;
  const int g = (int)(id % groups);
  const long long pix = id / groups;
  const int n = (int)(pix / (Ho * Wo)), r = (int)(pix - (long long)n * Ho * Wo);
  const int yo = r / Wo, xo = r - yo * Wo;
  float m[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) m[e] = -INFINITY;
  for (int ky = 0; ky < 3; ++ky) {
    const int yy = yo * 2 - 1 + ky;
    if (yy < 0 || yy >= H) continue;
    for (int kx = 0; kx < 3; ++kx) {
      const int xx = xo * 2 - 1 + kx;
      if (xx < 0 || xx >= W) continue;
      const ET* p = in + (((size_t)n * H + yy) * W + xx) * C + g * 8;
#pragma unroll
      for (int e = 0; e < 8; ++e) m[e] = fmaxf(m[e], elem<ET>::load(p + e));
    }
  }
  ET* po = out + (size_t)pix * C + g * 8;
#pragma unroll
  for (int e = 0; e < 8; ++e) elem<ET>::store(po + e, m[e]);
}

}  // namespace laud

using namespace laud;

extern "C" size_t laud_stem_workspace(int N, int Hin, int Win, int c_out, int dtype) {
  if (N <= 0 || Hin <= 0 || Win <= 0 || c_out <= 0 || (dtype != LAUD_F32 && dtype != LAUD_BF16)) return 0;
  return align_up((size_t)N * ((Hin - 1) / 2 + 1) * ((Win - 1) / 2 + 1) * c_out * elem_bytes(dtype), 256);
}

extern "C" int laud_stem(const void* x, int N, int Hin, int Win, int dtype, const void* w7, const float* s,
                         const float* t, int c_out, void* out, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !w7 || !s || !t || !out || N <= 0 || Hin <= 0 || Win <= 0 || c_out <= 0) return LAUD_ERR_INVALID_ARG;
  if (dtype != LAUD_F32 && dtype != LAUD_BF16) return LAUD_ERR_INVALID_ARG;
  if (c_out % 8 || c_out > 96) return LAUD_ERR_UNSUPPORTED;  // weights are held in LDS as float32
  if (!ws || ws_bytes < laud_stem_workspace(N, Hin, Win, c_out, dtype)) return LAUD_ERR_WORKSPACE;
  const int Hc = (Hin - 1) / 2 + 1, Wc = (Win - 1) / 2 + 1;  // 7x7, stride 2, pad 3
  const int Hp = (Hc - 1) / 2 + 1, Wp = (Wc - 1) / 2 + 1;    // 3x3, stride 2, pad 1
  if ((long long)N * Hc * Wc > 0x7fffffffLL) return LAUD_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  const int groups = c_out / 8, threads = 256 / groups * groups, ppb = threads / groups;
  const long long npix = (long long)N * Hc * Wc;
  const unsigned cblocks = (unsigned)((npix + ppb - 1) / ppb);
  const size_t lds = (size_t)kStemK * c_out * sizeof(float);
  const long long pool_items = (long long)N * Hp * Wp * groups;
  const unsigned pblocks = (unsigned)((pool_items + 255) / 256);
  if (dtype == LAUD_BF16) {
    hipLaunchKernelGGL((k_stem_conv<bf16_t>), dim3(cblocks), dim3(threads), lds, st, (const bf16_t*)x, N, Hin, Win,
                       (const bf16_t*)w7, s, t, c_out, Hc, Wc, (bf16_t*)ws);
    hipLaunchKernelGGL((k_maxpool3x3s2<bf16_t>), dim3(pblocks), dim3(256), 0, st, (const bf16_t*)ws, N, Hc, Wc, c_out,
                       Hp, Wp, (bf16_t*)out);
  } else {
    hipLaunchKernelGGL((k_stem_conv<float>), dim3(cblocks), dim3(threads), lds, st, (const float*)x, N, Hin, Win,
                       (const float*)w7, s, t, c_out, Hc, Wc, (float*)ws);
    hipLaunchKernelGGL((k_maxpool3x3s2<float>), dim3(pblocks), dim3(256), 0, st, (const float*)ws, N, Hc, Wc, c_out, Hp,
                       Wp, (float*)out);
  }
  return check_launch();
}
