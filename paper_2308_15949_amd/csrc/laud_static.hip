// Static stem of the ResNet body (the whole-body workload): 7x7 stride-2 conv on the 3-channel image with
// folded-BN affine and ReLU, then 3x3 stride-2 max pooling.  Outside the dynamic hot path (it runs once
// per image and is not masked): an im2col kernel feeds the dense MFMA GEMM of laud_gemm.hip, a plain
// kernel pools.
#include "laud_common.h"

namespace laud {

constexpr int kStemK = 7 * 7 * 3;  // reduction length of the stem conv ...

constexpr int kStemKp = 152;       // ... padded to a multiple of 8 (16-byte chunks of the GEMM)

// im2col of the 7x7 stride-2 pad-3 windows: row = output pixel, column k = (ky*7 + kx)*3 + c, zero
// outside the image and in the padding columns.  One thread per (row, 8 consecutive columns).
template <typename ET>
__global__ __launch_bounds__(256) void k_stem_im2col(const ET* __restrict__ x, int N, int Hin, int Win, int Ho, int Wo,
                                                     ET* __restrict__ cols) {
  constexpr int CH = kStemKp / 8;
  const long long id = (long long)blockIdx.x * 256 + threadIdx.x;
  if (id >= (long long)N * Ho * Wo * CH) return;
  const int ch = (int)(id % CH);
  const long long pix = id / CH;
  const int n = (int)(pix / (Ho * Wo)), r = (int)(pix - (long long)n * Ho * Wo);
  const int yo = r / Wo, xo = r - yo * Wo;
  ET v[8];
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int k = ch * 8 + e;
    const int tap = k / 3, c = k - tap * 3;
    const int yy = yo * 2 - 3 + tap / 7, xx = xo * 2 - 3 + tap % 7;
    const bool ok = k < kStemK && yy >= 0 && yy < Hin && xx >= 0 && xx < Win;
    v[e] = ok ? x[(((size_t)n * Hin + yy) * Win + xx) * 3 + c] : (ET)0;
  }
  // 8 elements = one 16-byte store (bf16) or two (float32)
  uint4 raw[sizeof(v) / 16];
  __builtin_memcpy(raw, v, sizeof(v));
  uint4* dst = reinterpret_cast<uint4*>(cols + (size_t)pix * kStemKp + ch * 8);
#pragma unroll
  for (int q = 0; q < (int)(sizeof(v) / 16); ++q) dst[q] = raw[q];
}

// Weights [c_out][7][7][3] -> [c_out][kStemKp] with zero padding columns.
template <typename ET>
__global__ void k_stem_pack_weights(const ET* __restrict__ w7, int c_out, ET* __restrict__ wp) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= c_out * kStemKp) return;
  const int o = i / kStemKp, k = i - o * kStemKp;
  wp[i] = k < kStemK ? w7[o * kStemK + k] : (ET)0;
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

namespace {
struct StemWs { size_t cols, wp, conv, bytes; };
StemWs stem_ws_layout(int N, int Hin, int Win, int c_out, int dtype) {
  const size_t eb = elem_bytes(dtype), rows = (size_t)N * ((Hin - 1) / 2 + 1) * ((Win - 1) / 2 + 1);
  StemWs w;
  size_t o = 0;
  w.cols = o; o += align_up(rows * kStemKp * eb, 256);
  w.wp = o;   o += align_up((size_t)c_out * kStemKp * eb, 256);
  w.conv = o; o += align_up(rows * c_out * eb, 256);
  w.bytes = o;
  return w;
}
}  // namespace

extern "C" size_t laud_stem_workspace(int N, int Hin, int Win, int c_out, int dtype) {
  if (N <= 0 || Hin <= 0 || Win <= 0 || c_out <= 0 || (dtype != LAUD_F32 && dtype != LAUD_BF16)) return 0;
  return stem_ws_layout(N, Hin, Win, c_out, dtype).bytes;
}

extern "C" int laud_stem(const void* x, int N, int Hin, int Win, int dtype, const void* w7, const float* s,
                         const float* t, int c_out, void* out, void* ws, size_t ws_bytes, void* stream) {
  if (!x || !w7 || !s || !t || !out || N <= 0 || Hin <= 0 || Win <= 0 || c_out <= 0) return LAUD_ERR_INVALID_ARG;
  if (dtype != LAUD_F32 && dtype != LAUD_BF16) return LAUD_ERR_INVALID_ARG;
  if (c_out % 8) return LAUD_ERR_UNSUPPORTED;
  if (!ws || ws_bytes < laud_stem_workspace(N, Hin, Win, c_out, dtype)) return LAUD_ERR_WORKSPACE;
  const int Hc = (Hin - 1) / 2 + 1, Wc = (Win - 1) / 2 + 1;  // 7x7, stride 2, pad 3
  const int Hp = (Hc - 1) / 2 + 1, Wp = (Wc - 1) / 2 + 1;    // 3x3, stride 2, pad 1
  const long long rows = (long long)N * Hc * Wc;
  if (rows > 0x7fffffffLL / 2) return LAUD_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  const StemWs L = stem_ws_layout(N, Hin, Win, c_out, dtype);
  char* wsb = (char*)ws;
  void *cols = wsb + L.cols, *wp = wsb + L.wp, *conv = wsb + L.conv;
  const unsigned iblocks = (unsigned)((rows * (kStemKp / 8) + 255) / 256);
  const unsigned wblocks = (unsigned)((c_out * kStemKp + 255) / 256);
  const unsigned pblocks = (unsigned)(((long long)N * Hp * Wp * (c_out / 8) + 255) / 256);
  if (dtype == LAUD_BF16) {
    hipLaunchKernelGGL((k_stem_im2col<bf16_t>), dim3(iblocks), dim3(256), 0, st, (const bf16_t*)x, N, Hin, Win, Hc, Wc,
                       (bf16_t*)cols);
    hipLaunchKernelGGL((k_stem_pack_weights<bf16_t>), dim3(wblocks), dim3(256), 0, st, (const bf16_t*)w7, c_out,
                       (bf16_t*)wp);
  } else {
    hipLaunchKernelGGL((k_stem_im2col<float>), dim3(iblocks), dim3(256), 0, st, (const float*)x, N, Hin, Win, Hc, Wc,
                       (float*)cols);
    hipLaunchKernelGGL((k_stem_pack_weights<float>), dim3(wblocks), dim3(256), 0, st, (const float*)w7, c_out,
                       (float*)wp);
  }
  if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;
  int rc = launch_dense_affine(dtype, cols, wp, s, t, conv, rows, kStemKp, c_out, 1, st);
  if (rc != LAUD_OK) return rc;
  if (dtype == LAUD_BF16)
    hipLaunchKernelGGL((k_maxpool3x3s2<bf16_t>), dim3(pblocks), dim3(256), 0, st, (const bf16_t*)conv, N, Hc, Wc, c_out,
                       Hp, Wp, (bf16_t*)out);
  else
    hipLaunchKernelGGL((k_maxpool3x3s2<float>), dim3(pblocks), dim3(256), 0, st, (const float*)conv, N, Hc, Wc, c_out, Hp,
                       Wp, (float*)out);
  return check_launch();
}
