// Static stem of the ResNet body (the whole-body workload): 7x7 stride-2 conv on the 3-channel image with
// folded-BN affine and ReLU, then 3x3 stride-2 max pooling.  Outside the dynamic hot path (it runs once
// per image and is not masked): the usual shape (bf16, 64 channels) is an implicit GEMM straight from the
// image, other shapes go through an im2col kernel and the dense MFMA GEMM of laud_gemm.hip; a plain kernel
// pools.
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

// ---- fused stem conv for the usual shape (bf16, 64 output channels) -----------------------------
// The 7x7 stride-2 conv as an implicit GEMM straight from the image: no im2col buffer in HBM (it is
// 13 times the image).  A block walks the 8 x 16-pixel output tiles of one band of 8 output rows; per tile
// it puts the 21 x 38 input pixels the tile's windows cover into LDS, four bf16 per pixel (the fourth is
// zero), and runs 32x32x16 MFMAs whose 8-element A fragments are two neighbouring pixels of one window
// row: K = 7 rows x 8 taps x 4 channels = 224 with zero weights at the eighth tap and the fourth channel.
// The weights are rearranged into that K order in LDS once per block.  Folded-BN affine and ReLU in the
// accumulators, output rows through LDS so that stores are 16 bytes.
typedef __attribute__((ext_vector_type(16))) float stem_f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 stem_bf16x8;
constexpr int kSTY = 8, kSTX = 16;                    // output tile: 128 GEMM rows
constexpr int kSPY = 2 * kSTY + 5, kSPW = 2 * kSTX + 6;  // 21 x 38 input pixels (38 is even and holds the padded 8th tap)
constexpr int kSK = 7 * 32;                           // reduction length in the padded order
constexpr int kSWS = kSK * 2 + 16;                    // LDS weight row stride in bytes
constexpr int kSOS = 64 * 2 + 16;                     // LDS output row stride in bytes
__global__ __launch_bounds__(256) void k_stem_conv_bf16(const bf16_t* __restrict__ x, int N, int Hin, int Win, int Hc,
                                                        int Wc, const bf16_t* __restrict__ w7,
                                                        const float* __restrict__ s, const float* __restrict__ t,
                                                        bf16_t* __restrict__ out) {
  __shared__ __align__(16) unsigned char s_w[64 * kSWS];
  __shared__ __align__(16) unsigned char s_p[kSPY * kSPW * 8];
  __shared__ __align__(16) unsigned char s_o[kSTY * kSTX * kSOS];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
  const int r = lane & 31, h = lane >> 5;
  for (int i = tid; i < 64 * kSK; i += 256) {
    const int col = i / kSK, k = i - col * kSK;
    const int ky = k >> 5, kx = (k & 31) >> 2, c = k & 3;
    bf16_t v = 0;
    if (kx < 7 && c < 3) v = w7[col * kStemK + (ky * 7 + kx) * 3 + c];
    *reinterpret_cast<bf16_t*>(s_w + col * kSWS + k * 2) = v;
  }
  const int nbands = (Hc + kSTY - 1) / kSTY;
  const int n = blockIdx.x / nbands, y0 = (blockIdx.x - n * nbands) * kSTY;
  const int col = wn * 32 + r;
  const float sc = s[col], sh = t[col];
  for (int x0 = 0; x0 < Wc; x0 += kSTX) {
    __syncthreads();  // the previous tile's reads of s_p and s_o are over (first pass: the weights are in place)
    for (int p = tid; p < kSPY * kSPW; p += 256) {
      const int py = p / kSPW, px = p - py * kSPW;
      const int iy = 2 * y0 - 3 + py, ix = 2 * x0 - 3 + px;
      bf16_t v0 = 0, v1 = 0, v2 = 0;
      if (iy >= 0 && iy < Hin && ix >= 0 && ix < Win) {
        const bf16_t* src = x + (((size_t)n * Hin + iy) * Win + ix) * 3;
        v0 = src[0]; v1 = src[1]; v2 = src[2];
      }
      uint2 pk;
      pk.x = (unsigned)v0 | ((unsigned)v1 << 16);
      pk.y = (unsigned)v2;
      *reinterpret_cast<uint2*>(s_p + p * 8) = pk;
    }
    __syncthreads();
    stem_f32x16 acc[2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][e] = 0.f;
#pragma unroll
    for (int st = 0; st < kSK / 16; ++st) {
      const int f = 2 * st + h, ky = f >> 2, j = f & 3;  // this lane's fragment: window row ky, taps 2j and 2j+1
      const uint4 b = *reinterpret_cast<const uint4*>(s_w + col * kSWS + (st * 16 + h * 8) * 2);
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int rr = wm * 64 + i * 32 + r, yo = rr >> 4, xo = rr & 15;
        const uint4 a = *reinterpret_cast<const uint4*>(s_p + ((2 * yo + ky) * kSPW + 2 * xo + 2 * j) * 8);
        acc[i] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(stem_bf16x8, a),
                                                         __builtin_bit_cast(stem_bf16x8, b), acc[i], 0, 0, 0);
      }
    }
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int e = 0; e < 16; ++e) {
        const int row = wm * 64 + i * 32 + 8 * (e >> 2) + 4 * h + (e & 3);
        *reinterpret_cast<bf16_t*>(s_o + row * kSOS + col * 2) = f32_to_bf16(fmaxf(acc[i][e] * sc + sh, 0.f));
      }
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int id = tid + q * 256, row = id >> 3, ch = id & 7;
      const int Y = y0 + (row >> 4), X = x0 + (row & 15);
      if (Y < Hc && X < Wc)
        *reinterpret_cast<uint4*>(out + (((size_t)n * Hc + Y) * Wc + X) * 64 + ch * 8) =
            *reinterpret_cast<const uint4*>(s_o + row * kSOS + ch * 16);
    }
  }
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

// Stem of the RegNet backbones: 3x3 stride-2 pad-1 conv from the 3-channel image, affine, ReLU.  One thread per
// output pixel: the 27 inputs of its window are read once into registers, then the output channels are produced
// eight at a time from the 27 x c_out float32 weights in LDS (all lanes read the same weight: a broadcast).
// HBM-bound: the image is read once (neighbouring windows overlap in cache) and the output written once.
template <typename ET>
__global__ __launch_bounds__(256) void k_stem3x3(const ET* __restrict__ in, int N, int H, int W, int Ho, int Wo,
                                                 const ET* __restrict__ w, const float* __restrict__ s,
                                                 const float* __restrict__ t, int C, ET* __restrict__ out) {
  extern __shared__ float s_w3[];  // [27][C] weights (tap-major, output channel fastest), then scale [C], shift [C]
  for (int i = threadIdx.x; i < 27 * C; i += 256) {
    const int o = i % C, k = i / C;
    s_w3[i] = elem<ET>::load(w + (size_t)o * 27 + k);
  }
  float* s_sc = s_w3 + 27 * C;
  float* s_sh = s_sc + C;
  for (int i = threadIdx.x; i < C; i += 256) { s_sc[i] = s[i]; s_sh[i] = t[i]; }
  __syncthreads();
  const long long pix = (long long)blockIdx.x * 256 + threadIdx.x;
  if (pix >= (long long)N * Ho * Wo) return;
  const int n = (int)(pix / (Ho * Wo)), r = (int)(pix - (long long)n * Ho * Wo);
  const int yo = r / Wo, xo = r - yo * Wo;
  float v[27];
#pragma unroll
  for (int ky = 0; ky < 3; ++ky) {
    const int yy = yo * 2 - 1 + ky;
#pragma unroll
    for (int kx = 0; kx < 3; ++kx) {
      const int xx = xo * 2 - 1 + kx;
      const bool ok = yy >= 0 && yy < H && xx >= 0 && xx < W;
      const ET* p = in + (((size_t)n * H + (ok ? yy : 0)) * W + (ok ? xx : 0)) * 3;
#pragma unroll
      for (int c = 0; c < 3; ++c) v[(ky * 3 + kx) * 3 + c] = ok ? elem<ET>::load(p + c) : 0.f;
    }
  }
  ET* po = out + (size_t)pix * C;
  for (int g = 0; g < C; g += 8) {
    float acc[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) acc[e] = 0.f;
#pragma unroll
    for (int k = 0; k < 27; ++k) {
      const float* wk = s_w3 + k * C + g;
#pragma unroll
      for (int e = 0; e < 8; ++e) acc[e] += v[k] * wk[e];
    }
    ET o8[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) elem<ET>::store(&o8[e], fmaxf(acc[e] * s_sc[g + e] + s_sh[g + e], 0.f));
    if constexpr (sizeof(ET) == 2) {
      uint4 q;
      __builtin_memcpy(&q, o8, 16);
      *reinterpret_cast<uint4*>(po + g) = q;
    } else {
      uint4 q0, q1;
      __builtin_memcpy(&q0, o8, 16);
      __builtin_memcpy(&q1, o8 + 4, 16);
      reinterpret_cast<uint4*>(po + g)[0] = q0;
      reinterpret_cast<uint4*>(po + g)[1] = q1;
    }
  }
}

}  // namespace laud

using namespace laud;

extern "C" int laud_stem3x3(const void* x, int N, int Hin, int Win, int dtype, const void* w3, const float* s,
                            const float* t, int c_out, void* out, void* stream) {
  if (!x || !w3 || !s || !t || !out || N <= 0 || Hin <= 0 || Win <= 0 || c_out <= 0) return LAUD_ERR_INVALID_ARG;
  if (dtype != LAUD_F32 && dtype != LAUD_BF16) return LAUD_ERR_INVALID_ARG;
  if (c_out % 8 || c_out > 256) return LAUD_ERR_UNSUPPORTED;
  const int Ho = (Hin - 1) / 2 + 1, Wo = (Win - 1) / 2 + 1;
  const long long work = (long long)N * Ho * Wo;
  if ((work + 255) / 256 > 0x7fffffffLL) return LAUD_ERR_UNSUPPORTED;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  const unsigned blocks = (unsigned)((work + 255) / 256);
  const size_t lds = (size_t)29 * c_out * sizeof(float);
  if (dtype == LAUD_BF16)
    hipLaunchKernelGGL((k_stem3x3<bf16_t>), dim3(blocks), dim3(256), lds, st, (const bf16_t*)x, N, Hin, Win, Ho, Wo,
                       (const bf16_t*)w3, s, t, c_out, (bf16_t*)out);
  else
    hipLaunchKernelGGL((k_stem3x3<float>), dim3(blocks), dim3(256), lds, st, (const float*)x, N, Hin, Win, Ho, Wo,
                       (const float*)w3, s, t, c_out, (float*)out);
  return check_launch();
}

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
  const unsigned pblocks0 = (unsigned)(((long long)N * Hp * Wp * (c_out / 8) + 255) / 256);
  if (dtype == LAUD_BF16 && c_out == 64) {  // the usual stem: conv straight from the image, then the pooling kernel
    const unsigned bands = (unsigned)(N * ((Hc + kSTY - 1) / kSTY));
    hipLaunchKernelGGL(k_stem_conv_bf16, dim3(bands), dim3(256), 0, st, (const bf16_t*)x, N, Hin, Win, Hc, Wc,
                       (const bf16_t*)w7, s, t, (bf16_t*)conv);
    if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;
    hipLaunchKernelGGL((k_maxpool3x3s2<bf16_t>), dim3(pblocks0), dim3(256), 0, st, (const bf16_t*)conv, N, Hc, Wc, c_out,
                       Hp, Wp, (bf16_t*)out);
    return check_launch();
  }
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
