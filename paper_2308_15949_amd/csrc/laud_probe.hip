// Achievable-peak probes: the two denominators a roofline fraction can be read against besides the
// published peaks -- what a bare MFMA loop and a plain copy kernel reach on the machine at hand.
// Measurement aids, not part of the method; the benchmark times them with events on their stream.
#include "laud_common.h"

namespace laud {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;

constexpr int kProbeThreads = 512;   // 8 waves: two per SIMD, like the GEMM kernels
constexpr int kProbeChains = 4;      // independent accumulators per wave (MFMA latency covered)

// Every wave issues iters * kProbeChains MFMAs (32x32x16 bf16, or 4 x 32x32x2 fp32 = the same FLOPs) on
// register operands: nothing but the matrix pipe is exercised.
template <bool BF16>
__global__ __launch_bounds__(kProbeThreads) void k_probe_mfma(int iters, float* sink) {
  f32x16 acc[kProbeChains];
#pragma unroll
  for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[c][e] = 0.f;
  const float seed = 1.0f + (float)(threadIdx.x & 7) * 0.125f;
  uint4 a = make_uint4(0x3f803f80u, 0x3f803f80u, 0x3f803f80u, 0x3f803f80u);  // bf16 ones
  uint4 b = a;
  if (threadIdx.x == 4096) a.x = 0;  // never true: keeps the operands out of constant folding
  for (int i = 0; i < iters; ++i) {
#pragma unroll
    for (int c = 0; c < kProbeChains; ++c) {
      if constexpr (BF16) {
        acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b),
                                                         acc[c], 0, 0, 0);
      } else {
#pragma unroll
        for (int u = 0; u < 4; ++u) acc[c] = __builtin_amdgcn_mfma_f32_32x32x2f32(seed, seed, acc[c], 0, 0, 0);
      }
    }
  }
  float s = 0.f;
#pragma unroll
  for (int c = 0; c < kProbeChains; ++c)
#pragma unroll
    for (int e = 0; e < 16; ++e) s += acc[c][e];
  if (s == -1.f) sink[0] = s;  // never true (sums are positive): the accumulators stay live
}

// Grid-stride copy, 16 bytes per lane and four loads in flight per lane.
__global__ __launch_bounds__(256) void k_probe_copy(const uint4* __restrict__ src, uint4* __restrict__ dst, size_t n16) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  for (; i + 3 * stride < n16; i += 4 * stride) {
    const uint4 v0 = src[i], v1 = src[i + stride], v2 = src[i + 2 * stride], v3 = src[i + 3 * stride];
    dst[i] = v0; dst[i + stride] = v1; dst[i + 2 * stride] = v2; dst[i + 3 * stride] = v3;
  }
  for (; i < n16; i += stride) dst[i] = src[i];
}

// Read-only stream: every lane sums its 16-byte pieces (eight loads in flight per lane); one word per block is
// written so that the loads stay.
__global__ __launch_bounds__(256) void k_probe_read(const uint4* __restrict__ src, size_t n16, unsigned* __restrict__ sink) {
  const size_t stride = (size_t)gridDim.x * 256;
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  unsigned acc = 0;
  for (; i + 7 * stride < n16; i += 8 * stride) {
    uint4 v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = src[i + u * stride];
#pragma unroll
    for (int u = 0; u < 8; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
  }
  for (; i < n16; i += stride) { const uint4 v = src[i]; acc += v.x ^ v.y ^ v.z ^ v.w; }
  if (acc == 0x9e3779b9u) sink[blockIdx.x & 15] = acc;  // (practically never: keeps the sum alive)
}

}  // namespace laud

using namespace laud;

extern "C" int laud_probe_mfma(int dtype, int iters, int blocks, double* flops, float* sink, void* stream) {
  if (iters <= 0 || blocks <= 0 || !sink || (dtype != LAUD_F32 && dtype != LAUD_BF16)) return LAUD_ERR_INVALID_ARG;
  clear_stale_error();
  hipStream_t st = (hipStream_t)stream;
  if (dtype == LAUD_BF16) hipLaunchKernelGGL((k_probe_mfma<true>), dim3(blocks), dim3(kProbeThreads), 0, st, iters, sink);
  else hipLaunchKernelGGL((k_probe_mfma<false>), dim3(blocks), dim3(kProbeThreads), 0, st, iters, sink);
  // one 32x32x16 MFMA (or its four 32x32x2 steps) = 2*32*32*16 FLOPs
  if (flops) *flops = (double)blocks * (kProbeThreads / kWave) * (double)iters * kProbeChains * 32768.0 / (dtype == LAUD_BF16 ? 1.0 : 2.0);
  return check_launch();
}

extern "C" int laud_probe_copy(const void* src, void* dst, size_t bytes, void* stream) {
  if (!src || !dst || bytes == 0 || bytes % 16 || (reinterpret_cast<uintptr_t>(src) & 15) ||
      (reinterpret_cast<uintptr_t>(dst) & 15))
    return LAUD_ERR_INVALID_ARG;
  clear_stale_error();
  hipLaunchKernelGGL(k_probe_copy, dim3(256 * 8), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, (uint4*)dst,
                     bytes / 16);
  return check_launch();
}

extern "C" int laud_probe_read(const void* src, size_t bytes, float* sink, void* stream) {
  if (!src || !sink || bytes == 0 || bytes % 16 || (reinterpret_cast<uintptr_t>(src) & 15)) return LAUD_ERR_INVALID_ARG;
  clear_stale_error();
  const size_t n16 = bytes / 16;
  size_t blocks = (n16 + 256 * 8 - 1) / (256 * 8);  // eight pieces per lane when the buffer is small
  if (blocks > 256 * 8) blocks = 256 * 8;
  hipLaunchKernelGGL(k_probe_read, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)src, n16,
                     reinterpret_cast<unsigned*>(sink));
  return check_launch();
}
