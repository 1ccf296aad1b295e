// Re-ordering of a block's w2 / w3 into the order the fused conv2 -> conv3 kernel streams them (shared by that
// kernel's file and by the GEMM kernel, whose spare workgroups do the copy while the first 1x1 runs).
#pragma once

#include "laud_common.h"

namespace laud {
namespace tail {
constexpr int kMid = 256;                     // mid width the fused kernel is built for
constexpr int kWaves = 8, kThreads = 512;
constexpr int kKch = kMid / 64;               // K slices (64 channels) per tap of the 3x3 and per column tile of the 1x1
constexpr int kSl2 = 9 * kKch;                // slices of the 3x3
constexpr int kSliceChunks = kWaves * 4 * 64; // 16-byte chunks of one packed weight slice (32 KB)
__host__ __device__ constexpr int packed_slices(int cout) { return kSl2 + cout / 256 * kKch; }
__host__ __device__ constexpr size_t packed_bytes(int cout) { return (size_t)packed_slices(cout) * kSliceChunks * 16; }
}  // namespace tail

// Chunk idx of the packed stream: slice b = idx / 2048 (b < 36: tap b/4, K chunk b%4 of the 3x3; then column tile
// (b-36)/4, K chunk (b-36)%4 of the last 1x1), wave w, K step kg, lane l hold the 16 bytes
// W[channel 32w + l%32 (+256*tile)][k = 64*chunk + 16*kg + 8*(l/32) .. +7]: the MFMA fragment of that lane, so that
// a wave instruction of the consumer reads 1 KB in a row.  Pure data movement.
__device__ __forceinline__ void tail_pack_chunk(int idx, const uint4* __restrict__ w2, const uint4* __restrict__ w3,
                                                uint4* __restrict__ out) {
  using namespace tail;
  const int l = idx & 63, kg = (idx >> 6) & 3, w = (idx >> 8) & 7, b = idx >> 11;
  const int k = kg * 16 + (l >> 5) * 8;  // within the 64-element slice
  if (b < kSl2) {
    const int tap = b / kKch, kc = b % kKch, ch = 32 * w + (l & 31);
    out[idx] = w2[((size_t)(ch * 9 + tap) * kMid + kc * 64 + k) / 8];
  } else {
    const int c = b - kSl2, ct = c / kKch, ks = c % kKch, ch = ct * 256 + 32 * w + (l & 31);
    out[idx] = w3[((size_t)ch * kMid + ks * 64 + k) / 8];
  }
}
}  // namespace laud
