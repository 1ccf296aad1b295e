// Squeeze-and-excitation module of the group-convolution / SE blocks (the RegNetY backbones of Sec. 4), applied
// to the compact rows h2 of the active patches between the 3x3 and the last 1x1 of a dynamic block.
#include "laud_common.h"

#include <algorithm>

namespace laud {

// The sample's active patches are a contiguous range of the ascending index list, so its h2 rows are
// contiguous too.  Four small kernels: per-sample channel means (fixed summation order: deterministic), the
// two fully connected layers batched over samples, and the rows multiplied by their sample's gate in place.
// The squeeze therefore averages over the sample's computed pixels; a sample without active patches has no rows.

constexpr int kSqThreads = 1024, kSqChunks = 128;

// grid (ceil(chunks per row / 128), N): z[n][c] = mean over the sample's rows of h2[row][c] for one block of
// up to 128 16-byte channel chunks (zeros for a sample without rows).  The threads are (chunk lane, row
// phase); every thread keeps eight row loads in flight; the row phases are added in a fixed order.
template <typename ET>
__global__ __launch_bounds__(kSqThreads) void k_se_squeeze(const ET* __restrict__ h2, const int32_t* __restrict__ idx,
                                                           const int32_t* __restrict__ count, int pps, int SS, int C,
                                                           float* __restrict__ z) {
  constexpr int EPC = elem<ET>::per16;
  __shared__ __align__(16) float s_part[kSqThreads * EPC];  // [row phase][chunk lane][EPC]
  const int n = blockIdx.y, tid = threadIdx.x;
  const int cnt = *count;
  const int lo = wave_lower_bound(idx, cnt, n * pps), hi = wave_lower_bound(idx, cnt, (n + 1) * pps);
  const int rows = (hi - lo) * SS;
  const int cpr = C / EPC;  // 16-byte chunks per row
  const int cb = blockIdx.x * kSqChunks, nch = min(kSqChunks, cpr - cb);
  int CP = 1;
  while (CP < nch) CP <<= 1;  // chunk lanes: a power of two that divides the thread count
  const int RP = kSqThreads / CP, cl = tid % CP, rp = tid / CP;
  const uint4* base = reinterpret_cast<const uint4*>(h2 + (long long)lo * SS * C) + cb;
  float acc[EPC];
#pragma unroll
  for (int e = 0; e < EPC; ++e) acc[e] = 0.f;
  if (cl < nch) {
    int r = rp;
    for (; r + 7 * RP < rows; r += 8 * RP) {
      uint4 v[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) v[u] = base[(size_t)(r + u * RP) * cpr + cl];
#pragma unroll
      for (int u = 0; u < 8; ++u) {
        ET t[EPC];
        __builtin_memcpy(t, &v[u], 16);
#pragma unroll
        for (int e = 0; e < EPC; ++e) acc[e] += elem<ET>::load(&t[e]);
      }
    }
    for (; r < rows; r += RP) {
      const uint4 v = base[(size_t)r * cpr + cl];
      ET t[EPC];
      __builtin_memcpy(t, &v, 16);
#pragma unroll
      for (int e = 0; e < EPC; ++e) acc[e] += elem<ET>::load(&t[e]);
    }
  }
#pragma unroll
  for (int e = 0; e < EPC; ++e) s_part[(rp * CP + cl) * EPC + e] = acc[e];
  __syncthreads();
  const float inv = rows > 0 ? 1.f / (float)rows : 0.f;
  for (int k = tid; k < nch * EPC; k += kSqThreads) {
    float t = 0.f;
    for (int q = 0; q < RP; ++q) t += s_part[q * CP * EPC + k];
    z[(size_t)n * C + cb * EPC + k] = t * inv;
  }
}

// The two small fully connected layers, batched over groups of kFcSamples samples so that a weight row read
// from L2 serves the whole group, and tiled over the outputs so that the grid fills the chip:
//   k_se_fc1: hid[n][k] = relu(w1[k] . z[n] + b1[k])
//   k_se_fc2: gate[n][c] = sigmoid(w2[c] . hid[n] + b2[c])
// One wave per four outputs at a time, lanes stride over the reduction with 16-byte loads, all loads of a
// step issued before their use.
constexpr int kFcSamples = 8, kFcThreads = 256, kFc1Tile = 16, kFc2Tile = 32;

// Sums 32 per-lane values over the 64 lanes of a wave with 32 shuffles instead of 32 x 6: each step exchanges
// one half of the remaining values with the partner lane and keeps the other half, so the number of values
// halves while the number of lanes summed doubles.  Returns, in lane l, the total of value
// 16*b5 + 8*b4 + 4*b3 + 2*b2 + b1 (b_i = bit i of l); lanes l and l^1 hold the same value.
template <int HALF>
__device__ __forceinline__ void wave_reduce_step(float (&v)[32], int lane) {  // xor distance 2*HALF
  const bool upper = (lane & (2 * HALF)) != 0;
#pragma unroll
  for (int i = 0; i < HALF; ++i) {
    const float keep = upper ? v[i + HALF] : v[i], send = upper ? v[i] : v[i + HALF];
    v[i] = keep + __shfl_xor(send, 2 * HALF, kWave);
  }
}
__device__ __forceinline__ float wave_reduce_32(float (&v)[32]) {
  const int lane = lane_id();
  wave_reduce_step<16>(v, lane);
  wave_reduce_step<8>(v, lane);
  wave_reduce_step<4>(v, lane);
  wave_reduce_step<2>(v, lane);
  wave_reduce_step<1>(v, lane);
  return v[0] + __shfl_xor(v[0], 1, kWave);
}

__global__ __launch_bounds__(kFcThreads) void k_se_fc1(const float* __restrict__ z, int N, int C, int se_w,
                                                       const float* __restrict__ w1, const float* __restrict__ b1,
                                                       float* __restrict__ hid) {
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.y * kFcSamples, k0 = blockIdx.x * kFc1Tile + wave * 4;
  if (k0 >= se_w) return;  // whole wave; the kernel has no barrier
  float acc[4 * kFcSamples];  // [output u][sample g]
#pragma unroll
  for (int i = 0; i < 4 * kFcSamples; ++i) acc[i] = 0.f;
  const int c4n = C / 4;
  for (int c4 = lane; c4 < c4n; c4 += kWave) {
    float4 w[4], zz[kFcSamples];
#pragma unroll
    for (int u = 0; u < 4; ++u) w[u] = reinterpret_cast<const float4*>(w1 + (size_t)min(k0 + u, se_w - 1) * C)[c4];
#pragma unroll
    for (int g = 0; g < kFcSamples; ++g) zz[g] = reinterpret_cast<const float4*>(z + (size_t)min(n0 + g, N - 1) * C)[c4];
#pragma unroll
    for (int g = 0; g < kFcSamples; ++g)
#pragma unroll
      for (int u = 0; u < 4; ++u)
        acc[u * kFcSamples + g] += w[u].x * zz[g].x + w[u].y * zz[g].y + w[u].z * zz[g].z + w[u].w * zz[g].w;
  }
  // even lane l ends up with the sum of (output u, sample g), 8u + g = l / 2: the 32 results leave in one
  // store, and the bias loads of the lanes run side by side instead of one after the other
  const float mine = wave_reduce_32(acc);
  if ((lane & 1) == 0) {
    const int n = n0 + (lane >> 1) % kFcSamples, k = k0 + (lane >> 1) / kFcSamples;
    if (n < N && k < se_w) hid[(size_t)n * se_w + k] = fmaxf(mine + b1[k], 0.f);
  }
}

__global__ __launch_bounds__(kFcThreads) void k_se_fc2(const float* __restrict__ hid, int N, int C, int se_w,
                                                       const float* __restrict__ w2, const float* __restrict__ b2,
                                                       float* __restrict__ gate) {
  __shared__ __align__(16) float s_h[kFcSamples][kSeMaxHidden];
  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int n0 = blockIdx.y * kFcSamples;
  for (int i = tid; i < kFcSamples * se_w; i += kFcThreads) {
    const int g = i / se_w, k = i - g * se_w;
    s_h[g][k] = hid[(size_t)min(n0 + g, N - 1) * se_w + k];
  }
  __syncthreads();
  const bool vec = (se_w % 4) == 0;  // every row of w2 16-byte aligned
  for (int pass = 0; pass < 2; ++pass) {
    const int c0 = blockIdx.x * kFc2Tile + wave * 8 + pass * 4;
    if (c0 >= C) break;
    float acc[4 * kFcSamples];  // [output u][sample g]
#pragma unroll
    for (int i = 0; i < 4 * kFcSamples; ++i) acc[i] = 0.f;
    if (vec) {
      for (int k4 = lane; k4 < se_w / 4; k4 += kWave) {
        float4 w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) w[u] = reinterpret_cast<const float4*>(w2 + (size_t)min(c0 + u, C - 1) * se_w)[k4];
#pragma unroll
        for (int g = 0; g < kFcSamples; ++g) {
          const float4 h = reinterpret_cast<const float4*>(s_h[g])[k4];
#pragma unroll
          for (int u = 0; u < 4; ++u) acc[u * kFcSamples + g] += w[u].x * h.x + w[u].y * h.y + w[u].z * h.z + w[u].w * h.w;
        }
      }
    } else {
      for (int k = lane; k < se_w; k += kWave) {
        float w[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) w[u] = w2[(size_t)min(c0 + u, C - 1) * se_w + k];
#pragma unroll
        for (int g = 0; g < kFcSamples; ++g) {
          const float h = s_h[g][k];
#pragma unroll
          for (int u = 0; u < 4; ++u) acc[u * kFcSamples + g] += w[u] * h;
        }
      }
    }
    const float mine = wave_reduce_32(acc);  // even lane l: (output u, sample g), 8u + g = l / 2
    if ((lane & 1) == 0) {
      const int n = n0 + (lane >> 1) % kFcSamples, c = c0 + (lane >> 1) / kFcSamples;
      if (n < N && c < C) gate[(size_t)n * C + c] = 1.f / (1.f + __expf(-(mine + b2[c])));
    }
  }
}

// h2[row][:] *= gate[sample of the row][:], rounded to the storage type; grid-stride over 16-byte chunks.
template <typename ET>
__global__ __launch_bounds__(256) void k_se_scale(ET* __restrict__ h2, const int32_t* __restrict__ idx,
                                                  const int32_t* __restrict__ count, int pps, int SS, int C,
                                                  const float* __restrict__ gate) {
  constexpr int EPC = elem<ET>::per16;
  const int cpr = C / EPC;
  const long long total = (long long)*count * SS * cpr;
  uint4* base = reinterpret_cast<uint4*>(h2);
  for (long long i = (long long)blockIdx.x * 256 + threadIdx.x; i < total; i += (long long)gridDim.x * 256) {
    const int row = (int)(i / cpr), c = (int)(i - (long long)row * cpr);
    const int n = idx[row / SS] / pps;
    uint4 v = base[i];
    const float4* g4 = reinterpret_cast<const float4*>(gate + (size_t)n * C + c * EPC);
    float g[EPC];
#pragma unroll
    for (int u = 0; u < EPC / 4; ++u) {
      const float4 q = g4[u];
      g[4 * u] = q.x; g[4 * u + 1] = q.y; g[4 * u + 2] = q.z; g[4 * u + 3] = q.w;
    }
    ET t[EPC];
    __builtin_memcpy(t, &v, 16);
#pragma unroll
    for (int e = 0; e < EPC; ++e) elem<ET>::store(&t[e], elem<ET>::load(&t[e]) * g[e]);
    __builtin_memcpy(&v, t, 16);
    base[i] = v;
  }
}

// The SE module on the compact rows h2 [rows][C] of the active patches (pps patches per sample, SS pixels per
// patch, at most cap_rows rows).  `scratch` (float32: means [N][C], gates [N][C], hidden units [N][se_w]) must not
// be in use: the callers pass the h1 region, which is dead once the 3x3 has run.
int launch_se(int dtype, int N, int pps, int SS, int C, const laud_group_se* e, void* h2, const int32_t* idx,
              const int32_t* count, float* scratch, long long cap_rows, hipStream_t st) {
  StageScope scope(LAUD_STAGE_SE, st);
  const int sw = e->se_width;
  float* z = scratch;
  float* gate = z + (size_t)N * C;
  float* hid = gate + (size_t)N * C;
  const int cpr = (int)(C * elem_bytes(dtype) / 16);
  const dim3 sq((unsigned)((cpr + kSqChunks - 1) / kSqChunks), (unsigned)N);
  const unsigned ngrp = (unsigned)((N + kFcSamples - 1) / kFcSamples);
  const dim3 g1((unsigned)((sw + kFc1Tile - 1) / kFc1Tile), ngrp), g2((unsigned)((C + kFc2Tile - 1) / kFc2Tile), ngrp);
  const unsigned sblocks = (unsigned)std::min<long long>((cap_rows * cpr + 1023) / 1024, 8192);
  if (dtype == LAUD_BF16)
    hipLaunchKernelGGL(k_se_squeeze<bf16_t>, sq, dim3(kSqThreads), 0, st, (const bf16_t*)h2, idx, count, pps, SS, C, z);
  else
    hipLaunchKernelGGL(k_se_squeeze<float>, sq, dim3(kSqThreads), 0, st, (const float*)h2, idx, count, pps, SS, C, z);
  hipLaunchKernelGGL(k_se_fc1, g1, dim3(kFcThreads), 0, st, z, N, C, sw, e->w_se1, e->b_se1, hid);
  hipLaunchKernelGGL(k_se_fc2, g2, dim3(kFcThreads), 0, st, hid, N, C, sw, e->w_se2, e->b_se2, gate);
  if (dtype == LAUD_BF16)
    hipLaunchKernelGGL(k_se_scale<bf16_t>, dim3(sblocks), dim3(256), 0, st, (bf16_t*)h2, idx, count, pps, SS, C, gate);
  else
    hipLaunchKernelGGL(k_se_scale<float>, dim3(sblocks), dim3(256), 0, st, (float*)h2, idx, count, pps, SS, C, gate);
  return check_launch();
}

}  // namespace laud
