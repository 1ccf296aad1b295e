// The first 1x1 of the block on EVERY pixel, with the one-channel spatial masker's per-pixel projection taken from the
// same reads of x (Sec. 3.4 "Operator fusion for spatial maskers"; App. B item 1), for gfx950: bf16, c_mid = 256,
// c_in a multiple of 256.  Same construction as the fused conv2 -> conv3 kernel (laud_tail.hip):
//
//   * one workgroup = 128 pixels x all 256 mid channels, 8 waves; wave w owns channels 32w .. 32w+31 and keeps its
//     weight fragments in registers, streamed from the packed copy of w1 (four K slices held / in flight);
//   * x reaches LDS with LDS-direct 16-byte loads into a four-stage ring of 128-byte K slices, swizzled on the
//     global side; one barrier per slice, in its middle; fragments are read one K step ahead of their MFMAs;
//   * the MFMAs compute the transposed tile, so after one lane swap per register pair a lane holds 16 consecutive
//     channels of a pixel: h1 = relu(s1 * acc + t1) leaves in 32-byte pieces, without an LDS transpose;
//   * the masker projection sum_c w[c] * x[pixel][c] is formed on the vector ALU from the activation fragments the
//     waves hold anyway: K step q of the tile is taken by wave q % 8, partial sums meet in LDS at the end.
#include "laud_common.h"
#include "laud_tail_pack.h"
#include "laud_tile_util.h"

#include <atomic>

namespace laud {

namespace head {
constexpr int kMid = 256;
constexpr int kPB = 4;                        // 32-pixel blocks per workgroup (and per wave)
constexpr int kBM = 32 * kPB;
constexpr int kThreads = 512, kWaves = 8;
constexpr int kAStage = kBM * 128;            // one 128-byte K slice of every pixel row (16 KB)
constexpr int kARing = 4;
constexpr int kWRing = 4;                     // weight slices in registers
constexpr int kAI = kPB / 2;                  // LDS-direct instructions per wave and activation slice (8 rows each)
constexpr int kTabOff = kARing * kAStage;     // s1, t1 [256] floats, masker weights [K] floats, partial sums [8][kBM]
constexpr unsigned kOob = 0x80000000u;
constexpr int kMaxK = 4096;
// ... then the output rows of the tile (int)
__host__ __device__ constexpr int lds_bytes(int K) { return kTabOff + 2 * kMid * 4 + K * 4 + kWaves * kBM * 4 + kBM * 4; }
}  // namespace head

// w1 [256][K] in MFMA fragment order: slice b (K chunk of 64), wave w, K step kg, lane l hold the 16 bytes
// W1[channel 32w + l%32][k = 64b + 16kg + 8*(l/32) .. +7].
__device__ __forceinline__ void head_pack_chunk(int idx, const uint4* __restrict__ w1, int K, uint4* __restrict__ out) {
  const int l = idx & 63, kg = (idx >> 6) & 3, w = (idx >> 8) & 7, b = idx >> 11;
  const int ch = 32 * w + (l & 31), k = 64 * b + kg * 16 + (l >> 5) * 8;
  out[idx] = w1[((size_t)ch * K + k) / 8];
}
__global__ __launch_bounds__(256) void k_pack_head_weights(const uint4* __restrict__ w1, int K, uint4* __restrict__ out) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx < (K / 64) * tail::kSliceChunks) head_pack_chunk(idx, w1, K, out);
}

template <bool PROJ>
__global__ __launch_bounds__(head::kThreads) void k_head(const HeadArgs a) {
  using namespace head;
  extern __shared__ __align__(16) unsigned char smem[];
  float* const s_s1 = reinterpret_cast<float*>(smem + kTabOff);
  float* const s_t1 = s_s1 + kMid;
  float* const s_wm = s_t1 + kMid;
  float* const s_part = s_wm + a.K;
  int* const s_orow = reinterpret_cast<int*>(s_part + kWaves * kBM);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l31 = lane & 31, lhi = lane >> 5, l8 = lane >> 3, l7 = lane & 7;
  const int K = a.K, NSL = K / 64;
  // dense: workgroup b takes rows 128b ..; sparse: the pixel lists are kept per group of samples, workgroup b takes
  // tile b % tiles_per_group of group b / tiles_per_group (list entries requested together with the group's count)
  int row0 = blockIdx.x * kBM, M = a.m_rows;
  const int32_t* listp = nullptr;
  int pixsp[kAI];
  if (a.list != nullptr) {
    const int g = blockIdx.x / a.tiles_per_group;
    row0 = (blockIdx.x - g * a.tiles_per_group) * kBM;
    listp = a.list + (size_t)g * a.group_rows;
#pragma unroll
    for (int i = 0; i < kAI; ++i) pixsp[i] = listp[min(row0 + 64 * i + 8 * wave + l8, a.group_rows - 1)];
    M = a.counts[g];
    if (row0 >= M) return;
  }

  // ---- weight stream: four slices in registers -------------------------------------------------------------------
  typedef const __attribute__((address_space(1))) u32x4* gptr16;
  const gptr16 wsrc = (gptr16)a.wpacked + wave * 256 + lane;
  u32x4 wr[kWRing][4];
  auto load_W = [&](int buf, int b) __attribute__((always_inline)) {
    const int bb = b < NSL ? b : NSL - 1;  // past the end: the last slice again (keeps the load count uniform)
#pragma unroll
    for (int kg = 0; kg < 4; ++kg) wr[buf][kg] = wsrc[(size_t)bb * tail::kSliceChunks + kg * 64];
  };
#pragma unroll
  for (int b = 0; b < kWRing; ++b) load_W(b, b);

  for (int i = tid; i < kMid; i += kThreads) { s_s1[i] = a.s1[i]; s_t1[i] = a.t1[i]; }
  if constexpr (PROJ)
    for (int i = tid; i < K; i += kThreads) s_wm[i] = a.wmask[i];

  // ---- activation rows: instruction i of wave w loads rows 64i + 8w .. +7; row r keeps chunk c at position
  // c ^ (r&7) ^ ((r>>3)&1) ---------------------------------------------------------------------------------------
  unsigned voffA[kAI];
#pragma unroll
  for (int i = 0; i < kAI; ++i) {
    const int r = 64 * i + 8 * wave + l8;
    const int rho = row0 + r;
    const unsigned c = (unsigned)l7 ^ ((unsigned)(l8 & 7) ^ (wave & 1u));
    const int pixel = rho < M ? (listp ? pixsp[i] : rho) : -1;
    voffA[i] = pixel >= 0 ? (unsigned)pixel * (unsigned)(K * 2) + c * 16u : kOob;
    if (l7 == 0) s_orow[r] = pixel;
  }
  const __amdgpu_buffer_rsrc_t xrs = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.x), 0, (int)kOob, 0x00020000);
  const unsigned ldsA = wave * 1024;
  auto issue_A = [&](int s) __attribute__((always_inline)) {
    const unsigned soff = (unsigned)s * 128u;
#pragma unroll
    for (int i = 0; i < kAI; ++i)
      dma16(xrs, s < NSL ? voffA[i] : kOob, soff, ldsA + (unsigned)(s & (kARing - 1)) * kAStage + i * 8192);
  };
#pragma unroll
  for (int s = 0; s < kARing - 1; ++s) issue_A(s);

  unsigned swz[4];
  {
    const unsigned f = (unsigned)(l31 & 7) ^ ((unsigned)(l31 >> 3) & 1u);
#pragma unroll
    for (int kg = 0; kg < 4; ++kg) swz[kg] = (unsigned)l31 * 128u + (((2u * kg + lhi) ^ f) << 4);
  }
  f32x16 acc[kPB];
  float psum[kPB];
#pragma unroll
  for (int t = 0; t < kPB; ++t) {
    psum[t] = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  }
  uint4 fa[2][kPB];
  auto read_frags = [&](int buf, int s, int kg) __attribute__((always_inline)) {
    const unsigned char* pa = smem + (unsigned)(s & (kARing - 1)) * kAStage + swz[kg];
#pragma unroll
    for (int t = 0; t < kPB; ++t) fa[buf][t] = *reinterpret_cast<const uint4*>(pa + t * 4096);
  };

  vm_wait<0>();
  lds_wait();
  wg_barrier();
  read_frags(0, 0, 0);

  // Four slices = sixteen K steps with static register indices.  Vector-memory operations of a wave in program
  // order, per slice s: A(s+R-1) x kAI [middle of s], W(s+4) x4 [end of s], R = kARing.  Needed at the barrier of
  // slice s: A(s+1), issued R-2 slices earlier -- R-2 weight slices and R-3 activation slices are younger.  Loads
  // past the last slice are issued all the same so that the count holds to the end.  (A deeper ring, R = 8, measured
  // slower: 27.8 against 25.4 us at 128 x 14 x 14 x 1024.)
  for (int s0 = 0; s0 < NSL; s0 += 4) {
#pragma unroll
    for (int g = 0; g < 16; ++g) {
      const int s = s0 + g / 4, kg = g % 4;
      if (kg < 3) read_frags((g + 1) & 1, s, kg + 1);
      else if (s + 1 < NSL) read_frags((g + 1) & 1, s + 1, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int t = 0; t < kPB; ++t) acc[t] = mma_bf16(wr[g / 4][kg], fa[g & 1][t], acc[t]);
      if constexpr (PROJ) {
        // this wave's share of the masker projection: K steps q with q % 8 == wave (s0 is a multiple of 4)
        if ((g & 7) == wave) {
          const float4 w0 = *reinterpret_cast<const float4*>(s_wm + s * 64 + kg * 16 + lhi * 8);
          const float4 w1 = *reinterpret_cast<const float4*>(s_wm + s * 64 + kg * 16 + lhi * 8 + 4);
#pragma unroll
          for (int t = 0; t < kPB; ++t) {
            const uint4 v = fa[g & 1][t];
            float p = psum[t];
            p += __uint_as_float(v.x << 16) * w0.x; p += __uint_as_float(v.x & 0xffff0000u) * w0.y;
            p += __uint_as_float(v.y << 16) * w0.z; p += __uint_as_float(v.y & 0xffff0000u) * w0.w;
            p += __uint_as_float(v.z << 16) * w1.x; p += __uint_as_float(v.z & 0xffff0000u) * w1.y;
            p += __uint_as_float(v.w << 16) * w1.z; p += __uint_as_float(v.w & 0xffff0000u) * w1.w;
            psum[t] = p;
          }
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if (kg == 1) {
        vm_wait<4 * (kARing - 2) + (kARing - 3) * kAI>();
        wg_barrier();
        issue_A(s + kARing - 1);
      }
      if (kg == 3) {
        load_W(g / 4, s + kWRing);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }

  // ---- h1 = relu(s1 * acc + t1), 32 bytes per lane and pixel ------------------------------------------------------
  {
    const int cb = wave * 32;
    __bf16* const outp = reinterpret_cast<__bf16*>(a.h1);
#pragma unroll
    for (int t = 0; t < kPB; ++t) {
      float v[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 sc = *reinterpret_cast<const float4*>(s_s1 + cb + 8 * g + 4 * lhi);
        const float4 sh = *reinterpret_cast<const float4*>(s_t1 + cb + 8 * g + 4 * lhi);
        v[4 * g + 0] = fmaxf(acc[t][4 * g + 0] * sc.x + sh.x, 0.f);
        v[4 * g + 1] = fmaxf(acc[t][4 * g + 1] * sc.y + sh.y, 0.f);
        v[4 * g + 2] = fmaxf(acc[t][4 * g + 2] * sc.z + sh.z, 0.f);
        v[4 * g + 3] = fmaxf(acc[t][4 * g + 3] * sc.w + sh.w, 0.f);
      }
      to_consecutive_channels(v);
      const uint4 c0 = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[8], v[9]), pack_bf16(v[10], v[11]));
      const uint4 c1 = make_uint4(pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]), pack_bf16(v[12], v[13]), pack_bf16(v[14], v[15]));
      const int pixel = s_orow[32 * t + l31];
      if (pixel >= 0) {
        uint4* dst = reinterpret_cast<uint4*>(outp + (size_t)pixel * kMid + cb + lhi * 16);
        dst[0] = c0;
        dst[1] = c1;
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  // ---- projection: the two K halves of a pixel sit in lanes l and l+32; then the eight waves' shares -------------
  if constexpr (PROJ) {
#pragma unroll
    for (int t = 0; t < kPB; ++t) {
      const float other = __shfl_xor(psum[t], 32, kWave);
      if (lhi == 0) s_part[wave * kBM + 32 * t + l31] = psum[t] + other;
    }
    lds_wait();
    wg_barrier();
    if (tid < kBM && s_orow[tid] >= 0) {
      float p = 0.f;
#pragma unroll
      for (int w = 0; w < kWaves; ++w) p += s_part[w * kBM + tid];
      a.proj[s_orow[tid]] = p;
    }
  }
}

// ---- host side -----------------------------------------------------------------------------------------------------
bool head_supported(int dtype, int c_in, int c_mid) {
  return dtype == LAUD_BF16 && c_mid == head::kMid && c_in % 256 == 0 && c_in <= head::kMaxK;
}
size_t head_packed_bytes(int c_in) { return align_up((size_t)(c_in / 64) * tail::kSliceChunks * 16, 256); }

int head_init_device() {
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_head<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          head::lds_bytes(head::kMaxK)) != hipSuccess)
    return LAUD_ERR_HIP;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_head<false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          head::lds_bytes(head::kMaxK)) != hipSuccess)
    return LAUD_ERR_HIP;
  return LAUD_OK;
}

int launch_head_pack(const void* w1, int c_in, void* packed, hipStream_t st) {
  const int chunks = (c_in / 64) * tail::kSliceChunks;
  hipLaunchKernelGGL(k_pack_head_weights, dim3((chunks + 255) / 256), dim3(256), 0, st, (const uint4*)w1, c_in, (uint4*)packed);
  return check_launch();
}

int launch_head(const HeadArgs& a, hipStream_t st) {
  static std::atomic<unsigned> done{0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return LAUD_ERR_HIP;
  const unsigned bit = dev >= 0 && dev < 32 ? 1u << dev : 0u;
  if (!(bit && (done.load(std::memory_order_acquire) & bit))) {
    if (head_init_device() != LAUD_OK) return LAUD_ERR_HIP;
    done.fetch_or(bit, std::memory_order_release);
  }
  // dense: m_rows rows; sparse: m_rows = number of groups, each with tiles_per_group tiles
  const unsigned grid = a.list ? (unsigned)(a.m_rows * a.tiles_per_group) : (unsigned)((a.m_rows + head::kBM - 1) / head::kBM);
  StageScope scope(LAUD_STAGE_CONV1, st);
  if (a.wmask)
    hipLaunchKernelGGL((k_head<true>), dim3(grid), dim3(head::kThreads), head::lds_bytes(a.K), st, a);
  else
    hipLaunchKernelGGL((k_head<false>), dim3(grid), dim3(head::kThreads), head::lds_bytes(a.K), st, a);
  return check_launch();
}

}  // namespace laud
