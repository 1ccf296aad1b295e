// The first 1x1 of the block on EVERY pixel, with the one-channel spatial masker's per-pixel projection taken from the
// same reads of x (Sec. 3.4 "Operator fusion for spatial maskers"; App. B item 1), for gfx950: bf16, c_mid = 256,
// c_in a multiple of 256.  Same construction as the fused conv2 -> conv3 kernel (laud_tail.hip):
//
//   * one workgroup = 64 or 128 pixels x all 256 mid channels, 8 waves; wave w owns channels 32w .. 32w+31 and keeps
//     its weight fragments in registers, streamed from the packed copy of w1 (four K slices held / in flight);
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
constexpr int kMaxPB = 4;                     // a workgroup takes PB = 2 or 4 blocks of 32 pixels
constexpr int kThreads = 512, kWaves = 8;
constexpr int kARing = 4;
constexpr int kWRing = 4;                     // weight slices in registers
constexpr unsigned kOob = 0x80000000u;
constexpr int kMaxK = 4096;
__host__ __device__ constexpr int a_stage(int pb) { return 32 * pb * 128; }  // one 128-byte K slice of every pixel row
// behind the activation ring: s1, t1 [256] floats, masker weights [K] floats, partial sums [8][32*pb], then the
// output rows of the tile (int)
__host__ __device__ constexpr int tab_off(int pb) { return kARing * a_stage(pb); }
__host__ __device__ constexpr int lds_bytes(int K, int pb) { return tab_off(pb) + 2 * kMid * 4 + K * 4 + kWaves * 32 * pb * 4 + 32 * pb * 4; }
// time of one tile of 64 / 128 pixels in the same unit (measured 14-17 and 21-26 us at K = 1024): a workgroup streams
// all of w1 whatever its height
constexpr int kCost2 = 2, kCost4 = 3;
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

// One tile of 32*PB rows: rows row0 .. of the dense map, or (listed) of a pixel list with M entries whose entries for
// this lane's rows (row0 + 64i + 8*wave + lane/8) the caller has already requested.
template <bool PROJ, int PB>
__device__ __forceinline__ void head_tile(const HeadArgs& a, const int row0, const int M, const bool listed,
                                          const int (&pixsp)[PB / 2]) {
  using namespace head;
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int kBM = 32 * PB, kAStage = a_stage(PB), kTabOff = tab_off(PB);
  constexpr int kAI = PB / 2;  // LDS-direct instructions per wave and activation slice (8 rows each)
  static_assert(PB % 2 == 0, "an activation instruction of all eight waves covers 64 rows");
  float* const s_s1 = reinterpret_cast<float*>(smem + kTabOff);
  float* const s_t1 = s_s1 + kMid;
  float* const s_wm = s_t1 + kMid;
  float* const s_part = s_wm + a.K;
  int* const s_orow = reinterpret_cast<int*>(s_part + kWaves * kBM);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l31 = lane & 31, lhi = lane >> 5, l8 = lane >> 3, l7 = lane & 7;
  const int K = a.K, NSL = K / 64;
  // Channel skipping (dense rows only): the mask multiplies the 3x3's input, so h1 is stored as zero in the groups a
  // row's sample drops.  Bit t: the row of pixel block t this lane stores keeps the group of this wave's 32 channels.
  unsigned hkeep = ~0u;
  if (a.rbits != nullptr && !listed) {
    hkeep = 0;
#pragma unroll
    for (int t = 0; t < PB; ++t) {
      const int n = min(row0 + 32 * t + l31, M - 1) / a.hw;
      hkeep |= (((unsigned)a.rbits[n] >> ((wave * 32) / a.cs_group)) & 1u) << t;
    }
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
    const int pixel = rho < M ? (listed ? pixsp[i] : rho) : -1;
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
  f32x16 acc[PB];
  float psum[PB];
#pragma unroll
  for (int t = 0; t < PB; ++t) {
    psum[t] = 0.f;
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
  }
  uint4 fa[2][PB];
  auto read_frags = [&](int buf, int s, int kg) __attribute__((always_inline)) {
    const unsigned char* pa = smem + (unsigned)(s & (kARing - 1)) * kAStage + swz[kg];
#pragma unroll
    for (int t = 0; t < PB; ++t) fa[buf][t] = *reinterpret_cast<const uint4*>(pa + t * 4096);
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
      for (int t = 0; t < PB; ++t) acc[t] = mma_bf16(wr[g / 4][kg], fa[g & 1][t], acc[t]);
      if constexpr (PROJ) {
        // this wave's share of the masker projection: K steps q with q % 8 == wave (s0 is a multiple of 4)
        if ((g & 7) == wave) {
          const float4 w0 = *reinterpret_cast<const float4*>(s_wm + s * 64 + kg * 16 + lhi * 8);
          const float4 w1 = *reinterpret_cast<const float4*>(s_wm + s * 64 + kg * 16 + lhi * 8 + 4);
#pragma unroll
          for (int t = 0; t < PB; ++t) {
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
    for (int t = 0; t < PB; ++t) {
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
      const int pixel = s_orow[32 * t + l31];
      if (!((hkeep >> t) & 1u)) {  // channel skipping: the row's sample drops the group of this wave's channels
#pragma unroll
        for (int e = 0; e < 16; ++e) v[e] = 0.f;
      }
      to_consecutive_channels(v);
      const uint4 c0 = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[8], v[9]), pack_bf16(v[10], v[11]));
      const uint4 c1 = make_uint4(pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]), pack_bf16(v[12], v[13]), pack_bf16(v[14], v[15]));
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
    for (int t = 0; t < PB; ++t) {
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

// The tile height: dense rows are known on the host (a.pb set); for pixel lists the counts live on the device, and
// every workgroup takes the same decision from them -- the height with the smaller (rounds of workgroups over the
// compute units) x (time of one tile), as in the fused conv2 -> conv3 kernel.
template <bool PROJ>
__global__ __launch_bounds__(head::kThreads) void k_head(const HeadArgs a) {
  using namespace head;
  int pb = a.pb;
  const int lane = threadIdx.x & 63, wv = threadIdx.x >> 6, l8 = lane >> 3;
  if (a.slist != nullptr) {
    // Rows = the pixels of the kept samples, in list order: row -> (slot = row / hw, pixel of sample slist[slot]).  The
    // count lives on the device, so the height is decided here (as for pixel lists), and the sample ids of this lane's
    // rows are requested for both candidate heights together with the count.
    const int r8 = 8 * wv + l8;
    auto pix_of = [&](int row) __attribute__((always_inline)) {
      const int slot = row / a.hw;
      return a.slist[min(slot, a.scap - 1)] * a.hw + (row - slot * a.hw);
    };
    const int p2[1] = {pix_of((int)blockIdx.x * 64 + r8)};
    const int p4[2] = {pix_of((int)blockIdx.x * 128 + r8), pix_of((int)blockIdx.x * 128 + 64 + r8)};
    const int M = *a.scount * a.hw;
    if (pb == 0) {
      const int t2 = (M + 63) >> 6, t4 = (M + 127) >> 7;
      const int c2 = ((t2 + a.wg_target - 1) / a.wg_target) * kCost2, c4 = ((t4 + a.wg_target - 1) / a.wg_target) * kCost4;
      pb = c2 <= c4 ? 2 : 4;
    }
    const int row0 = blockIdx.x * 32 * pb;
    if (row0 >= M) return;
    if (pb == 2) head_tile<PROJ, 2>(a, row0, M, true, p2);
    else head_tile<PROJ, 4>(a, row0, M, true, p4);
    return;
  }
  if (a.list == nullptr) {
    const int row0 = blockIdx.x * 32 * pb;
    if (row0 >= a.m_rows) return;
    const int none2[1] = {0}, none4[2] = {0, 0};
    if (pb == 2) head_tile<PROJ, 2>(a, row0, a.m_rows, false, none2);
    else head_tile<PROJ, 4>(a, row0, a.m_rows, false, none4);
    return;
  }
  if constexpr (!PROJ) {
    // Pixel lists per group of samples: a.m_rows groups of up to a.group_rows entries.  Workgroup id -> (group =
    // id % groups, tile = id / groups): consecutive ids (which go round-robin over the XCDs) cycle through the groups
    // at equal tile index, so the tiles that exist come first and evenly spread, the idle workgroups last.  Group
    // and tile do not depend on the counts, so the list entries of both candidate heights are requested together
    // with the counts: one memory round trip before the rows themselves.
    const int g = blockIdx.x % a.m_rows, tile = blockIdx.x / a.m_rows;
    const int32_t* const listp = a.list + (size_t)g * a.group_rows;
    const int cap = a.group_rows - 1;
    const int r8 = 8 * wv + l8;
    int p2[1], p4[2];
    p2[0] = listp[min(tile * 64 + r8, cap)];
    p4[0] = listp[min(tile * 128 + r8, cap)];
    p4[1] = listp[min(tile * 128 + 64 + r8, cap)];
    const int M = a.counts[g];
    if (pb == 0) {
      // the height with the smaller (rounds of workgroups over the compute units) x (time of one tile); the counts
      // are read one per lane and summed across the wave (every wave does the same)
      int t2 = 0, t4 = 0;
      for (int g0 = 0; g0 < a.m_rows; g0 += kWave) {
        const int c = g0 + lane < a.m_rows ? a.counts[g0 + lane] : 0;
        int v2 = (c + 63) >> 6, v4 = (c + 127) >> 7;
#pragma unroll
        for (int d = 32; d > 0; d >>= 1) { v2 += __shfl_xor(v2, d, kWave); v4 += __shfl_xor(v4, d, kWave); }
        t2 += v2;
        t4 += v4;
      }
      const int c2 = ((t2 + a.wg_target - 1) / a.wg_target) * kCost2, c4 = ((t4 + a.wg_target - 1) / a.wg_target) * kCost4;
      pb = c2 <= c4 ? 2 : 4;
    }
    const int row0 = tile * 32 * pb;
    if (row0 >= M) return;
    if (pb == 2) head_tile<false, 2>(a, row0, M, true, p2);
    else head_tile<false, 4>(a, row0, M, true, p4);
  }
}

// ---- host side -----------------------------------------------------------------------------------------------------
bool head_supported(int dtype, int c_in, int c_mid) {
  return dtype == LAUD_BF16 && c_mid == head::kMid && c_in % 256 == 0 && c_in <= head::kMaxK;
}
size_t head_packed_bytes(int c_in) { return align_up((size_t)(c_in / 64) * tail::kSliceChunks * 16, 256); }

static int g_head_cus[32];  // compute units of device d (written before the device's bit in launch_head's `done`)

int head_init_device() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) return LAUD_ERR_HIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return LAUD_ERR_HIP;
  g_head_cus[dev] = cus;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_head<true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          head::lds_bytes(head::kMaxK, head::kMaxPB)) != hipSuccess)
    return LAUD_ERR_HIP;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_head<false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          head::lds_bytes(head::kMaxK, head::kMaxPB)) != hipSuccess)
    return LAUD_ERR_HIP;
  return LAUD_OK;
}

int launch_head_pack(const void* w1, int c_in, void* packed, hipStream_t st) {
  const int chunks = (c_in / 64) * tail::kSliceChunks;
  hipLaunchKernelGGL(k_pack_head_weights, dim3((chunks + 255) / 256), dim3(256), 0, st, (const uint4*)w1, c_in, (uint4*)packed);
  return check_launch();
}

int launch_head(const HeadArgs& args, hipStream_t st) {
  static std::atomic<unsigned> done{0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) return LAUD_ERR_HIP;
  const unsigned bit = 1u << dev;
  if (!(done.load(std::memory_order_acquire) & bit)) {
    if (head_init_device() != LAUD_OK) return LAUD_ERR_HIP;
    done.fetch_or(bit, std::memory_order_release);
  }
  HeadArgs a = args;
  a.wg_target = g_head_cus[dev];
  unsigned grid;
  int lds_pb = head::kMaxPB;
  if (a.slist != nullptr) {
    // pixels of listed samples: capacity m_rows = scap * hw rows, the count is on the device
    if (a.pb != 2 && a.pb != 4) a.pb = 0;
    grid = (unsigned)((a.m_rows + (a.pb == 4 ? 127 : 63)) / (a.pb == 4 ? 128 : 64));
  } else if (a.list == nullptr) {
    // dense rows: the count is known here; the same rounds x tile-time cost the kernel uses for lists
    if (a.pb != 2 && a.pb != 4) {
      const long long t2 = (a.m_rows + 63) / 64, t4 = (a.m_rows + 127) / 128;
      const long long c2 = ((t2 + a.wg_target - 1) / a.wg_target) * head::kCost2;
      const long long c4 = ((t4 + a.wg_target - 1) / a.wg_target) * head::kCost4;
      a.pb = c2 <= c4 ? 2 : 4;
    }
    grid = (unsigned)((a.m_rows + 32 * a.pb - 1) / (32 * a.pb));
    lds_pb = a.pb;
  } else {
    // m_rows groups, each with up to group_rows entries: enough workgroups for the smaller tile height
    if (a.pb != 2 && a.pb != 4) a.pb = 0;
    const int h = a.pb ? 32 * a.pb : 64;
    grid = (unsigned)a.m_rows * (unsigned)((a.group_rows + h - 1) / h);
  }
  StageScope scope(LAUD_STAGE_CONV1, st);
  if (a.wmask)
    hipLaunchKernelGGL((k_head<true>), dim3(grid), dim3(head::kThreads), head::lds_bytes(a.K, lds_pb), st, a);
  else
    hipLaunchKernelGGL((k_head<false>), dim3(grid), dim3(head::kThreads), head::lds_bytes(a.K, lds_pb), st, a);
  return check_launch();
}

}  // namespace laud
