// conv2 (3x3) -> conv3 (1x1) -> residual add of the dynamic bottleneck in ONE kernel for gfx950: the 3x3's
// output tile h2 never leaves the CU (Sec. 3.4 operator fusion; App. B items 2-3: gather inside the 3x3, scatter-add
// in the last 1x1).  bf16 operands, float32 accumulation; c_mid = 256, c_out a multiple of 256.
//
// One workgroup = 64 active pixels (rows of the compact list: active patch x pixel in patch) x all 256 mid channels,
// 8 waves (two per SIMD).  Wave w owns mid channels 32w .. 32w+31 of the 3x3 and, per 256-wide column tile of the
// last 1x1, output channels 32w .. 32w+31 of that tile, for all 64 pixels: the weight rows a wave multiplies are the
// rows it loads itself, so weights need no barrier; only the activation slices (loaded cooperatively) do.
//
//   * Operands reach LDS with LDS-direct 16-byte buffer loads (no VGPR staging, no ds_write): a wave instruction
//     drops 64 x 16 bytes = 8 rows of a 128-byte K slice.  Bank conflicts are avoided by an XOR swizzle of the 16-byte
//     chunk position applied on the global side: chunk c of row r lies at position c ^ (r&7) ^ ((r>>3)&1).
//   * Rings: 4 activation stages (8 KB each), 3 weight stages (32 KB each).  One barrier per slice, placed in the
//     middle of the slice's MFMAs; fragments of the next K step (also across slices) are read before the current
//     step's MFMAs are issued.
//   * The MFMAs compute the transposed tile (weights as the first operand): a lane then holds, for one pixel,
//     4 x 4 consecutive channels; one v_permlane32_swap per register pair turns that into 16 consecutive channels
//     per lane, so h2 goes to LDS, and the result to memory, in 16-byte pieces without an LDS transpose.
//   * h2 (64 x 256 bf16) overlays the activation ring once the 3x3 is done; the last 1x1 streams w3 through the
//     same weight ring (no barrier at all in that phase), reads the residual 32 bytes per lane and pixel, adds,
//     applies the activation, rounds and stores.
//
// Vector-memory counter discipline: the LDS-direct loads are issued from inline assembly, so the compiler does
// not know them.  Every wait for them is an explicit s_waitcnt vmcnt(n), n = number of LOADS this wave issued
// after the ones needed (loads return in order; stores in flight only make such a wait longer, never shorter).
#include "laud_common.h"

#include <atomic>
#include <type_traits>

namespace laud {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

namespace tail {
constexpr int kMid = 256;
constexpr int kBM = 64;                       // pixels per workgroup
constexpr int kWaves = 8, kThreads = 512;
constexpr int kAStage = kBM * 128;            // 8 KB: 64 rows x one 128-byte K slice
constexpr int kBStage = kMid * 128;           // 32 KB: 256 weight rows x one K slice
constexpr int kARing = 4, kBRing = 3;
constexpr int kBOff = 0;                      // weight ring
constexpr int kAOff = kBRing * kBStage;       // activation ring, later the h2 tile (64 x 512 bytes)
constexpr int kTabOff = kAOff + kARing * kAStage;
constexpr int kKch = kMid / 64;               // K slices per tap (3x3) and per column tile (1x1)
constexpr int kSl2 = 9 * kKch;                // slices of the 3x3
constexpr unsigned kOob = 0x80000000u;        // offset outside every descriptor: reads as zero
// float tables in LDS behind the rings: s2, t2 [256], then s3, t3 [cout], then 64 output rows (int)
// ... then 1 KB that the L2 warm-up loads land in (never read)
__host__ __device__ constexpr int lds_bytes(int cout) { return kTabOff + (2 * kMid + 2 * cout) * 4 + kBM * 4 + 1024; }
}  // namespace tail

// LDS-direct load of 16 bytes per lane: lane l's chunk lands at LDS byte address lds_base + 16*l.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}
// 16-byte load into registers the compiler does not track: the caller waits with vm_wait before use.
__device__ __forceinline__ u32x4 load16_untracked(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff) {
  u32x4 v;
  asm volatile("buffer_load_dwordx4 %0, %1, %2, %3 offen" : "=v"(v) : "v"(voff), "s"(rsrc), "s"(soff) : "memory");
  return v;
}
template <int N>
__device__ __forceinline__ void vm_wait() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
// the same wait, tied to registers written by load16_untracked so that their uses stay behind it
template <int N>
__device__ __forceinline__ void vm_wait_regs(u32x4& a, u32x4& b, u32x4& c, u32x4& d) {
  asm volatile("s_waitcnt vmcnt(%4)" : "+v"(a), "+v"(b), "+v"(c), "+v"(d) : "n"(N) : "memory");
}
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }
__device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

__device__ __forceinline__ f32x16 mma_bf16(const uint4& first, const uint4& second, f32x16 acc) {
  return __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, first), __builtin_bit_cast(bf16x8, second),
                                                 acc, 0, 0, 0);
}
__device__ __forceinline__ unsigned pack_bf16(float lo, float hi) {
  const f32x2 v = {lo, hi};
  return __builtin_bit_cast(unsigned, __builtin_convertvector(v, bf16x2));
}

// Accumulator e of a lane belongs to channel 8*(e/4) + 4*(lane/32) + e%4 of the wave's 32.  After these eight
// swaps v[] holds, in the order 0-3, 8-11, 4-7, 12-15, the sixteen consecutive channels 16*(lane/32) .. +15.
__device__ __forceinline__ void to_consecutive_channels(float (&v)[16]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[i]), __float_as_uint(v[8 + i]), false, false);
    v[i] = __uint_as_float(r[0]);
    v[8 + i] = __uint_as_float(r[1]);
    auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(v[4 + i]), __float_as_uint(v[12 + i]), false, false);
    v[4 + i] = __uint_as_float(q[0]);
    v[12 + i] = __uint_as_float(q[1]);
  }
}

#ifdef LAUD_TAIL_DBG
__device__ long long g_tail_dbg[1024 * 64];
#define TAIL_STAMP(i) do { if (tid == 0 && blockIdx.x < 1024) g_tail_dbg[blockIdx.x * 64 + (i)] = (long long)__builtin_readcyclecounter(); } while (0)
#else
#define TAIL_STAMP(i) do { } while (0)
#endif

template <int NCT>  // column tiles of 256 output channels (cout = 256 * NCT)
__global__ __launch_bounds__(tail::kThreads) void k_tail(const TailArgs a) {
  using namespace tail;
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int COUT = 256 * NCT;
  float* const s_s2 = reinterpret_cast<float*>(smem + kTabOff);
  float* const s_t2 = s_s2 + kMid;
  float* const s_s3 = s_t2 + kMid;
  float* const s_t3 = s_s3 + COUT;
  int* const s_orow = reinterpret_cast<int*>(s_t3 + COUT);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l31 = lane & 31, lhi = lane >> 5, l8 = lane >> 3, l7 = lane & 7;

  // ---- which tile: consecutive workgroup ids go round-robin over the 8 XCDs; each XCD takes a contiguous run
  // of row tiles (neighbouring tiles share halo rows of h1 in that XCD's L2) --------------------------------
  TAIL_STAMP(0);
  const int SS = a.S * a.S;
  const int M = *a.count * SS;
  const int ntiles = (M + kBM - 1) / kBM;
  const int tpx = (ntiles + 7) >> 3;
  const int xcd = blockIdx.x & 7, slot = blockIdx.x >> 3;
  const int rt = xcd * tpx + slot;
  if (slot >= tpx || rt >= ntiles) return;
  const int row0 = rt * kBM;

  const __amdgpu_buffer_rsrc_t w2rs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.w2), 0, (int)kOob, 0x00020000);
  const __amdgpu_buffer_rsrc_t w3rs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.w3), 0, (int)kOob, 0x00020000);

  // ---- weight slices: wave w loads (and later multiplies) rows 32w .. 32w+31, four instructions of 8 rows -------
  // row R = 32w + 8i + lane/8 sits at LDS position lane%8 of its row and must hold chunk (lane%8) ^ f(R),
  // f(R) = (R&7) ^ ((R>>3)&1) = (lane/8) ^ (i&1)
  unsigned voffB2[4], voffB3[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const unsigned R = 32u * wave + 8u * i + l8;
    const unsigned c = (unsigned)l7 ^ ((unsigned)l8 ^ (i & 1u));
    voffB2[i] = R * (9u * kMid * 2u) + c * 16u;
    voffB3[i] = R * (kMid * 2u) + c * 16u;
  }
  const unsigned ldsB = kBOff + wave * 4096;  // this wave's 32 rows inside a weight stage
  // b = stream index of a weight slice: 0 .. kSl2-1 the 3x3 (tap-major), then the column tiles of the 1x1
  auto issue_B = [&](int b) __attribute__((always_inline)) {
    const unsigned base = ldsB + (unsigned)(b % kBRing) * kBStage;
    if (b < kSl2) {
      const unsigned soff = (unsigned)((b / kKch) * kMid + (b % kKch) * 64) * 2u;
#pragma unroll
      for (int i = 0; i < 4; ++i) dma16(w2rs, voffB2[i], soff, base + i * 1024);
    } else {
      const int c = b - kSl2;
      const unsigned soff = (unsigned)((c / kKch) * 256 * kMid + (c % kKch) * 64) * 2u;
#pragma unroll
      for (int i = 0; i < 4; ++i) dma16(w3rs, voffB3[i], soff, base + i * 1024);
    }
  };
  issue_B(0);
  issue_B(1);

  // ---- L2 warm-up: every workgroup of an XCD walks w2 and w3 in the same order at the same time, so without help
  // each slice would be fetched into that XCD's L2 at the moment all of them need it, and all of them would wait
  // for memory.  Instead the XCD's workgroups touch one 16-byte piece of every 128-byte line up front, in stream
  // order, sharing the lines among them; the loads land in a spare KB of LDS nobody reads.
  {
    constexpr int kLines2 = kSl2 * kMid;           // w2: per slice one line per row
    constexpr int kLines = kLines2 + COUT * kMid * 2 / 128;
    const unsigned dummy = (unsigned)(kTabOff + (2 * kMid + 2 * COUT) * 4 + kBM * 4);
    int base = __builtin_amdgcn_readfirstlane(slot * kThreads + wave * 64);
    for (int it = 0; it < 8 && base < kLines; ++it, base += tpx * kThreads) {
      const int L = base + lane;
      if (base < kLines2) {
        const unsigned sl = (unsigned)L / kMid, row = (unsigned)L % kMid;
        dma16(w2rs, row * (9u * kMid * 2u) + sl * 128u, 0u, dummy);
      } else {
        dma16(w3rs, (unsigned)(L - kLines2) * 128u, 0u, dummy);
      }
    }
  }

  // ---- per-channel affine tables and output rows -------------------------------------------------------------
  for (int i = tid; i < kMid; i += kThreads) { s_s2[i] = a.s2[i]; s_t2[i] = a.t2[i]; }
  for (int i = tid; i < COUT; i += kThreads) { s_s3[i] = a.s3[i]; s_t3[i] = a.t3[i]; }

  // ---- activation rows: lane loads chunk position lane%8 of row 8w + lane/8 ---------------------------------
  const int sy = a.stride;
  const int Hp = a.Ho / a.S, Wp = a.Wo / a.S;
  unsigned voffA = 0, amask = 0;
  {
    const int r = 8 * wave + l8;
    const int rho = row0 + r;
    if (rho < M) {
      const int p = rho / SS, j = rho - p * SS;
      const int q = a.list[p];
      const int n = q / (Hp * Wp), r2 = q - n * (Hp * Wp);
      const int py = r2 / Wp, px = r2 - py * Wp;
      const int yo = py * a.S + j / a.S, xo = px * a.S + j % a.S;
      const int y = yo * sy, x = xo * sy;  // centre of the 3x3 on the input grid
      const unsigned pix = (unsigned)(n * a.H * a.W + y * a.W + x);
      const unsigned c = (unsigned)l7 ^ ((unsigned)(l8 & 7) ^ (wave & 1u));
      voffA = pix * (kMid * 2u) + c * 16u;
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const int yy = y + t / 3 - 1, xx = x + t % 3 - 1;
        if (yy >= 0 && yy < a.H && xx >= 0 && xx < a.W) amask |= 1u << t;
      }
      if (l7 == 0) s_orow[r] = n * (a.Ho * a.Wo) + yo * a.Wo + xo;
    } else if (l7 == 0) {
      s_orow[r] = -1;
    }
  }
  // taps reach one row and one pixel back: the descriptor starts that far before h1
  const long long ashift = (long long)(a.W + 1) * kMid * 2;
  const __amdgpu_buffer_rsrc_t h1rs = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(reinterpret_cast<const char*>(a.h1)) - ashift, 0, (int)kOob, 0x00020000);
  const unsigned ldsA = kAOff + wave * 1024;
  auto issue_A = [&](int s) __attribute__((always_inline)) {
    const int tap = s / kKch, kc = s - tap * kKch;
    const int ky = tap / 3, kx = tap - ky * 3;
    const unsigned soff = (unsigned)((ky * a.W + kx) * kMid + kc * 64) * 2u;
    const unsigned v = ((amask >> tap) & 1u) ? voffA : kOob;
    dma16(h1rs, v, soff, ldsA + (unsigned)(s & (kARing - 1)) * kAStage);
  };
  issue_A(0);
  issue_A(1);
  issue_A(2);

  // ---- fragment addresses: row lane%32 of a 32-row block, chunk 2*kg + lane/32, swizzled ------------------------
  unsigned swz[4];
  {
    const unsigned f = (unsigned)(l31 & 7) ^ ((unsigned)(l31 >> 3) & 1u);
#pragma unroll
    for (int kg = 0; kg < 4; ++kg) swz[kg] = (unsigned)l31 * 128u + (((2u * kg + lhi) ^ f) << 4);
  }

  f32x16 acc[2];
#pragma unroll
  for (int t = 0; t < 2; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  uint4 fw[2], fa[2][2];  // double-buffered fragments: weights, activations of pixel blocks 0 / 1
  auto read_frags2 = [&](int buf, int s, int kg) __attribute__((always_inline)) {
    const unsigned char* pb = smem + kBOff + (unsigned)(s % kBRing) * kBStage + wave * 4096 + swz[kg];
    const unsigned char* pa = smem + kAOff + (unsigned)(s & (kARing - 1)) * kAStage + swz[kg];
    fw[buf] = *reinterpret_cast<const uint4*>(pb);
    fa[buf][0] = *reinterpret_cast<const uint4*>(pa);
    fa[buf][1] = *reinterpret_cast<const uint4*>(pa + 4096);
  };

  // ---- the 3x3 -----------------------------------------------------------------------------------------------
  // issued so far, in order: B0, B1 (4 loads each), A0, A1, A2 (1 each)
  vm_wait<1>();  // B0, B1, A0, A1 of this wave have landed
  lds_wait();    // the tables written above
  wg_barrier();  // ... and everybody else's; also publishes the tables
  TAIL_STAMP(1);
  read_frags2(0, 0, 0);

  // One slice.  VM_SYNC: loads allowed in flight when the next slice's activations are needed (middle of the
  // slice); VM_B: when the next slice's weights are needed (end of the slice); ISSUE_A / LAST as named.
  auto slice2 = [&](int s, auto vm_sync, auto vm_b, auto issue_a, auto last) __attribute__((always_inline)) {
    TAIL_STAMP(2 + s);
#pragma unroll
    for (int kg = 0; kg < 4; ++kg) {
      const int cur = kg & 1, nxt = cur ^ 1;
      if (kg < 3) {
        read_frags2(nxt, s, kg + 1);
      } else if (!decltype(last)::value) {
        vm_wait<decltype(vm_b)::value>();  // own weights of slice s+1 (activations were covered by the barrier)
        read_frags2(nxt, s + 1, 0);
      }
      __builtin_amdgcn_sched_barrier(0);  // the next step's fragment reads stay ahead of this step's MFMAs
      acc[0] = mma_bf16(fw[cur], fa[cur][0], acc[0]);
      acc[1] = mma_bf16(fw[cur], fa[cur][1], acc[1]);
      __builtin_amdgcn_sched_barrier(0);
      if (kg == 1) {
        if (!decltype(last)::value) {
          vm_wait<decltype(vm_sync)::value>();  // own part of the activations of slice s+1
          wg_barrier();                          // everyone's; and everyone is done with slice s-1
        }
        issue_B(s + 2);
        if (decltype(issue_a)::value) issue_A(s + 3);
      }
    }
  };
  using std::integral_constant;
  typedef integral_constant<bool, true> T_;
  typedef integral_constant<bool, false> F_;
  for (int s = 0; s < kSl2 - 3; ++s) slice2(s, integral_constant<int, 5>{}, integral_constant<int, 6>{}, T_{}, F_{});
  slice2(kSl2 - 3, integral_constant<int, 5>{}, integral_constant<int, 5>{}, F_{}, F_{});
  slice2(kSl2 - 2, integral_constant<int, 4>{}, integral_constant<int, 4>{}, F_{}, F_{});
  slice2(kSl2 - 1, integral_constant<int, 0>{}, integral_constant<int, 0>{}, F_{}, T_{});

  // ---- h2 = relu(s2 * acc + t2) -> LDS over the activation ring ----------------------------------------------
  TAIL_STAMP(38);
  wg_barrier();  // every wave has finished reading the activation ring
  {
    const int cb = wave * 32;
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      float v[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 sc = *reinterpret_cast<const float4*>(s_s2 + cb + 8 * g + 4 * lhi);
        const float4 sh = *reinterpret_cast<const float4*>(s_t2 + cb + 8 * g + 4 * lhi);
        v[4 * g + 0] = fmaxf(acc[t][4 * g + 0] * sc.x + sh.x, 0.f);
        v[4 * g + 1] = fmaxf(acc[t][4 * g + 1] * sc.y + sh.y, 0.f);
        v[4 * g + 2] = fmaxf(acc[t][4 * g + 2] * sc.z + sh.z, 0.f);
        v[4 * g + 3] = fmaxf(acc[t][4 * g + 3] * sc.w + sh.w, 0.f);
      }
      to_consecutive_channels(v);
      const uint4 c0 = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[8], v[9]), pack_bf16(v[10], v[11]));
      const uint4 c1 = make_uint4(pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]), pack_bf16(v[12], v[13]), pack_bf16(v[14], v[15]));
      // pixel row r, 512 bytes per row; 16-byte chunk c sits at position c ^ (r & 15)
      const unsigned r = 32u * t + l31;
      const unsigned ch = wave * 4u + lhi * 2u;
      unsigned char* row = smem + kAOff + r * 512u;
      *reinterpret_cast<uint4*>(row + ((ch ^ (r & 15u)) << 4)) = c0;
      *reinterpret_cast<uint4*>(row + (((ch + 1u) ^ (r & 15u)) << 4)) = c1;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;  // the last 1x1 starts from zero
    }
  }
  lds_wait();
  wg_barrier();  // h2 complete
  TAIL_STAMP(39);

  // ---- the last 1x1, column tile by column tile ------------------------------------------------------------------
  const __amdgpu_buffer_rsrc_t resrs =
      __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(a.res), 0, (int)kOob, 0x00020000);
  const int orow0 = s_orow[l31], orow1 = s_orow[32 + l31];
  const unsigned chan_b = (unsigned)(wave * 32 + lhi * 16) * 2u;  // byte offset of this lane's 16 channels in a tile
  const unsigned voffR0 = orow0 >= 0 ? (unsigned)orow0 * (COUT * 2u) + chan_b : kOob;
  const unsigned voffR1 = orow1 >= 0 ? (unsigned)orow1 * (COUT * 2u) + chan_b : kOob;
  unsigned hswz[2];  // h2 fragment row bases: pixel block t, row lane%32
#pragma unroll
  for (int t = 0; t < 2; ++t) hswz[t] = kAOff + (32u * t + l31) * 512u;
  const unsigned hx = (unsigned)(l31 & 15);
  auto read_frags3 = [&](int buf, int b, int ks, int kg) __attribute__((always_inline)) {
    const unsigned char* pb = smem + kBOff + (unsigned)(b % kBRing) * kBStage + wave * 4096 + swz[kg];
    fw[buf] = *reinterpret_cast<const uint4*>(pb);
    const unsigned c = (unsigned)(ks * 8 + 2 * kg) + lhi;
    fa[buf][0] = *reinterpret_cast<const uint4*>(smem + hswz[0] + ((c ^ hx) << 4));
    fa[buf][1] = *reinterpret_cast<const uint4*>(smem + hswz[1] + ((c ^ hx) << 4));
  };
  constexpr int kNB = kSl2 + NCT * kKch;  // slices in the weight stream
  // in flight here: B(kSl2) (waited for below), B(kSl2+1)
  vm_wait<4>();
  read_frags3(0, kSl2, 0, 0);
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
    u32x4 r00, r01, r10, r11;  // residual: pixel block 0 / 1, channels 0-7 / 8-15 of the lane's sixteen
#pragma unroll
    for (int ks = 0; ks < kKch; ++ks) {
      const int b = kSl2 + ct * kKch + ks;
      TAIL_STAMP(40 + ct * kKch + ks);
#pragma unroll
      for (int kg = 0; kg < 4; ++kg) {
        const int cur = kg & 1, nxt = cur ^ 1;
        if (kg < 3) {
          read_frags3(nxt, b, ks, kg + 1);
        } else if (b + 1 < kNB) {
          // weights of slice b+1; younger loads: B(b+2) if it exists, and the residual if issued in this slice
          constexpr int kRes = 4;
          const bool has2 = b + 2 < kNB;
          if (ks == 0) { if (has2) vm_wait<4 + kRes>(); else vm_wait<kRes>(); }
          else { if (has2) vm_wait<4>(); else vm_wait<0>(); }
          read_frags3(nxt, b + 1, (ks + 1) % kKch, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        acc[0] = mma_bf16(fw[cur], fa[cur][0], acc[0]);
        acc[1] = mma_bf16(fw[cur], fa[cur][1], acc[1]);
        __builtin_amdgcn_sched_barrier(0);
        if (kg == 1) {
          if (ks == 0) {
            const unsigned so = (unsigned)ct * 512u;
            r00 = load16_untracked(resrs, voffR0, so);
            r01 = load16_untracked(resrs, voffR0 + 16u, so);
            r10 = load16_untracked(resrs, voffR1, so);
            r11 = load16_untracked(resrs, voffR1 + 16u, so);
          }
          if (b + 2 < kNB) issue_B(b + 2);
        }
      }
    }
    // epilogue of the column tile: younger loads than the residual = the weight slices issued since (4 each)
    {
      const int left = kNB - (kSl2 + ct * kKch) - 2;                     // weight slices not yet issued when the tile began
      const int after = left < 0 ? 0 : (left < kKch ? left : kKch);     // ... of which this tile issued
      switch (after) {  // (folds to one case once the tile loop is unrolled)
        case 4: vm_wait_regs<16>(r00, r01, r10, r11); break;
        case 3: vm_wait_regs<12>(r00, r01, r10, r11); break;
        case 2: vm_wait_regs<8>(r00, r01, r10, r11); break;
        case 1: vm_wait_regs<4>(r00, r01, r10, r11); break;
        default: vm_wait_regs<0>(r00, r01, r10, r11); break;
      }
    }
    const int cb = ct * 256 + wave * 32;
    __bf16* const outp = reinterpret_cast<__bf16*>(a.out);
#pragma unroll
    for (int t = 0; t < 2; ++t) {
      float v[16];
#pragma unroll
      for (int g = 0; g < 4; ++g) {
        const float4 sc = *reinterpret_cast<const float4*>(s_s3 + cb + 8 * g + 4 * lhi);
        const float4 sh = *reinterpret_cast<const float4*>(s_t3 + cb + 8 * g + 4 * lhi);
        v[4 * g + 0] = acc[t][4 * g + 0] * sc.x + sh.x;
        v[4 * g + 1] = acc[t][4 * g + 1] * sc.y + sh.y;
        v[4 * g + 2] = acc[t][4 * g + 2] * sc.z + sh.z;
        v[4 * g + 3] = acc[t][4 * g + 3] * sc.w + sh.w;
      }
      to_consecutive_channels(v);
      const u32x4 ra = t == 0 ? r00 : r10, rb = t == 0 ? r01 : r11;
      // v order: [0-3]=ch0-3, [8-11]=ch4-7 (chunk a); [4-7]=ch8-11, [12-15]=ch12-15 (chunk b)
      const int o0[4] = {0, 2, 8, 10}, o1[4] = {4, 6, 12, 14};
      unsigned pa[4], pb[4];
#pragma unroll
      for (int d = 0; d < 4; ++d) {
        float x0 = v[o0[d]] + __uint_as_float(ra[d] << 16), x1 = v[o0[d] + 1] + __uint_as_float(ra[d] & 0xffff0000u);
        float y0 = v[o1[d]] + __uint_as_float(rb[d] << 16), y1 = v[o1[d] + 1] + __uint_as_float(rb[d] & 0xffff0000u);
        if (a.relu) { x0 = fmaxf(x0, 0.f); x1 = fmaxf(x1, 0.f); y0 = fmaxf(y0, 0.f); y1 = fmaxf(y1, 0.f); }
        pa[d] = pack_bf16(x0, x1);
        pb[d] = pack_bf16(y0, y1);
      }
      const int orow = t == 0 ? orow0 : orow1;
      if (orow >= 0) {
        uint4* dst = reinterpret_cast<uint4*>(outp + (size_t)orow * COUT + cb + lhi * 16);
        dst[0] = make_uint4(pa[0], pa[1], pa[2], pa[3]);
        dst[1] = make_uint4(pb[0], pb[1], pb[2], pb[3]);
      }
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;
    }
  }
  TAIL_STAMP(56);
}

#ifdef LAUD_TAIL_DBG
}  // namespace laud
extern "C" int laud_tail_dbg_read(long long* host, int nblocks) {
  return hipMemcpyFromSymbol(host, HIP_SYMBOL(laud::g_tail_dbg), (size_t)nblocks * 64 * 8) == hipSuccess ? 0 : -1;
}
namespace laud {
#endif

// ---- host side ---------------------------------------------------------------------------------------------------
bool tail_supported(int dtype, int c_mid, int c_out) {
  return dtype == LAUD_BF16 && c_mid == tail::kMid && (c_out == 1024);
}

int tail_init_device() {
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tail<4>), hipFuncAttributeMaxDynamicSharedMemorySize,
                             tail::lds_bytes(1024)) == hipSuccess ? LAUD_OK : LAUD_ERR_HIP;
}

int launch_tail(const TailArgs& a, long long cap_rows, hipStream_t st) {
  static std::atomic<unsigned> done{0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return LAUD_ERR_HIP;
  const unsigned bit = dev >= 0 && dev < 32 ? 1u << dev : 0u;
  if (!(bit && (done.load(std::memory_order_acquire) & bit))) {
    if (tail_init_device() != LAUD_OK) return LAUD_ERR_HIP;
    done.fetch_or(bit, std::memory_order_release);
  }
  const long long tiles = (cap_rows + tail::kBM - 1) / tail::kBM;
  const unsigned grid = (unsigned)(((tiles + 7) / 8) * 8);
  StageScope scope(LAUD_STAGE_CONV2, st);
  hipLaunchKernelGGL((k_tail<4>), dim3(grid), dim3(tail::kThreads), tail::lds_bytes(1024), st, a);
  return check_launch();
}

}  // namespace laud
