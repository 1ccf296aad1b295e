// conv2 (3x3) -> conv3 (1x1) -> residual add of the dynamic bottleneck in ONE kernel for gfx950: the 3x3's
// output tile h2 never leaves the CU (Sec. 3.4 operator fusion; App. B items 2-3: gather inside the 3x3, scatter-add
// in the last 1x1).  bf16 operands, float32 accumulation; c_mid = 256, c_out a multiple of 256.
//
// One workgroup = 32, 64 or 96 active pixels (rows of the compact list: active patch x pixel in patch; the height is
// chosen on the device from the count, see k_tail) x all 256 mid channels, 8 waves (two per SIMD).  Wave w owns mid
// channels 32w .. 32w+31 of the 3x3 and, per 256-wide column tile of the last 1x1, output channels 32w .. 32w+31 of
// that tile, for all pixels of the tile: the weight rows a wave multiplies are the rows it loads itself, so weights
// need no barrier; only the activation slices (loaded cooperatively) do.
//
//   * Operands reach LDS with LDS-direct 16-byte buffer loads (no VGPR staging, no ds_write): a wave instruction
//     drops 64 x 16 bytes = 8 rows of a 128-byte K slice.  Bank conflicts are avoided by an XOR swizzle of the 16-byte
//     chunk position applied on the global side: chunk c of row r lies at position c ^ (r&7) ^ ((r>>3)&1).
//   * Rings: 4 activation stages (4 KB per 32 pixels each), 4 weight stages (32 KB each, in registers).  One barrier
//     per slice, placed in the middle of the slice's MFMAs; fragments of the next K step (also across slices) are
//     read before the current step's MFMAs are issued.
//   * The MFMAs compute the transposed tile (weights as the first operand): a lane then holds, for one pixel,
//     4 x 4 consecutive channels; one v_permlane32_swap per register pair turns that into 16 consecutive channels
//     per lane, so h2 goes to LDS, and the result to memory, in 16-byte pieces without an LDS transpose.
//   * h2 (pixels x 256 bf16) sits behind the activation ring in LDS; the last 1x1 streams w3 through the
//     same weight ring (no barrier at all in that phase), reads the residual 32 bytes per lane and pixel, adds,
//     applies the activation, rounds and stores.
//
// Channel skipping (Fig. 2(c)) rides on the same kernel (template flag CS): the "patches" are whole samples in
// mask-pattern order, the 3x3 leaves out the 64-channel input slices whose group no row of the tile keeps, and h2 is
// stored as zero in the groups a row drops.
//
// Vector-memory counter discipline: the LDS-direct loads are issued from inline assembly, so the compiler does
// not know them.  Every wait for them is an explicit s_waitcnt vmcnt(n), n = number of LOADS this wave issued
// after the ones needed (loads return in order; stores in flight only make such a wait longer, never shorter).
#include "laud_common.h"
#include "laud_tail_pack.h"
#include "laud_tile_util.h"

#include <atomic>
#include <type_traits>

namespace laud {

namespace tail {
// A workgroup takes PB blocks of 32 pixels (PB = 1 .. 3, chosen per launch on the device from the number of active
// pixels, see k_tail); the LDS layout depends on it.
constexpr int kMaxPB = 3;
constexpr int kARing = 4;
constexpr int kWRing = 3;                     // weight slices held / in flight in registers (4 without a channel mask)
constexpr unsigned kOob = 0x80000000u;        // offset outside every descriptor: reads as zero
__host__ __device__ constexpr int a_stage(int pb) { return 32 * pb * 128; }        // one 128-byte K slice of every pixel row
__host__ __device__ constexpr int h2_off(int pb) { return kARing * a_stage(pb); }  // h2 tile: 32*pb pixels x 512 bytes
__host__ __device__ constexpr int tab_off(int pb) { return h2_off(pb) + 32 * pb * kMid * 2; }
// float tables in LDS behind the tiles: s2, t2 [256], then s3, t3 [cout], then the tile's output rows (int)
__host__ __device__ constexpr int lds_bytes(int pb, int cout) { return tab_off(pb) + (2 * kMid + 2 * cout) * 4 + 32 * pb * 4; }
}  // namespace tail

__global__ __launch_bounds__(256) void k_pack_tail_weights(const uint4* __restrict__ w2, const uint4* __restrict__ w3,
                                                           uint4* __restrict__ out, int nslices) {
  const int idx = blockIdx.x * 256 + threadIdx.x;
  if (idx < nslices * tail::kSliceChunks) tail_pack_chunk(idx, w2, w3, out);
}

#ifdef LAUD_TAIL_DBG
__device__ long long g_tail_dbg[1024 * 64];
#define TAIL_STAMP(i) do { if (tid == 0 && blockIdx.x < 1024) g_tail_dbg[blockIdx.x * 64 + (i)] = (long long)__builtin_readcyclecounter(); } while (0)
__device__ long long g_tail_fine[8 * 64];
// fine stamps: every wave of workgroup 0, slot i (0..63)
#define TAIL_FINE(i) do { if (blockIdx.x == 0 && lane == 0) g_tail_fine[wave * 64 + (i)] = (long long)__builtin_readcyclecounter(); } while (0)
#else
#define TAIL_STAMP(i) do { } while (0)
#define TAIL_FINE(i) do { } while (0)
#endif

// One tile: rows row0 .. row0 + 32*PB - 1 of the compact list of active pixels (M rows exist).
template <int NCT, int PB, bool CS>  // NCT column tiles of 256 output channels (cout = 256 * NCT); CS: channel mask
__device__ __forceinline__ void tail_tile(const TailArgs& a, const int row0, const int M) {
  using namespace tail;
  extern __shared__ __align__(16) unsigned char smem[];
  constexpr int COUT = 256 * NCT;
  constexpr int kBM = 32 * PB;
  constexpr int kAStage = a_stage(PB), kAOff = 0, kH2Off = h2_off(PB), kTabOff = tab_off(PB);
  constexpr int kNB = kSl2 + NCT * kKch;  // slices in the weight stream
  // LDS-direct instructions per wave and activation slice: an instruction of all eight waves covers 64 rows; with an
  // odd PB the last one is issued by waves 0-3 only
  constexpr int kAI = (PB + 1) / 2;
  // Two accumulator sets (the epilogue of a column tile behind the next tile's MFMAs) while the registers allow it:
  // three pixel blocks keep one set and run the epilogue after its tile
  constexpr bool DUAL = PB <= 2;
  float* const s_s2 = reinterpret_cast<float*>(smem + kTabOff);
  float* const s_t2 = s_s2 + kMid;
  float* const s_s3 = s_t2 + kMid;
  float* const s_t3 = s_s3 + COUT;
  int* const s_orow = reinterpret_cast<int*>(s_t3 + COUT);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int l31 = lane & 31, lhi = lane >> 5, l8 = lane >> 3, l7 = lane & 7;
  const bool lastA = !(PB & 1) || wave < 4;  // this wave takes part in the last activation instruction of a slice

  TAIL_STAMP(0);
  const int SS = a.S * a.S;
  int qsp[(PB + 1) / 2];
#pragma unroll
  for (int i = 0; i < (PB + 1) / 2; ++i) qsp[i] = a.list[min((row0 + 64 * i + 8 * wave + l8) / SS, a.cap_patches - 1)];
  // ---- channel skipping: which input slices of the 3x3 this tile needs ---------------------------------------------
  // The tile's rows belong to the list entries (samples) row0/SS .. (row0+kBM-1)/SS; a K chunk (64 input channels) is
  // needed if any of them keeps the chunk's group.  n2 = slices of the 3x3 that are multiplied (9 taps x kept
  // chunks, tap-major); position i of that sequence is slice sid(i) of the packed stream, and the stream goes on
  // into the last 1x1 (all of it: h2 is zero where a row drops a group) behind position n2.
  int n2 = kSl2;
  unsigned kcpack = 0xe4u;  // kept K chunks, two bits each (0, 1, 2, 3)
  int nkc = kKch;
  if constexpr (CS) {
    const int e0 = row0 / SS, e1 = min(row0 + kBM - 1, M - 1) / SS;
    unsigned u = 0;
    for (int e = e0; e <= e1; ++e) u |= a.sbits[e];
    kcpack = 0; nkc = 0;
#pragma unroll
    for (int kc = 0; kc < kKch; ++kc)
      if ((u >> ((kc * 64) / a.cs_group)) & 1u) { kcpack |= (unsigned)kc << (2 * nkc); ++nkc; }
    n2 = 9 * nkc;
  }
  auto sid = [&](int i) __attribute__((always_inline)) -> int {  // packed-stream slice at position i
    if constexpr (!CS) return i;
    if (i >= n2) return kSl2 + (i - n2);
    const int tap = i / nkc, j = i - tap * nkc;
    return tap * kKch + (int)((kcpack >> (2 * j)) & 3u);
  };

  // ... and, per pixel block t of this lane's rows, whether the row keeps the group of this wave's 32 channels (bit t)
  unsigned hkeep = ~0u;
  if constexpr (CS) {
    hkeep = 0;
#pragma unroll
    for (int t = 0; t < PB; ++t) {
      const int e = min(row0 + 32 * t + l31, M - 1) / SS;
      hkeep |= (((unsigned)a.sbits[e] >> ((wave * 32) / a.cs_group)) & 1u) << t;
    }
  }

  // ---- weight stream: a ring of slices in registers (one in use, the others in flight) ------------------------------
  typedef const __attribute__((address_space(1))) u32x4* gptr16;
  const gptr16 wsrc = (gptr16)a.wpacked + wave * 256 + lane;
  // Weight slices held / in flight in registers: four (every compute unit streams the same 1.7 MB at once, which keeps
  // the L2 at its bandwidth limit and its latency high: 37.3 against 38.3 us per launch with three); three with a
  // channel mask, whose slice sequences have 9, 18, 27 or 36 entries.
  constexpr int WR = CS ? kWRing : 4;
  static_assert(kSl2 % WR == 0, "the slice groups of the 3x3 must end where the last 1x1 starts");
  u32x4 wr[WR][4];
  auto load_W = [&](int buf, int i) __attribute__((always_inline)) {  // position i of the slice sequence
    const int b = sid(i);
#pragma unroll
    for (int kg = 0; kg < 4; ++kg) wr[buf][kg] = wsrc[(size_t)b * kSliceChunks + kg * 64];
  };
#pragma unroll
  for (int b = 0; b < WR; ++b) load_W(b, b);

  // ---- per-channel affine tables --------------------------------------------------------------------------------
  for (int i = tid; i < kMid; i += kThreads) { s_s2[i] = a.s2[i]; s_t2[i] = a.t2[i]; }
  for (int i = tid; i < COUT; i += kThreads) { s_s3[i] = a.s3[i]; s_t3[i] = a.t3[i]; }

  // ---- activation rows: instruction i of wave w loads rows 64i + 8w .. +7, lane l the chunk position l%8 of row
  // 64i + 8w + l/8; row r keeps chunk c at position c ^ f(r), f(r) = (r&7) ^ ((r>>3)&1) (conflict-free fragment
  // reads; the swizzle is applied on the global side) -----------------------------------------------------------
  const int sy = a.stride;
  const int Hp = a.Ho / a.S, Wp = a.Wo / a.S;
  unsigned voffA[kAI], amask[kAI];
#pragma unroll
  for (int i = 0; i < kAI; ++i) {
    voffA[i] = 0; amask[i] = 0;
    const int r = 64 * i + 8 * wave + l8;
    const int rho = row0 + r;
    if (r >= kBM) continue;
    if (rho < M) {
      const int p = rho / SS, j = rho - p * SS;
      const int q = qsp[i];
      const int n = q / (Hp * Wp), r2 = q - n * (Hp * Wp);
      const int py = r2 / Wp, px = r2 - py * Wp;
      const int yo = py * a.S + j / a.S, xo = px * a.S + j % a.S;
      const int y = yo * sy, x = xo * sy;  // centre of the 3x3 on the input grid
      const unsigned pix = (unsigned)(n * a.H * a.W + y * a.W + x);
      const unsigned c = (unsigned)l7 ^ ((unsigned)(l8 & 7) ^ (wave & 1u));
      voffA[i] = pix * (kMid * 2u) + c * 16u;
      unsigned mk = 0;
#pragma unroll
      for (int t = 0; t < 9; ++t) {
        const int yy = y + t / 3 - 1, xx = x + t % 3 - 1;
        if (yy >= 0 && yy < a.H && xx >= 0 && xx < a.W) mk |= 1u << t;
      }
      amask[i] = mk;
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
  auto issue_A = [&](int s) __attribute__((always_inline)) {  // position s of the slice sequence -> ring stage s % 4
    const int b = s < n2 ? sid(s) : kSl2;
    const int tap = b / kKch, kc = b - tap * kKch;
    const int ky = tap / 3, kx = tap - ky * 3;
    const unsigned soff = (unsigned)((ky * a.W + kx) * kMid + kc * 64) * 2u;
#pragma unroll
    for (int i = 0; i < kAI; ++i) {
      if (i == kAI - 1 && !lastA) break;
      const unsigned v = (tap < 9 && ((amask[i] >> tap) & 1u)) ? voffA[i] : kOob;  // (positions past the 3x3: zeros)
      dma16(h1rs, v, soff, ldsA + (unsigned)(s & (kARing - 1)) * kAStage + i * 8192);
    }
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

  f32x16 acc[PB];
#pragma unroll
  for (int t = 0; t < PB; ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;

  uint4 fa[2][PB];  // activation fragments of the pixel blocks, read one K step ahead of their MFMAs
  auto read_frags2 = [&](int buf, int s, int kg) __attribute__((always_inline)) {
    const unsigned char* pa = smem + kAOff + (unsigned)(s & (kARing - 1)) * kAStage + swz[kg];
#pragma unroll
    for (int t = 0; t < PB; ++t) fa[buf][t] = *reinterpret_cast<const uint4*>(pa + t * 4096);
  };

  // ---- the 3x3 -----------------------------------------------------------------------------------------------
  vm_wait<0>();  // everything issued so far (weights 0-2, activations 0-2 of this wave) has landed
  lds_wait();    // the tables written above
  wg_barrier();  // ... and everybody else's
  TAIL_STAMP(1);
  read_frags2(0, 0, 0);

  // WR slices = 4 WR K steps with static register indices (weight buffer g/4, fragment buffer g%2).
  // One barrier per slice, in its middle: behind it everyone's activations of the next slice have landed and
  // everyone is done with the slice before this one, whose stage is refilled (three slices ahead).
  // Vector-memory operations of a wave in program order, per slice s: A(s+3) x kAI [middle of s], W(s+3) x4 [end
  // of s].  Needed at the barrier of slice s: A(s+1), issued two slices earlier -- W(s+1), A(s+2), W(s+2) are
  // younger: 8 + (this wave's activation instructions per slice) loads.  Activation loads past the last slice are issued all the same (they read as zeros
  // into stages nobody reads any more) so that the count holds to the end.
  auto group2 = [&](int s0) __attribute__((always_inline)) {
#pragma unroll
    for (int g = 0; g < 4 * WR; ++g) {
      const int s = s0 + g / 4, kg = g % 4;
      if (kg == 0) TAIL_STAMP(2 + s);
      if (kg < 3) read_frags2((g + 1) & 1, s, kg + 1);
      else if (s + 1 < n2) read_frags2((g + 1) & 1, s + 1, 0);
      __builtin_amdgcn_sched_barrier(0);  // the next step's fragment reads stay ahead of this step's MFMAs
#pragma unroll
      for (int t = 0; t < PB; ++t) acc[t] = mma_bf16(wr[g / 4][kg], fa[g & 1][t], acc[t]);
      __builtin_amdgcn_sched_barrier(0);
      if (kg == 1) {
        if (lastA) vm_wait<8 + kAI>(); else vm_wait<8 + kAI - 1>();  // own part of the activations of slice s+1
        wg_barrier();        // everyone's; and everyone is done with slice s-1
        issue_A(s + 3);
      }
      if (kg == 3) {
        load_W(g / 4, s + WR);  // (the stream continues into the last 1x1)
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  };
  for (int s = 0; s < n2; s += WR) group2(s);

  // ---- h2 = relu(s2 * acc + t2) -> LDS -------------------------------------------------------------------------
  TAIL_STAMP(38);
  {
    const int cb = wave * 32;
#pragma unroll
    for (int t = 0; t < PB; ++t) {
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
      if constexpr (CS) {  // the mask multiplies the 3x3's output: a row that drops this wave's group stores zeros
        if (!((hkeep >> t) & 1u)) {
#pragma unroll
          for (int e = 0; e < 16; ++e) v[e] = 0.f;
        }
      }
      to_consecutive_channels(v);
      const uint4 c0 = make_uint4(pack_bf16(v[0], v[1]), pack_bf16(v[2], v[3]), pack_bf16(v[8], v[9]), pack_bf16(v[10], v[11]));
      const uint4 c1 = make_uint4(pack_bf16(v[4], v[5]), pack_bf16(v[6], v[7]), pack_bf16(v[12], v[13]), pack_bf16(v[14], v[15]));
      // pixel row r, 512 bytes per row; 16-byte chunk c sits at position c ^ (r & 15)
      const unsigned r = 32u * t + l31;
      const unsigned ch = wave * 4u + lhi * 2u;
      unsigned char* row = smem + kH2Off + r * 512u;
      *reinterpret_cast<uint4*>(row + ((ch ^ (r & 15u)) << 4)) = c0;
      *reinterpret_cast<uint4*>(row + (((ch + 1u) ^ (r & 15u)) << 4)) = c1;
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[t][e] = 0.f;  // the last 1x1 starts from zero
      __builtin_amdgcn_sched_barrier(0);              // one pixel block at a time (register pressure)
    }
  }
  lds_wait();
  wg_barrier();  // h2 complete
  TAIL_STAMP(39);

  // ---- the last 1x1, column tile by column tile: no activation loads, no barriers ------------------------------
  // Two accumulator sets alternate between column tiles: while tile ct is multiplied into one, the other (tile
  // ct-1) goes through its epilogue -- affine, residual add, activation, rounding, store -- in half-block pieces
  // placed behind the MFMAs of tile ct's first K steps, so the vector ALU works in the shadow of the matrix pipe.
  int orow[PB];        // output row of this lane's pixel in block t (row 0 where the pixel does not exist: reads stay
  unsigned exists = 0;  // in range, nothing is stored), and whether it exists
#pragma unroll
  for (int t = 0; t < PB; ++t) {
    const int o = s_orow[32 * t + l31];
    orow[t] = o < 0 ? 0 : o;
    exists |= (o >= 0 ? 1u : 0u) << t;
  }
  const unsigned hrow = kH2Off + (unsigned)l31 * 512u;  // h2 fragment rows: pixel block t at + t * 32 * 512
  const unsigned hx = (unsigned)(l31 & 15);
  auto read_frags3 = [&](int buf, int ks, int kg) __attribute__((always_inline)) {
    const unsigned c = (unsigned)(ks * 8 + 2 * kg) + lhi;
#pragma unroll
    for (int t = 0; t < PB; ++t)
      fa[buf][t] = *reinterpret_cast<const uint4*>(smem + hrow + t * (32 * 512) + ((c ^ hx) << 4));
  };
  const float floor_ = a.relu ? 0.f : -__builtin_inff();  // the activation after the add as one max (NaN passes through)
  const __bf16* const resp = reinterpret_cast<const __bf16*>(a.res);
  __bf16* const outp = reinterpret_cast<__bf16*>(a.out);
  f32x16 acc2[DUAL ? PB : 1];  // the second accumulator set (odd column tiles)
#pragma unroll
  for (int t = 0; t < (DUAL ? PB : 1); ++t)
#pragma unroll
    for (int e = 0; e < 16; ++e) acc2[t][e] = 0.f;
  uint4 res[PB][2];  // residual of the tile whose epilogue is pending: per pixel block, channels 0-7 / 8-15
#pragma unroll
  for (int t = 0; t < PB; ++t) res[t][0] = res[t][1] = make_uint4(0, 0, 0, 0);

  // Half a pixel block of the epilogue of column tile ct: accumulator groups h and h+2 of a lane (channels
  // 8h + 4*(lane/32) .. +3 and 16 + 8h + 4*(lane/32) .. +3) become, after four lane swaps, eight consecutive channels.
  auto epilogue_half = [&](int ct, int t, int h, f32x16& A) __attribute__((always_inline)) {
    const int cb = ct * 256 + wave * 32;
    const float4 sc0 = *reinterpret_cast<const float4*>(s_s3 + cb + 8 * h + 4 * lhi);
    const float4 sh0 = *reinterpret_cast<const float4*>(s_t3 + cb + 8 * h + 4 * lhi);
    const float4 sc1 = *reinterpret_cast<const float4*>(s_s3 + cb + 8 * (h + 2) + 4 * lhi);
    const float4 sh1 = *reinterpret_cast<const float4*>(s_t3 + cb + 8 * (h + 2) + 4 * lhi);
    float v0[4] = {A[4 * h + 0] * sc0.x + sh0.x, A[4 * h + 1] * sc0.y + sh0.y, A[4 * h + 2] * sc0.z + sh0.z,
                   A[4 * h + 3] * sc0.w + sh0.w};
    float v1[4] = {A[4 * h + 8] * sc1.x + sh1.x, A[4 * h + 9] * sc1.y + sh1.y, A[4 * h + 10] * sc1.z + sh1.z,
                   A[4 * h + 11] * sc1.w + sh1.w};
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v0[i]), __float_as_uint(v1[i]), false, false);
      v0[i] = __uint_as_float(r[0]);
      v1[i] = __uint_as_float(r[1]);
      A[4 * h + i] = 0.f;  // the set is free for the tile after next
      A[4 * h + 8 + i] = 0.f;
    }
    const unsigned rv[4] = {res[t][h].x, res[t][h].y, res[t][h].z, res[t][h].w};
    const float x[8] = {v0[0], v0[1], v0[2], v0[3], v1[0], v1[1], v1[2], v1[3]};
    unsigned pk[4];
#pragma unroll
    for (int d = 0; d < 4; ++d) {
      const float lo = fmaxf(x[2 * d] + __uint_as_float(rv[d] << 16), floor_);
      const float hi = fmaxf(x[2 * d + 1] + __uint_as_float(rv[d] & 0xffff0000u), floor_);
      pk[d] = pack_bf16(lo, hi);
    }
    if ((exists >> t) & 1u)
      *reinterpret_cast<uint4*>(outp + (size_t)orow[t] * COUT + cb + lhi * 16 + h * 8) = make_uint4(pk[0], pk[1], pk[2], pk[3]);
  };
  // The 32 bytes of residual a lane needs for half a pixel block of column tile ct
  auto load_residual_half = [&](int ct, int t, int h) __attribute__((always_inline)) {
    res[t][h] = *reinterpret_cast<const uint4*>(resp + (size_t)orow[t] * COUT + ct * 256 + wave * 32 + lhi * 16 + h * 8);
  };

  read_frags3(0, 0, 0);
#pragma unroll
  for (int ct = 0; ct < NCT; ++ct) {
#pragma unroll
    for (int st = 0; st < 4 * kKch; ++st) {
      const int ks = st / 4, kg = st % 4;
      const int b = kSl2 + ct * kKch + ks;
      const int BUF = b % WR;
      if (kg == 0) TAIL_STAMP(40 + ct * kKch + ks);
      const int cur = st & 1, nxt = cur ^ 1;
      if (kg < 3) read_frags3(nxt, ks, kg + 1);
      else if (b + 1 < kNB) read_frags3(nxt, (ks + 1) % kKch, 0);
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int t = 0; t < PB; ++t) {
        if (DUAL && (ct & 1)) acc2[t] = mma_bf16(wr[BUF][kg], fa[cur][t], acc2[t]);
        else acc[t] = mma_bf16(wr[BUF][kg], fa[cur][t], acc[t]);
      }
      // Odd steps 1, 3, ...: one half pixel block each.  With two accumulator sets the previous tile's epilogue piece
      // runs behind these MFMAs; the residual registers it frees are refilled at once with this tile's values, a
      // whole tile ahead of their use.
      if ((st & 1) && st / 2 < 2 * PB) {
        const int pi = st / 2, t = pi / 2, h = pi % 2;
        if constexpr (DUAL) {
          if (ct > 0) { if (ct & 1) epilogue_half(ct - 1, t, h, acc[t]); else epilogue_half(ct - 1, t, h, acc2[t]); }
        }
        load_residual_half(ct, t, h);
      }
      // the weight register just used is refilled for one ring length later
      if (b + WR < kNB) wr[BUF][kg] = wsrc[(size_t)(b + WR) * kSliceChunks + kg * 64];
      __builtin_amdgcn_sched_barrier(0);
    }
    if constexpr (!DUAL) {  // one accumulator set: the epilogue follows its tile
#pragma unroll
      for (int pi = 0; pi < 2 * PB; ++pi) {
        epilogue_half(ct, pi / 2, pi % 2, acc[pi / 2]);
        __builtin_amdgcn_sched_barrier(0);
      }
    }
  }
  if constexpr (DUAL) {  // the last tile's epilogue
#pragma unroll
    for (int pi = 0; pi < 2 * PB; ++pi) {
      const int t = pi / 2, h = pi % 2;
      if ((NCT - 1) & 1) epilogue_half(NCT - 1, t, h, acc2[t]); else epilogue_half(NCT - 1, t, h, acc[t]);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  TAIL_STAMP(56);
}

// The tile height is chosen on the device, where the number of active patches is known.  A workgroup streams all
// weights whatever its height, and one workgroup fits a compute unit, so the time of a launch is (rounds of
// workgroups over the compute units) x (time of one tile); tiles of 32 / 64 / 96 pixels take about 3 : 4 : 6 time
// units (measured; a small tile is bound by its weight stream, a large one by LDS fragment reads + MFMAs).  Every
// workgroup evaluates the same three candidates and takes the cheapest: a small active set spreads over the whole
// chip, a large one does not leave a nearly empty last round.
template <int NCT, bool CS>
__global__ __launch_bounds__(tail::kThreads) void k_tail(const TailArgs a) {
  using namespace tail;
  const int SS = a.S * a.S, b32 = blockIdx.x * 32;
  const int M = *a.count * SS;
  const int t32 = (M + 31) >> 5;
  int pb = a.pb;
  if (pb < 1 || pb > kMaxPB) {
    constexpr int kCost[kMaxPB] = {3, 4, 6};
    int best = 0x7fffffff;
    pb = 1;
#pragma unroll
    for (int c = 1; c <= kMaxPB; ++c) {
      const int tiles = (t32 + c - 1) / c;
      const int cost = ((tiles + a.wg_target - 1) / a.wg_target) * kCost[c - 1];
      if (cost < best) { best = cost; pb = c; }
    }
  }
  const int row0 = b32 * pb;
  if (row0 >= M) return;
  switch (pb) {
    case 1: tail_tile<NCT, 1, CS>(a, row0, M); break;
    case 2: tail_tile<NCT, 2, CS>(a, row0, M); break;
    default: tail_tile<NCT, 3, CS>(a, row0, M); break;
  }
}

#ifdef LAUD_TAIL_DBG
}  // namespace laud
extern "C" int laud_tail_fine_read(long long* host) {
  return hipMemcpyFromSymbol(host, HIP_SYMBOL(laud::g_tail_fine), 8 * 64 * 8) == hipSuccess ? 0 : -1;
}
extern "C" int laud_tail_dbg_read(long long* host, int nblocks) {
  return hipMemcpyFromSymbol(host, HIP_SYMBOL(laud::g_tail_dbg), (size_t)nblocks * 64 * 8) == hipSuccess ? 0 : -1;
}
namespace laud {
#endif

// ---- host side ---------------------------------------------------------------------------------------------------
bool tail_supported(int dtype, int c_mid, int c_out) {
  return dtype == LAUD_BF16 && c_mid == tail::kMid && (c_out == 1024);
}
size_t tail_packed_bytes(int c_mid, int c_out) { (void)c_mid; return align_up(tail::packed_bytes(c_out), 256); }

static int g_tail_cus[32];  // compute units of device d (written before the device's bit in launch_tail's `done`)

int tail_init_device() {
  int dev = 0, cus = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) return LAUD_ERR_HIP;
  if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) return LAUD_ERR_HIP;
  g_tail_cus[dev] = cus;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tail<4, false>), hipFuncAttributeMaxDynamicSharedMemorySize,
                          tail::lds_bytes(tail::kMaxPB, 1024)) != hipSuccess)
    return LAUD_ERR_HIP;
  return hipFuncSetAttribute(reinterpret_cast<const void*>(&k_tail<4, true>), hipFuncAttributeMaxDynamicSharedMemorySize,
                             tail::lds_bytes(tail::kMaxPB, 1024)) == hipSuccess ? LAUD_OK : LAUD_ERR_HIP;
}

int launch_tail_pack(const void* w2, const void* w3, int c_out, void* packed, hipStream_t st) {
  const int nslices = tail::packed_slices(c_out);
  const int chunks = nslices * tail::kSliceChunks;
  hipLaunchKernelGGL(k_pack_tail_weights, dim3((chunks + 255) / 256), dim3(256), 0, st, (const uint4*)w2, (const uint4*)w3,
                     (uint4*)packed, nslices);
  return check_launch();
}

int launch_tail(const TailArgs& args, long long cap_rows, hipStream_t st) {
  static std::atomic<unsigned> done{0};
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 32) return LAUD_ERR_HIP;
  const unsigned bit = 1u << dev;
  if (!(done.load(std::memory_order_acquire) & bit)) {
    if (tail_init_device() != LAUD_OK) return LAUD_ERR_HIP;
    done.fetch_or(bit, std::memory_order_release);
  }
  TailArgs a = args;
  a.wg_target = g_tail_cus[dev];
  // one workgroup per 32 rows of the capacity: enough for the smallest tile height; workgroups past the last tile
  // of the height chosen on the device leave at once
  const unsigned grid = (unsigned)((cap_rows + 31) / 32);
  StageScope scope(LAUD_STAGE_CONV2, st);
  if (a.sbits)
    hipLaunchKernelGGL((k_tail<4, true>), dim3(grid), dim3(tail::kThreads), tail::lds_bytes(tail::kMaxPB, 1024), st, a);
  else
    hipLaunchKernelGGL((k_tail<4, false>), dim3(grid), dim3(tail::kThreads), tail::lds_bytes(tail::kMaxPB, 1024), st, a);
  return check_launch();
}

}  // namespace laud
