// The three convolutions of the dynamic bottleneck as gathered implicit GEMMs on gfx950 MFMA.
//
// One kernel template, k_gemm<MODE, ET, BM, BN, WGN>, computes a BM x BN output tile with 2 x WGN
// waves of 32x32 MFMA tiles; A (activations) and B (weights, [N][K] K-contiguous) are staged
// through LDS in 128-byte K slices.  What differs per MODE is only where a row of A
// comes from and where a row of the result goes:
//
//   CONV1  rows = pixels of the dilated active set (list of pixel ids): the gather is fused
//          into the first 1x1 (Sec. 3.4 "Fusing gather and dynamic convolution"); result
//          h1 = relu(s1*acc + t1) stored at the pixel's own position.
//   CONV2  rows = (active patch, pixel in patch); the K loop runs over the nine taps, the A row
//          of tap (ky,kx) is h1 at the shifted pixel, or zeros outside the image (App. B item 2:
//          fetch by index, output patches stored densely); result h2 dense, patch-major.
//   CONV3  rows = the dense h2 rows; epilogue reads the residual at the patch's position, adds,
//          and stores at that position (Sec. 3.4 "Fusing scatter and add"; App. B item 3).
//   DENSE1 conv1 on every pixel, with the one-channel masker's per-pixel projection computed from the
//          same A slices (Sec. 3.4 "Operator fusion for spatial maskers"; App. B item 1): x is read
//          once for both.
//   U1..3  the three convs of the UNFUSED three-step schedule (Sec. 3.1: gather, compute, scatter), on
//          the densely gathered halo tiles: U1 = conv1 on all (S+2)^2 positions of every active patch
//          (positions outside the image are written as zeros: the padding is the 3x3's), U2 = 3x3
//          inside the gathered tile, U3 = last 1x1 into a dense buffer (a separate kernel scatters).
//   SD1..3 static dense convs of the always-executed first block of a stage: 1x1 with a spatial stride
//          (SD1: conv1 with stride 1, shortcut with the block's stride), 3x3 with stride (SD2), last
//          1x1 with the shortcut already in the output buffer as residual (SD3).
//   G2     CONV2 as a group convolution (the RegNetY blocks of Sec. 4; Sec. 3.2 on group convolutions):
//          the tile's BN output channels read only the BN input channels of their own groups, so the
//          reduction per tap is that window of channels and the weight tile is block-diagonal -- chunks
//          outside an output channel's group read as zeros, the ones inside come from w2 [m][3][3][g].
//   CS1..3 the same three convs for channel skipping (Fig. 2(c)): one sample per blockIdx.y,
//          output channels / reduction channels gathered through the sample's kept-group list,
//          i.e. the weight gather is fused into the conv (Sec. 3.4).
//
// Accumulation is float32 (bf16: v_mfma_f32_32x32x16_bf16, fp32: v_mfma_f32_32x32x2_f32).
#include "laud_common.h"
#include "laud_tail_pack.h"

#include <algorithm>
#include <atomic>

namespace laud {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));
typedef const __attribute__((address_space(1))) u32x4* gptr16;  // 16-byte chunk in global memory

enum { M_CONV1 = 0, M_CONV2 = 1, M_CONV3 = 2, M_CS1 = 3, M_CS2 = 4, M_CS3 = 5, M_DENSE1 = 6, M_U1 = 7, M_U2 = 8, M_U3 = 9,
       M_SD1 = 10, M_SD2 = 11, M_SD3 = 12, M_G2 = 13 };

// 256 bytes of zeros in device memory: the source of the zero chunks of the pointer-based weight gather
// of channel skipping (every other load gets its zeros from the buffer descriptor's range check).  Not
// declared const on purpose: the compiler must treat a load from it like any other load (it would
// otherwise fold the zeros in and turn the pointer select back into a branch around the load).
__device__ uint4 g_zero_page[16];

constexpr int kMaxGroups = 1024;  // channel-skip decisions per sample the kernels can hold in LDS

struct GemmArgs {
  const void* A;         // activations the rows are gathered from
  const void* Wt;        // weights [Ncols][ldw]
  const float* scale;    // per-output-channel affine
  const float* shift;
  void* Out;
  const void* Res;       // residual (CONV3 / CS3); may alias Out
  const int32_t* count;  // device: number of units (pixels for CONV1, patches for CONV2/3)
  const int32_t* list;   // device: pixel ids (CONV1) or active patch ids (CONV2/3)
  const uint8_t* cmask;  // CS: [N][D]
  int K;                 // reduction length per tap (full width)
  int ldw;               // weight row stride, elements
  int Ncols;             // output channels (full width)
  int H, W, S;
  int lda;               // A row stride, elements
  int ldo;               // Out/Res row stride, elements
  int relu;
  int D, G;              // CS: groups per sample, channels per group
  int row_tiles, col_tiles;
  int group_rows, tiles_per_group;  // CONV1: pixel lists are kept per group of samples
  int m_rows;            // DENSE1, SD1..3: number of rows (all output pixels), known on the host
  int stride, Ho, Wo;    // SD1, SD2: spatial stride and output size (H, W are the input size)
  int gw;                // G2: channels per group of the 3x3
  // Workgroups past the tiles (CONV1 / DENSE1 launches only) copy the block's w2 / w3 into the fused tail kernel's
  // streaming order while the first 1x1 runs; pk_out == null: none.
  const void* pk_w2; const void* pk_w3; void* pk_out; int pk_chunks; int pk_first_block;
  const float* wmask;    // DENSE1: masker weights [K] or null
  float* proj;           // DENSE1: per-pixel masker projection sum_c w[c]*x[pixel][c], [m_rows]
};

// ---- one 16-byte fragment pair -> MFMA ------------------------------------------------------
template <typename ET>
__device__ __forceinline__ void mma16(f32x16& acc, const uint4& a, const uint4& b) {
  if constexpr (sizeof(ET) == 2) {
    acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), acc,
                                                  0, 0, 0);
  } else {
    // Four k-steps of the 32x32x2 fp32 MFMA; lane group l/32 holds k-slots {4h..4h+3} of this
    // 8-wide K group for A and B alike, so the pairing of A and B elements is consistent.
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.x), __uint_as_float(b.x), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.y), __uint_as_float(b.y), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.z), __uint_as_float(b.z), acc, 0, 0, 0);
    acc = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(a.w), __uint_as_float(b.w), acc, 0, 0, 0);
  }
}

// Element-wise form of the kept-channel gather for group widths that do not fill a 16-byte chunk: the
// elements at offsets eoff[] of a weight row; every load is issued (an element that must read as zero has a valid
// offset and is dropped afterwards), so the loads of a slice stay in flight together.
// UE = elements moved per load (1, 2 or 4: a group is a whole number of such units, so a unit never straddles two
// groups and is aligned to its own size); eoff[] / okbits are per element, a unit is described by its first one.
template <typename ET, int UE>
__device__ __forceinline__ uint4 gather_elems(const ET* w, const int (&eoff)[elem<ET>::per16], unsigned okbits) {
  constexpr int EPC = elem<ET>::per16;
  struct alignas(UE * sizeof(ET)) Unit { ET v[UE]; };
  Unit tmp[EPC / UE];
#pragma unroll
  for (int u = 0; u < EPC / UE; ++u) tmp[u] = *reinterpret_cast<const Unit*>(w + eoff[u * UE]);
#pragma unroll
  for (int u = 0; u < EPC / UE; ++u)
    if (!((okbits >> (u * UE)) & 1u)) {
#pragma unroll
      for (int e = 0; e < UE; ++e) tmp[u].v[e] = (ET)0;
    }
  uint4 r;
  __builtin_memcpy(&r, tmp, 16);
  return r;
}

// Zeroes the elements of a 16-byte chunk from position `nvalid` on.
template <typename ET>
__device__ __forceinline__ uint4 mask_tail(uint4 v, int nvalid) {
  constexpr int EPC = elem<ET>::per16;
  ET tmp[EPC];
  __builtin_memcpy(tmp, &v, 16);
#pragma unroll
  for (int e = 0; e < EPC; ++e)
    if (e >= nvalid) tmp[e] = (ET)0;
  __builtin_memcpy(&v, tmp, 16);
  return v;
}

// first position of a sorted list whose value is not below `key`
__device__ __forceinline__ int lower_bound_dev(const int32_t* v, int n, int key) {
  int lo = 0, hi = n;
  while (lo < hi) {
    const int mid = (lo + hi) >> 1;
    if (v[mid] < key) lo = mid + 1; else hi = mid;
  }
  return lo;
}

template <int MODE, typename ET, int BM, int BN, int WGN>
__global__ __launch_bounds__(128 * WGN) void k_gemm(const GemmArgs a) {
  // 2 x WGN waves; each wave owns a (BM/2) x (BN/WGN) sub-tile of 32x32 MFMA tiles.
  constexpr int NT = 128 * WGN;          // threads per workgroup
  constexpr int RPP = NT / 8;            // tile rows covered by one pass of the loading threads
  constexpr int EPC = elem<ET>::per16;   // elements per 16-byte chunk
  constexpr int BKE = 8 * EPC;           // K elements per LDS slice (128 bytes per row)
  constexpr int LSTR = 144;              // LDS row stride in bytes (128 + 16 pad)
  constexpr int AR = BM / RPP, BR = BN / RPP;
  constexpr int TM = BM / 64, TN = BN / (32 * WGN);
  static_assert(AR >= 1 && BR >= 1 && TN >= 1, "tile too small for this many waves");
  constexpr bool TAPS = (MODE == M_CONV2 || MODE == M_CS2 || MODE == M_U2 || MODE == M_SD2 || MODE == M_G2);
  constexpr bool CS = (MODE >= M_CS1 && MODE <= M_CS3);

  constexpr int A_BYTES = BM * LSTR, B_BYTES = BN * LSTR, STAGE_BYTES = A_BYTES + B_BYTES;
  constexpr int CSTR = BN * 4 + 32;      // epilogue staging row stride in bytes
  // dynamic LDS = max(two pipeline stages, epilogue staging) [+ K floats of masker weights in DENSE1];
  // the launcher sizes it the same way
  constexpr int MAIN_BYTES = (2 * STAGE_BYTES > BM * CSTR) ? 2 * STAGE_BYTES : BM * CSTR;
  extern __shared__ __align__(16) unsigned char smem[];  // two pipeline stages, reused by the epilogue
  __shared__ int s_row[BM];
  __shared__ unsigned char s_inact[MODE == M_SD1 ? BM : 1];  // SD1 with a patch list: row lies in an inactive patch
  __shared__ int s_kgrp[CS ? kMaxGroups : 1];
  __shared__ int s_nkept;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  if constexpr (MODE == M_CONV1 || MODE == M_DENSE1) {
    if (a.pk_out != nullptr && (int)blockIdx.x >= a.pk_first_block) {
      const int nextra = (int)gridDim.x - a.pk_first_block;
      for (int idx = ((int)blockIdx.x - a.pk_first_block) * NT + tid; idx < a.pk_chunks; idx += nextra * NT)
        tail_pack_chunk(idx, (const uint4*)a.pk_w2, (const uint4*)a.pk_w3, (uint4*)a.pk_out);
      return;
    }
  }
  const int wm = wave / WGN, wn = wave % WGN;
  const int HW = a.H * a.W, SS = a.S * a.S;
  // Dynamic blocks with a spatial stride (a.stride > 1) keep their mask on the output grid Ho x Wo;
  // everywhere else the output grid is the input grid.
  const int sy = a.stride > 1 ? a.stride : 1;
  const int oH = a.stride > 1 ? a.Ho : a.H, oW = a.stride > 1 ? a.Wo : a.W;
  const int Hp = oH / a.S, Wp = oW / a.S;
  const ET* __restrict__ Ap = (const ET*)a.A;
  const ET* __restrict__ Wp_ = (const ET*)a.Wt;
  // ---- which tile ---------------------------------------------------------------------------
  int rt, ct, sample = 0, M;
  const int32_t* listp = a.list;
  if constexpr (!CS) {
    // XCD-aware decode: consecutive workgroup ids go round-robin over the 8 XCDs, so the column
    // tiles of one row tile (same A rows) are given to the same XCD, one after the other.
    const int L = blockIdx.x, xcd = L & 7, s = L >> 3;
    rt = (s / a.col_tiles) * 8 + xcd;
    ct = s % a.col_tiles;
    if (rt >= a.row_tiles) return;
    if constexpr (MODE == M_CONV1) {
      // the dilated pixel lists are per group of samples: tile -> (group, tile within the group)
      const int g = rt / a.tiles_per_group;
      rt -= g * a.tiles_per_group;
      listp += (size_t)g * a.group_rows;
      M = a.count[g];
    } else if constexpr (MODE == M_DENSE1 || (MODE >= M_SD1 && MODE <= M_SD3)) {
      M = a.m_rows;
    } else {
      M = *a.count * (MODE == M_U1 ? (a.S + 2) * (a.S + 2) : SS);
    }
  } else {
    rt = blockIdx.x % a.row_tiles;
    ct = blockIdx.x / a.row_tiles;
    sample = blockIdx.y;
    M = HW;
  }
  const int row0 = rt * BM, col0 = ct * BN;
  if (row0 >= M) return;

  // ---- channel skipping: kept-group list of this sample (ballot + prefix, one wave) ----------
  int ncols = a.Ncols, keff = a.K;
  if constexpr (CS) {
    if (wave == 0) {
      int base = 0;
      for (int g0 = 0; g0 < a.D; g0 += kWave) {
        const int g = g0 + lane;
        const bool f = g < a.D && a.cmask[(size_t)sample * a.D + g] != 0;
        const unsigned long long b = __ballot(f);
        if (f) s_kgrp[base + ballot_prefix(b)] = g;
        base += __popcll(b);
      }
      if (lane == 0) s_nkept = base;
    }
    __syncthreads();
    const int kw = s_nkept * a.G;
    if (MODE != M_CS3) ncols = kw;
    if (MODE != M_CS1) keff = kw;
    if (col0 >= ncols) return;
  }
  // group convolution: the reduction runs over the input channels col0 .. col0+BN-1 (the groups of this
  // tile's output channels; the launcher makes BN a multiple of the group width)
  if constexpr (MODE == M_G2) keff = min(BN, a.K - col0);

  // ---- row descriptors ------------------------------------------------------------------------
  // Each thread keeps, for the AR activation rows and BR weight rows it loads, one 32-bit byte offset
  // that already includes its 16-byte chunk, plus (tap modes) a 9-bit mask of the taps that fall
  // inside the image.  A chunk that must read as zero (tap outside the image, row past the end, K
  // tail) is never masked afterwards: its load is pointed outside the operand's descriptor (below).
  const int cc = tid & 7;    // 16-byte chunk within the 128-byte K slice
  const int lr = tid >> 3;   // first row this thread loads
  // The kept-channel weight gather of channel skipping (CS2 / CS3) still reads through pointers; its
  // zero chunks come from a page of zeros.  Hide where that page's address comes from (knowing that it
  // is a dereferenceable global, the compiler would split `load(ok ? row : zeros)` into two loads under
  // a branch) but keep the fact that it is global memory, so that the loads stay global_load (vmcnt
  // only) and not flat_load.
  unsigned long long zaddr = reinterpret_cast<unsigned long long>(&g_zero_page[0]);
#if defined(__HIP_DEVICE_COMPILE__)  // the constraint names a GPU register class: device pass only
  asm volatile("" : "+s"(zaddr));
#endif
  const gptr16 zpage = (gptr16)zaddr;
  // Activation (and, outside the kept-channel gather of channel skipping, weight) chunks are fetched with
  // buffer loads: a resource descriptor over the operand, a per-thread 32-bit byte offset that is fixed
  // for the whole K loop, and a wave-uniform scalar offset per K slice.  A chunk that must read as zero
  // gets the offset 0x80000000, which lies outside the descriptor's 2 GiB range: the hardware returns
  // zeros for it.  A load then costs one select instead of 64-bit pointer arithmetic.
  constexpr unsigned kOob = 0x80000000u;
  constexpr int ROWW_IS_TILE = (MODE == M_U2);
  // taps reach one row and one pixel back: the descriptor starts that far before the operand so that
  // the scalar tap offsets are never negative
  const long long ashift = TAPS ? (long long)((ROWW_IS_TILE ? a.S + 2 : a.W) + 1) * a.lda * (long long)sizeof(ET) : 0;
  const __amdgpu_buffer_rsrc_t arsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(reinterpret_cast<const char*>(Ap)) - ashift, 0, (int)kOob, 0x00020000);
  const __amdgpu_buffer_rsrc_t wrsrc = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<char*>(reinterpret_cast<const char*>(Wp_)), 0, (int)kOob, 0x00020000);
  unsigned voffA[AR];        // byte offset of (row, this thread's chunk) inside the activation operand
  unsigned amask[AR];        // tap modes: bit t set = tap t readable; other modes: bit 0 = row valid
#pragma unroll
  for (int i = 0; i < AR; ++i) {
    const int rho = row0 + lr + RPP * i;
    voffA[i] = 0;
    amask[i] = 0;
    if (rho < M) {
      size_t pixrow;  // row of A (pixel id or compact row)
      int y = 0, x = 0;
      if constexpr (MODE == M_CONV1) {
        pixrow = (size_t)listp[rho];
      } else if constexpr (MODE == M_CONV3 || MODE == M_DENSE1 || MODE == M_U1 || MODE == M_U3) {
        pixrow = (size_t)rho;
      } else if constexpr (MODE == M_SD3) {
        pixrow = (size_t)rho;
      } else if constexpr (MODE == M_SD1 || MODE == M_SD2) {
        // row = output pixel (n, yo, xo); the input pixel under it (centre of the 3x3) is (yo*stride, xo*stride)
        const int n = rho / (a.Ho * a.Wo), r2 = rho - n * (a.Ho * a.Wo);
        y = (r2 / a.Wo) * a.stride;
        x = (r2 % a.Wo) * a.stride;
        pixrow = (size_t)n * HW + (size_t)y * a.W + x;
      } else if constexpr (MODE == M_U2) {
        // row = (patch p, pixel j of the patch); its centre inside the gathered (S+2) x (S+2) tile
        const int E = a.S + 2;
        const int p = rho / SS, j = rho - p * SS;
        pixrow = (size_t)p * E * E + (size_t)(j / a.S + 1) * E + (j % a.S + 1);
      } else if constexpr (MODE == M_CONV2 || MODE == M_G2) {
        const int p = rho / SS, j = rho - p * SS;
        const int q = a.list[p];
        const int n = q / (Hp * Wp), r2 = q - n * (Hp * Wp);
        const int py = r2 / Wp, px = r2 - py * Wp;
        y = (py * a.S + j / a.S) * sy;  // centre of the 3x3 on the input grid
        x = (px * a.S + j % a.S) * sy;
        pixrow = (size_t)n * HW + (size_t)y * a.W + x;
      } else if constexpr (MODE == M_CS2) {
        y = rho / a.W;
        x = rho - y * a.W;
        pixrow = (size_t)sample * HW + rho;
      } else {  // CS1, CS3
        pixrow = (size_t)sample * HW + rho;
      }
      voffA[i] = (unsigned)((pixrow * a.lda + cc * EPC + (MODE == M_G2 ? col0 : 0)) * sizeof(ET));
      if constexpr (MODE == M_U2) {
        amask[i] = 0x1ffu;  // every tap lies inside the gathered tile
      } else if constexpr (TAPS) {
        unsigned mk = 0;
#pragma unroll
        for (int t = 0; t < 9; ++t) {
          const int yy = y + t / 3 - 1, xx = x + t % 3 - 1;
          if (yy >= 0 && yy < a.H && xx >= 0 && xx < a.W) mk |= 1u << t;
        }
        amask[i] = mk;
      } else {
        amask[i] = 1u;
      }
    }
  }
  if (tid < BM) {
    const int rho = row0 + tid;
    int o = -1;
    if (rho < M) {
      if constexpr (MODE == M_CONV1) {
        o = listp[rho];
      } else if constexpr (MODE == M_CONV2 || MODE == M_DENSE1 || MODE == M_U2 || MODE == M_U3 || MODE >= M_SD1) {
        o = rho;  // (G2 included)
      } else if constexpr (MODE == M_U1) {
        // gathered position (p, e): inside the image -> row rho, outside -> -2 - rho (stored as zeros)
        const int E = a.S + 2;
        const int p = rho / (E * E), e = rho - p * (E * E);
        const int q = a.list[p];
        const int r2 = q % (Hp * Wp);
        const int yy = (r2 / Wp) * a.S - 1 + e / E, xx = (r2 % Wp) * a.S - 1 + e % E;
        o = (yy >= 0 && yy < a.H && xx >= 0 && xx < a.W) ? rho : -2 - rho;
      } else if constexpr (MODE == M_CONV3) {
        const int p = rho / SS, j = rho - p * SS;
        const int q = a.list[p];
        const int n = q / (Hp * Wp), r2 = q - n * (Hp * Wp);
        const int py = r2 / Wp, px = r2 - py * Wp;
        o = n * (oH * oW) + (py * a.S + j / a.S) * oW + (px * a.S + j % a.S);
      } else {
        o = sample * HW + rho;
      }
    }
    s_row[tid] = o;
    if constexpr (MODE == M_SD1) {
      // shortcut of a dynamic first block: the activation is applied here only where the branch will
      // not be added (inactive patches); active rows get it in the last conv's epilogue
      bool inact = true;
      if (a.list != nullptr && rho < M) {
        const int n = rho / (a.Ho * a.Wo), r2 = rho - n * (a.Ho * a.Wo);
        const int q = (n * Hp + (r2 / a.Wo) / a.S) * Wp + (r2 % a.Wo) / a.S;
        const int cnt = *a.count;
        const int pos = lower_bound_dev(a.list, cnt, q);
        inact = !(pos < cnt && a.list[pos] == q);
      }
      s_inact[tid] = inact ? 1 : 0;
    }
  }

  // ---- weight-row descriptors -----------------------------------------------------------------
  const ET* wrow[BR];
  unsigned voffW[BR];
  int wrel[BR];  // G2: first channel of this thread's chunk of the window's first slice, relative to the row's group
  bool cvalid[BR];
#pragma unroll
  for (int i = 0; i < BR; ++i) {
    const int c = col0 + lr + RPP * i;
    cvalid[i] = c < ncols;
    int wr = cvalid[i] ? c : col0;  // a column past the end re-reads the tile's first row: its result is dropped
    if constexpr (MODE == M_CS1 || MODE == M_CS2) wr = s_kgrp[wr / a.G] * a.G + (wr % a.G);
    wrow[i] = Wp_ + (size_t)wr * a.ldw;
    if constexpr (!(MODE == M_CS2 || MODE == M_CS3)) wrow[i] += cc * EPC;
    voffW[i] = (unsigned)(((size_t)wr * a.ldw + cc * EPC) * sizeof(ET));
    wrel[i] = 0;
    if constexpr (MODE == M_G2) {
      voffW[i] = (unsigned)((size_t)wr * a.ldw * sizeof(ET));
      wrel[i] = col0 + cc * EPC - (wr / a.gw) * a.gw;
    }
  }
  // DENSE1: the first column tile also accumulates the masker projection of its rows, on the vector
  // ALU, from the A chunks on their way from registers to LDS (each thread: AR rows x one chunk).
  const bool do_proj = (MODE == M_DENSE1) && ct == 0 && a.wmask != nullptr;
  float* const s_wm = reinterpret_cast<float*>(smem + MAIN_BYTES);  // masker weights (DENSE1 only)
  float pacc[AR];
#pragma unroll
  for (int i = 0; i < AR; ++i) pacc[i] = 0.f;
  if constexpr (MODE == M_DENSE1) {
    if (do_proj)
      for (int k = tid; k < a.K; k += NT) s_wm[k] = a.wmask[k];
    __syncthreads();  // the first store_slice below already reads s_wm
  }

  const int kchunks = (keff + BKE - 1) / BKE;
  const int KT = (TAPS ? 9 : 1) * kchunks;
  const bool kvec = (a.G % EPC) == 0;  // kept-channel gather can use 16-byte loads

  // Issues the loads of this thread's 16-byte chunks of the next K slice (A: AR rows, B: BR weight
  // rows).  All loads are unconditional and branch-free, so the compiler can count the loads in
  // flight instead of draining them.  Slices are visited in order; (tap, kc) advance per call.
  const int gK = a.K, gG = a.G;
  const int gshift = (gG & (gG - 1)) == 0 ? __builtin_ctz((unsigned)gG) : -1;  // log2 of a power-of-two group width
  // elements per load of the element-wise kept-channel gather: the largest of 4, 2, 1 that divides the group width
  // and stays within 8 bytes
  const int gunit = (gG % 4 == 0 && sizeof(ET) == 2) ? 4 : (gG % 2 == 0 ? 2 : 1);
  // Scalar state of the load side, advanced once per slice: byte offsets of the slice in the activation
  // and weight operands, the position (tap, K chunk) and the tap's bit for the rows' tap masks.  Past the
  // last tap the bit has left the masks' range and `live` is off, so null slices select nothing.
  constexpr int NTAPS = TAPS ? 9 : 1;
  constexpr int SLICE_B = BKE * (int)sizeof(ET);  // 128
  const int rowW = ROWW_IS_TILE ? a.S + 2 : a.W;
  const int pix_b = a.lda * (int)sizeof(ET);
  const int back_b = (kchunks - 1) * SLICE_B;     // from a tap's last slice back to its first
  const int a_pixjump = pix_b - back_b, a_rowjump = (rowW - 2) * pix_b - back_b;
  // weights: next slice of the same tap / first slice of the next tap (G2: a tap is gw channels wide and
  // the slice position inside it goes into the per-thread offset)
  const int w_step = MODE == M_G2 ? 0 : SLICE_B;
  const int w_tapjump = MODE == M_G2 ? a.gw * (int)sizeof(ET) : gK * (int)sizeof(ET) - back_b;
  // only a tap's last K chunk can be partial: whether this thread's chunk of it lies inside K
  const bool lastok = (kchunks - 1) * BKE + cc * EPC < keff;
  int ld_tap = 0, ld_kc = 0, ld_kx = -1, s_a = 0, s_w = 0;
  unsigned tapbit = 1u;
  bool live = true;
  auto load_slice = [&](u32x4 (&ra)[AR], u32x4 (&rb)[BR]) __attribute__((always_inline)) -> int {
    const int tap = ld_tap;
    const int ke = ld_kc * BKE + cc * EPC;  // this thread's first (compact) K element
    const int kcb = ld_kc * BKE;
    // (with an empty reduction -- channel skipping with every group dropped -- kchunks is 0 and no chunk is inside K)
    const bool kok = ld_kc < kchunks - 1 || (ld_kc == kchunks - 1 && lastok);
    const bool kv = kok && live;            // slices past the end read as zeros
    const int asoff = s_a, wsoff = s_w;
    const unsigned tb = tapbit;
    // branch-free advance (scalar selects)
    const bool wrap = ld_kc + 1 == kchunks;       // last K chunk of the tap
    const bool rowwrap = wrap && ld_kx == 1;      // ... of the last tap of a tap row
    s_a += wrap ? (rowwrap ? a_rowjump : a_pixjump) : SLICE_B;
    s_w += wrap ? w_tapjump : w_step;
    ld_kc = wrap ? 0 : ld_kc + 1;
    ld_kx = rowwrap ? -1 : ld_kx + (wrap ? 1 : 0);
    ld_tap += wrap ? 1 : 0;
    tapbit <<= wrap ? 1 : 0;
    live = ld_tap < NTAPS;
#pragma unroll
    for (int i = 0; i < AR; ++i) {
      const bool ok = kok && (amask[i] & tb);
      ra[i] = __builtin_amdgcn_raw_buffer_load_b128(arsrc, ok ? voffA[i] : kOob, asoff, 0);
    }
    // narrow groups (kept-channel gather element by element): the chunk's element offsets inside a weight
    // row are the same for every row of this thread
    int eoff[EPC];
    unsigned eok = 0;
    if constexpr (MODE == M_CS2 || MODE == M_CS3) {
      if (!kvec) {
#pragma unroll
        for (int e = 0; e < EPC; ++e) {
          const bool ok = kv && ke + e < keff;
          const int kk = ok ? ke + e : 0;
          const int g = gshift >= 0 ? kk >> gshift : kk / gG;
          eoff[e] = (keff > 0 ? s_kgrp[g] : 0) * gG + (kk - g * gG);
          eok |= ok ? (1u << e) : 0u;
        }
      }
    }
#pragma unroll
    for (int i = 0; i < BR; ++i) {
      if constexpr (MODE == M_CS2 || MODE == M_CS3) {
        const ET* wtap = wrow[i] + (long long)tap * gK;
        if (kvec) {
          rb[i] = *(kv ? (gptr16)(wtap + s_kgrp[ke / gG] * gG + (ke % gG)) : zpage);
        } else {
          // the compact K range ends on a group boundary, so a unit is inside it or outside it as a whole
          const uint4 g = gunit == 4 ? gather_elems<ET, (EPC >= 4 ? 4 : 1)>(wtap, eoff, eok)
                          : gunit == 2 ? gather_elems<ET, 2>(wtap, eoff, eok)
                                       : gather_elems<ET, 1>(wtap, eoff, eok);
          rb[i] = u32x4{g.x, g.y, g.z, g.w};
        }
      } else if constexpr (MODE == M_G2) {
        const int rel = wrel[i] + kcb;  // chunk's first channel inside the row's group, if it is in it
        const bool ing = kv && (unsigned)rel < (unsigned)a.gw;
        rb[i] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, ing ? voffW[i] + (unsigned)rel * (unsigned)sizeof(ET) : kOob,
                                                      wsoff, 0);
      } else {
        rb[i] = __builtin_amdgcn_raw_buffer_load_b128(wrsrc, kv ? voffW[i] : kOob, wsoff, 0);
      }
    }
    return ke;
  };
  auto store_slice = [&](int buf, const u32x4 (&ra)[AR], const u32x4 (&rb)[BR], int ke) __attribute__((always_inline)) {
    unsigned char* sA = smem + buf * STAGE_BYTES;
    unsigned char* sB = sA + A_BYTES;
#pragma unroll
    for (int i = 0; i < AR; ++i) {
      u32x4 v = ra[i];
      if constexpr (MODE == M_CS2 || MODE == M_CS3) {
        // compact rows are valid up to keff only; what lies beyond in the scratch buffer is undefined
        if (!kvec && ke + EPC > keff) {
          const uint4 t = mask_tail<ET>(make_uint4(v.x, v.y, v.z, v.w), keff - ke);
          v = u32x4{t.x, t.y, t.z, t.w};
        }
      }
      *reinterpret_cast<u32x4*>(sA + (lr + RPP * i) * LSTR + cc * 16) = v;
      if constexpr (MODE == M_DENSE1) {
        if (do_proj && ke < keff) {
          ET xe[EPC];
          __builtin_memcpy(xe, &v, 16);
#pragma unroll
          for (int e = 0; e < EPC; ++e) pacc[i] += elem<ET>::load(&xe[e]) * s_wm[ke + e];
        }
      }
    }
#pragma unroll
    for (int i = 0; i < BR; ++i) *reinterpret_cast<u32x4*>(sB + (lr + RPP * i) * LSTR + cc * 16) = rb[i];
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;


  auto compute = [&](int buf) __attribute__((always_inline)) {
    const unsigned char* pa = smem + buf * STAGE_BYTES + (wm * (BM / 2) + (lane & 31)) * LSTR + (lane >> 5) * 16;
    const unsigned char* pb = smem + buf * STAGE_BYTES + A_BYTES + (wn * (BN / WGN) + (lane & 31)) * LSTR +
                              (lane >> 5) * 16;
#pragma unroll
    for (int kg = 0; kg < 4; ++kg) {
      uint4 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const uint4*>(pa + i * 32 * LSTR + kg * 32);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const uint4*>(pb + j * 32 * LSTR + kg * 32);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j) mma16<ET>(acc[i][j], fa[i], fb[j]);
    }
  };

  constexpr int CPR = BN / EPC;                 // 16-byte output chunks per tile row
  constexpr int EPI = (BM * CPR + NT - 1) / NT;  // epilogue chunks per thread
  constexpr bool RES = (MODE == M_CONV3 || MODE == M_CS3 || MODE == M_SD3);
  // Software pipeline: PF register sets hold the slices in flight from L2 / HBM, two LDS stages.
  // Step s multiplies slice s out of stage s%2 while slice s+1 moves from its registers to the other
  // stage and slices s+2 .. s+PF are in flight: one barrier per slice, PF-1 slices of load latency
  // covered.  Every step is identical -- slices past the end load zeros (offset outside the descriptor) and add
  // nothing -- so the loop carries no conditional loads and the compiler's load counting holds.
  constexpr int PF = 2;
  static_assert(PF % 2 == 0, "stage parity must be static per unrolled step");
  u32x4 ra[PF][AR], rb[PF][BR];
  int kes[PF];
#pragma unroll
  for (int d = 0; d < PF; ++d) kes[d] = load_slice(ra[d], rb[d]);
  store_slice(0, ra[0], rb[0], kes[0]);
  kes[0] = load_slice(ra[0], rb[0]);
  __syncthreads();  // stage 0 is ready; also publishes s_row
  for (int s0 = 0; s0 < KT; s0 += PF) {
#pragma unroll
    for (int d = 0; d < PF; ++d) {
      const int nx = (d + 1) % PF;            // register set of slice s0+d+1
      store_slice((d + 1) & 1, ra[nx], rb[nx], kes[nx]);
      kes[nx] = load_slice(ra[nx], rb[nx]);
      compute(d & 1);
      __syncthreads();
    }
  }
  if constexpr (MODE == M_DENSE1) {
    if (do_proj) {
#pragma unroll
      for (int i = 0; i < AR; ++i) {
        float v = pacc[i];  // partial over this thread's chunk column; the row's 8 chunk columns are 8 adjacent lanes
        v += __shfl_xor(v, 1, kWave);
        v += __shfl_xor(v, 2, kWave);
        v += __shfl_xor(v, 4, kWave);
        const int rho = row0 + lr + RPP * i;
        if (cc == 0 && rho < M) a.proj[rho] = v;
      }
    }
  }

  // ---- epilogue ---------------------------------------------------------------------------------
  // Affine (+ReLU) in the accumulator layout (32x32 tile: lane l holds column l%32, rows
  // 8*(e/4) + 4*(l/32) + e%4), then through LDS so that global traffic is 16 bytes per lane:
  // residual read, add, rounding and the scatter store all happen on whole 16-byte channel chunks.
  {
    float* stg = reinterpret_cast<float*>(smem);
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const int cl = wn * (BN / WGN) + j * 32 + (lane & 31);
      const int col = col0 + cl;
      float sc = 0.f, sh = 0.f;
      if (col < ncols) {
        int ch = col;
        if constexpr (MODE == M_CS1 || MODE == M_CS2) ch = s_kgrp[col / a.G] * a.G + (col % a.G);
        sc = a.scale[ch];
        sh = a.shift[ch];
      }
#pragma unroll
      for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int e = 0; e < 16; ++e) {
          const int rl = wm * (BM / 2) + i * 32 + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
          float v = acc[i][j][e] * sc + sh;
          if constexpr (MODE == M_SD1) {
            if (a.relu && s_inact[rl]) v = fmaxf(v, 0.f);
          } else if constexpr (!(MODE == M_CONV3 || MODE == M_CS3 || MODE == M_U3 || MODE == M_SD3)) {
            v = fmaxf(v, 0.f);
          }
          stg[rl * (CSTR / 4) + cl] = v;
        }
      }
    }
  }
  __syncthreads();
  {
    ET* Op = (ET*)a.Out;
    const ET* Rp = (const ET*)a.Res;
#pragma unroll
    for (int q = 0; q < EPI; ++q) {
      const int id = tid + q * NT;
      if (id >= BM * CPR) continue;
      const int rl = id / CPR, chk = id - rl * CPR;
      int orow = s_row[rl];
      const int col = col0 + chk * EPC;
      bool zero_row = false;
      if constexpr (MODE == M_U1) {
        if (orow <= -2) { orow = -2 - orow; zero_row = true; }
      }
      if (orow < 0 || col >= ncols) continue;
      const float* sp = reinterpret_cast<const float*>(smem + rl * CSTR) + chk * EPC;
      float v[EPC];
#pragma unroll
      for (int u = 0; u < EPC / 4; ++u) {
        const float4 t4 = reinterpret_cast<const float4*>(sp)[u];
        v[4 * u] = t4.x; v[4 * u + 1] = t4.y; v[4 * u + 2] = t4.z; v[4 * u + 3] = t4.w;
      }
      if (zero_row) {
#pragma unroll
        for (int e = 0; e < EPC; ++e) v[e] = 0.f;
      }
      const size_t off = (size_t)orow * a.ldo + col;
      if (col + EPC <= ncols) {
        if constexpr (RES) {
          // the residual is read here, not ahead of the K loop: requested early it only delays the first
          // slices (loads return in order) and measured slower
          const u32x4 rraw = *(gptr16)(Rp + off);
          ET rr[EPC];
          __builtin_memcpy(rr, &rraw, 16);
#pragma unroll
          for (int e = 0; e < EPC; ++e) {
            v[e] += elem<ET>::load(&rr[e]);
            if (a.relu) v[e] = fmaxf(v[e], 0.f);
          }
        }
        if constexpr (MODE == M_U3) {
          // the unfused schedule's branch output stays float32 so that the stand-alone scatter adds
          // the residual before the only rounding, like the fused epilogue does
          float* fo = reinterpret_cast<float*>(a.Out) + off;
#pragma unroll
          for (int u = 0; u < EPC / 4; ++u)
            reinterpret_cast<float4*>(fo)[u] = make_float4(v[4 * u], v[4 * u + 1], v[4 * u + 2], v[4 * u + 3]);
        } else {
          ET ov[EPC];
#pragma unroll
          for (int e = 0; e < EPC; ++e) elem<ET>::store(&ov[e], v[e]);
          uint4 oraw;
          __builtin_memcpy(&oraw, ov, 16);
          *reinterpret_cast<uint4*>(Op + off) = oraw;
        }
      } else {  // ragged last chunk (channel-skip widths that are not a multiple of the chunk)
        for (int e = 0; e < ncols - col; ++e) {
          float u = v[e];
          if constexpr (RES) {
            u += elem<ET>::load(Rp + off + e);
            if (a.relu) u = fmaxf(u, 0.f);
          }
          elem<ET>::store(Op + off + e, u);
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------------------
// dilated active set: which pixels need conv1 (the patch pixels and their one-pixel halo)
// ------------------------------------------------------------------------------------------------

// One block per group of `gs` consecutive samples: writes the ids of the group's needed pixels in
// ascending order at pix[g*gs*H*W ...] and their number at need_counts[g] (ordered, no atomics, no
// dependency between blocks).  The group's patch mask is rebuilt in LDS from the sorted index list.
constexpr int kNeedThreads = 1024;
__global__ __launch_bounds__(kNeedThreads) void k_need(const int32_t* __restrict__ idx,
                                                       const int32_t* __restrict__ count, int N, int H, int W, int S,
                                                       int stride, int Ho, int Wo, int gs,
                                                       int32_t* __restrict__ need_counts,
                                                       int32_t* __restrict__ pix) {
  extern __shared__ unsigned char s_pm[];  // [ns*Hp*Wp] patch masks of the group's samples
  constexpr int NW = kNeedThreads / kWave;
  __shared__ int scan[2][NW];
  const int g = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  // the patch grid lives on the output grid Ho x Wo (= H x W when stride is 1); pixels are input pixels
  const int Hp = Ho / S, Wp = Wo / S, pps = Hp * Wp, HW = H * W;
  const int n0 = g * gs, ns = min(gs, N - n0);
  const int cnt = *count;
  for (int i = tid; i < ns * pps; i += kNeedThreads) s_pm[i] = 0;
  __syncthreads();
  // The group's slice of the sorted index list: short lists are scanned whole by all threads (a
  // handful of independent loads each); longer ones are searched 64 probes at a time by every wave.
  int lo = 0, hi = cnt;
  if (cnt > 16 * kNeedThreads) {
    lo = wave_lower_bound(idx, cnt, n0 * pps);
    hi = wave_lower_bound(idx, cnt, (n0 + ns) * pps);
  }
  // eight entries per thread requested before any is used: one round trip per batch, not per entry
  for (int i0 = lo + tid; i0 < hi; i0 += 8 * kNeedThreads) {
    int e[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) e[u] = idx[min(i0 + u * kNeedThreads, hi - 1)];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const unsigned v = (unsigned)(e[u] - n0 * pps);
      if (i0 + u * kNeedThreads < hi && v < (unsigned)(ns * pps)) s_pm[v] = 1;
    }
  }
  __syncthreads();
  int32_t* out = pix + (size_t)g * gs * HW;
  int running = 0;
  for (int p0 = 0, it = 0; p0 < ns * HW; p0 += kNeedThreads, ++it) {
    const int pp = p0 + tid;
    bool need = false;
    if (pp < ns * HW) {
      const int ln = pp / HW, q = pp - ln * HW;
      const int y = q / W, x = q - y * W;
      // output pixel yo reads input rows stride*yo-1 .. stride*yo+1, so input row y serves the output
      // rows ceil((y-1)/stride) .. floor((y+1)/stride), clipped to the output grid
      const int yo0 = max((y - 1 + stride - 1) / stride, 0), yo1 = min((y + 1) / stride, Ho - 1);
      const int xo0 = max((x - 1 + stride - 1) / stride, 0), xo1 = min((x + 1) / stride, Wo - 1);
      const unsigned char* pm = s_pm + ln * pps;
      for (int py = yo0 / S; py <= yo1 / S; ++py)
        for (int px = xo0 / S; px <= xo1 / S; ++px) need |= pm[py * Wp + px] != 0;
    }
    const unsigned long long b = __ballot(need);
    int tot;
    const int wo = scan_wave_counts(__popcll(b), NW, scan[it & 1], &tot);
    if (need) out[running + wo + ballot_prefix(b)] = n0 * HW + pp;
    running += tot;
  }
  if (tid == 0) need_counts[g] = running;
}

// Out-of-place call: pixels of inactive patches are copied bit for bit.  One block per patch.
__global__ __launch_bounds__(256) void k_copy_inactive(const uint4* __restrict__ x, uint4* __restrict__ out, int H,
                                                       int W, int S, int cpp, const int32_t* __restrict__ idx,
                                                       const int32_t* __restrict__ count) {
  const int q = blockIdx.x, cnt = *count;
  const int pos = lower_bound_dev(idx, cnt, q);
  if (pos < cnt && idx[pos] == q) return;  // active: the conv3 epilogue writes it
  const int Hp = H / S, Wp = W / S;
  const int n = q / (Hp * Wp), r = q - n * (Hp * Wp);
  const int py = r / Wp, px = r - py * Wp;
  const int total = S * S * cpp;
  for (int c = threadIdx.x; c < total; c += 256) {
    const int j = c / cpp, cv = c - j * cpp;
    const size_t off = (((size_t)n * H + (py * S + j / S)) * W + (px * S + j % S)) * cpp + cv;
    out[off] = x[off];
  }
}

// ------------------------------------------------------------------------------------------------
// host side
// ------------------------------------------------------------------------------------------------
struct Tile { int bm, bn, waves; };

// Tile choice: a function of the shapes alone.
static Tile pick_tile(int ncols, long long total_rows) {
  if (ncols < 128) return {64, 64, 4};
  // eight waves hide each other's LDS and load stalls; the large tile needs enough rows to fill the chip
  return total_rows >= 8192 ? Tile{128, 128, 8} : Tile{64, 128, 8};
}

// More than 64 KB of dynamic LDS has to be requested once per kernel and device.  The request is idempotent, so
// threads that race on a first call only repeat it; laud_init() makes it for every kernel up front (so that no
// first call falls inside a stream capture).
template <int MODE, typename ET, int BM, int BN, int WGN>
static int gemm_request_lds() {
  static std::atomic<unsigned> done{0};  // one bit per device ordinal (ordinals >= 32 repeat the request)
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return LAUD_ERR_HIP;
  const unsigned bit = dev >= 0 && dev < 32 ? 1u << dev : 0u;
  if (bit && (done.load(std::memory_order_acquire) & bit)) return LAUD_OK;
  constexpr int kStages = 2 * (BM + BN) * 144;  // two pipeline stages of 144-byte rows
  constexpr int kStaging = BM * (BN * 4 + 32);  // fp32 tile the epilogue transposes through
  constexpr int kLds = kStages > kStaging ? kStages : kStaging;
  if (hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm<MODE, ET, BM, BN, WGN>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, kLds + (MODE == M_DENSE1 ? 4096 * 4 : 0)) != hipSuccess)
    return LAUD_ERR_HIP;
  done.fetch_or(bit, std::memory_order_release);
  return LAUD_OK;
}

template <int MODE, typename ET, int BM, int BN, int WGN>
static int launch_gemm_t(GemmArgs a, long long cap_rows, int nsamples, hipStream_t st) {
  constexpr bool CS = (MODE >= M_CS1 && MODE <= M_CS3);
  a.row_tiles = (int)((cap_rows + BM - 1) / BM);
  if constexpr (MODE == M_CONV1) {  // cap_rows = rows per group of samples, nsamples = number of groups
    a.tiles_per_group = a.row_tiles;
    a.row_tiles *= nsamples;
  }
  a.col_tiles = (a.Ncols + BN - 1) / BN;
  dim3 grid;
  if (!CS) grid = dim3((unsigned)(((a.row_tiles + 7) / 8) * 8 * a.col_tiles));
  else grid = dim3((unsigned)(a.row_tiles * a.col_tiles), (unsigned)nsamples);
  if constexpr (MODE == M_CONV1 || MODE == M_DENSE1) {
    if (a.pk_out != nullptr) {  // spare workgroups for the weight re-ordering: one chunk per thread
      a.pk_first_block = (int)grid.x;
      grid.x += (unsigned)((a.pk_chunks + 128 * WGN - 1) / (128 * WGN));
    }
  } else {
    a.pk_out = nullptr;
  }
  constexpr int kStages = 2 * (BM + BN) * 144;  // two pipeline stages of 144-byte rows
  constexpr int kStaging = BM * (BN * 4 + 32);  // fp32 tile the epilogue transposes through
  constexpr int kLds = kStages > kStaging ? kStages : kStaging;
  if (gemm_request_lds<MODE, ET, BM, BN, WGN>() != LAUD_OK) return LAUD_ERR_HIP;
  const int lds = kLds + ((MODE == M_DENSE1 && a.wmask) ? a.K * 4 : 0);  // + masker weights
  hipLaunchKernelGGL((k_gemm<MODE, ET, BM, BN, WGN>), grid, dim3(128 * WGN), lds, st, a);
  return check_launch();
}

template <int MODE, typename ET>
static int launch_gemm_e(const GemmArgs& a, long long cap_rows, int nsamples, hipStream_t st) {
  const Tile t = pick_tile(a.Ncols, cap_rows * (MODE == M_CONV1 || (MODE >= M_CS1 && MODE <= M_CS3) ? nsamples : 1));
  if (t.waves == 8) {
    if (t.bm == 128) return launch_gemm_t<MODE, ET, 128, 128, 4>(a, cap_rows, nsamples, st);
    return launch_gemm_t<MODE, ET, 64, 128, 4>(a, cap_rows, nsamples, st);
  }
  return launch_gemm_t<MODE, ET, 64, 64, 2>(a, cap_rows, nsamples, st);
}

// The LDS requests of every tile a mode can be launched with, for both element types.
template <int MODE>
static int gemm_request_lds_mode() {
  int rc = LAUD_OK;
  auto keep = [&rc](int r) { if (r != LAUD_OK) rc = r; };
  keep(gemm_request_lds<MODE, bf16_t, 64, 64, 2>());
  keep(gemm_request_lds<MODE, float, 64, 64, 2>());
  if constexpr (MODE != M_G2) {
    keep(gemm_request_lds<MODE, bf16_t, 64, 128, 4>());
    keep(gemm_request_lds<MODE, float, 64, 128, 4>());
    keep(gemm_request_lds<MODE, bf16_t, 128, 128, 4>());
    keep(gemm_request_lds<MODE, float, 128, 128, 4>());
  }
  return rc;
}
template <int... MODES>
static int gemm_request_lds_modes() {
  int rc = LAUD_OK;
  ((rc = (gemm_request_lds_mode<MODES>() != LAUD_OK ? LAUD_ERR_HIP : rc)), ...);
  return rc;
}
int gemm_init_device() {
  return gemm_request_lds_modes<M_CONV1, M_CONV2, M_CONV3, M_CS1, M_CS2, M_CS3, M_DENSE1, M_U1, M_U2, M_U3, M_SD1, M_SD2,
                                M_SD3, M_G2>();
}

template <int MODE>
static int launch_gemm(int dtype, const GemmArgs& a, long long cap_rows, int nsamples, hipStream_t st) {
  constexpr int kStage[14] = {LAUD_STAGE_CONV1, LAUD_STAGE_CONV2, LAUD_STAGE_CONV3, LAUD_STAGE_CS1, LAUD_STAGE_CS2,
                              LAUD_STAGE_CS3,   LAUD_STAGE_CONV1, LAUD_STAGE_CONV1, LAUD_STAGE_CONV2, LAUD_STAGE_CONV3,
                              LAUD_STAGE_CONV1, LAUD_STAGE_CONV2, LAUD_STAGE_CONV3, LAUD_STAGE_CONV2};
  StageScope scope(kStage[MODE], st);
  return dtype == LAUD_BF16 ? launch_gemm_e<MODE, bf16_t>(a, cap_rows, nsamples, st)
                            : launch_gemm_e<MODE, float>(a, cap_rows, nsamples, st);
}

// The kernels address an operand through a buffer descriptor with 32-bit byte offsets and keep the upper
// half of that range for "reads as zero": one operand (activations of a layer, its weights) has to stay
// below 2 GiB, including the distance the 3x3's descriptor is moved back by (one row and one pixel, `tap_rowlen`
// pixels per row) and the same distance a tap can reach forward.
static bool operand_too_big(long long rows, long long row_elems, int dtype, long long tap_rowlen = 0) {
  const unsigned long long eb = elem_bytes(dtype);
  const unsigned long long shift = tap_rowlen > 0 ? (unsigned long long)(tap_rowlen + 1) * row_elems * eb : 0;
  return (unsigned long long)rows * (unsigned long long)row_elems * eb + 2 * shift >= 0x7f000000ull;
}

// 16-byte loads and stores need 16-byte aligned bases.
static bool misaligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
static bool block_params_misaligned(const laud_bottleneck* p) {
  return misaligned16(p->w1) || misaligned16(p->w2) || misaligned16(p->w3);
}
// two ranges of `bytes` bytes that are neither identical nor disjoint
static bool partial_overlap(const void* x, const void* out, size_t bytes_x, size_t bytes_out) {
  const char *a = (const char*)x, *b = (const char*)out;
  if (a == b) return false;
  return (a < b && a + bytes_x > b) || (b < a && b + bytes_out > a);
}

static int validate_block(const void* x, const laud_fmap& fx, const laud_bottleneck* p, const void* out) {
  if (!x || !out || !p || !valid_fmap(fx)) return LAUD_ERR_INVALID_ARG;
  if (!p->w1 || !p->w2 || !p->w3 || !p->s1 || !p->t1 || !p->s2 || !p->t2 || !p->s3 || !p->t3)
    return LAUD_ERR_INVALID_ARG;
  if (p->c_in <= 0 || p->c_mid <= 0 || p->c_out <= 0 || p->c_in != fx.C) return LAUD_ERR_INVALID_ARG;
  if (p->c_out != p->c_in) return LAUD_ERR_UNSUPPORTED;
  if (p->c_in % 8 || p->c_mid % 8) return LAUD_ERR_UNSUPPORTED;
  if (misaligned16(x) || misaligned16(out) || block_params_misaligned(p)) return LAUD_ERR_UNSUPPORTED;
  if ((long long)fx.N * fx.H * fx.W > 0x7fffffffLL / 2) return LAUD_ERR_UNSUPPORTED;
  if (operand_too_big((long long)fx.N * fx.H * fx.W, p->c_in > p->c_mid ? p->c_in : p->c_mid, fx.dtype, fx.W))
    return LAUD_ERR_UNSUPPORTED;
  const size_t bytes = (size_t)fx.N * fx.H * fx.W * fx.C * elem_bytes(fx.dtype);
  if (partial_overlap(x, out, bytes, bytes)) return LAUD_ERR_INVALID_ARG;
  return LAUD_OK;
}

// Channel skipping on the fused kernels: the samples ordered by mask pattern (ascending pattern, ascending sample
// id inside a pattern; ballots and prefix counts, no atomics, so the order is reproducible), so that the rows of a
// tile share their kept groups and whole input slices can be skipped.  One block of four waves; pattern p = sum of
// (kept group g) << g, D <= 4 (16 patterns), N <= 4096 (sixteen rounds of 256 samples, one sample per thread).
// perm [N]: sample ids in that order; sbits [N]: their patterns in that order; rbits [N]: patterns by sample id;
// count: N as a device integer (the kernels read their row count from the device).
constexpr int kCsSortThreads = 256, kCsSortPatterns = 16, kCsSortMaxN = 4096;
__global__ __launch_bounds__(kCsSortThreads) void k_cs_sort(const uint8_t* __restrict__ cmask, int N, int D,
                                                            int32_t* __restrict__ perm, uint8_t* __restrict__ sbits,
                                                            uint8_t* __restrict__ rbits, int32_t* __restrict__ count) {
  constexpr int kSlots = kCsSortMaxN / kWave;      // (round, wave) pairs
  __shared__ int s_cnt[kCsSortPatterns][kSlots];   // samples of pattern p in slot (round * 4 + wave); then their base
  const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
  const int rounds = (N + kCsSortThreads - 1) / kCsSortThreads;
  for (int r = 0; r < rounds; ++r) {
    const int n = r * kCsSortThreads + tid;
    unsigned key = 0;
    if (n < N) {
      for (int g = 0; g < D; ++g) key |= (cmask[(size_t)n * D + g] != 0 ? 1u : 0u) << g;
      rbits[n] = (uint8_t)key;
    }
#pragma unroll
    for (int p = 0; p < kCsSortPatterns; ++p) {
      const unsigned long long b = __ballot(n < N && key == (unsigned)p);
      if (lane == 0) s_cnt[p][r * 4 + wave] = __popcll(b);
    }
  }
  __syncthreads();
  // exclusive prefix over (pattern major, slot minor): thread p sums its pattern's slots, thread 0 the patterns
  __shared__ int s_tot[kCsSortPatterns];
  const int nslots = rounds * 4;
  if (tid < kCsSortPatterns) {
    int acc = 0;
    for (int q = 0; q < nslots; ++q) { const int v = s_cnt[tid][q]; s_cnt[tid][q] = acc; acc += v; }
    s_tot[tid] = acc;
  }
  __syncthreads();
  if (tid == 0) {
    int acc = 0;
    for (int p = 0; p < kCsSortPatterns; ++p) { const int v = s_tot[p]; s_tot[p] = acc; acc += v; }
    *count = N;
  }
  __syncthreads();
  for (int r = 0; r < rounds; ++r) {
    const int n = r * kCsSortThreads + tid;
    unsigned key = 0;
    if (n < N)
      for (int g = 0; g < D; ++g) key |= (cmask[(size_t)n * D + g] != 0 ? 1u : 0u) << g;
    int pos = 0;
#pragma unroll
    for (int p = 0; p < kCsSortPatterns; ++p) {
      const unsigned long long b = __ballot(n < N && key == (unsigned)p);
      if (key == (unsigned)p) pos = s_tot[p] + s_cnt[p][r * 4 + wave] + ballot_prefix(b);
    }
    if (n < N) { perm[pos] = n; sbits[pos] = (uint8_t)key; }
  }
}

struct DynWs { size_t need_counts, scnt, pix, h1, h2, blocks, wpack, bytes; };
static DynWs dyn_ws_layout(const laud_fmap& fx, int c_mid) {
  const size_t npix = (size_t)fx.N * fx.H * fx.W, eb = elem_bytes(fx.dtype);
  DynWs w;
  size_t o = 0;
  w.need_counts = o; o += align_up((size_t)fx.N * 4, 256);  // (fused-masker variant: the kept-sample list of a layer gate)
  w.scnt = o;        o += 256;                               // ... and its length
  w.pix = o;         o += align_up(npix * 4, 256);
  w.h1 = o;          o += align_up(npix * c_mid * eb, 256);
  w.h2 = o;          o += align_up(npix * c_mid * eb, 256);
  w.blocks = o;      o += compact_ws_bytes((long long)npix);  // block counts of a large compaction
  // weights in MFMA fragment order for the fused conv2 -> conv3 kernel (identity block: c_out = C)
  w.wpack = o;       o += (head_supported(fx.dtype, fx.C, c_mid) ? head_packed_bytes(fx.C) : 0) +
                          (tail_supported(fx.dtype, c_mid, fx.C) ? tail_packed_bytes(c_mid, fx.C) : 0);
  w.bytes = o;
  return w;
}

// h1, h2: compact scratch activations.  perm / sbits / rbits / cnt: the samples ordered by mask pattern, the patterns
// in that order and in sample order, and the sample count as a device integer (the fused-kernel path); wpack: room
// for the re-ordered weights of a block that brings none.
struct CsWs { size_t h1, h2, perm, sbits, rbits, cnt, wpack, bytes; };
static CsWs cs_ws_layout(const laud_fmap& fx, int c_mid) {
  const size_t npix = (size_t)fx.N * fx.H * fx.W, eb = elem_bytes(fx.dtype);
  CsWs w;
  w.h1 = 0;
  w.h2 = align_up(npix * c_mid * eb, 256);
  w.perm = 2 * w.h2;
  w.sbits = w.perm + align_up((size_t)fx.N * 4, 256);
  w.rbits = w.sbits + align_up((size_t)fx.N, 256);
  w.cnt = w.rbits + align_up((size_t)fx.N, 256);
  w.wpack = w.cnt + 256;
  w.bytes = w.wpack + (head_supported(fx.dtype, fx.C, c_mid) ? head_packed_bytes(fx.C) : 0) +
            (tail_supported(fx.dtype, c_mid, fx.C) ? tail_packed_bytes(c_mid, fx.C) : 0);
  return w;
}

int launch_dense_affine(int dtype, const void* A, const void* Wt, const float* scale, const float* shift, void* Out,
                        long long rows, int K, int ncols, int relu, hipStream_t stream) {
  if (operand_too_big(rows, K, dtype) || operand_too_big(ncols, K, dtype)) return LAUD_ERR_UNSUPPORTED;
  GemmArgs a{};
  a.H = 1; a.W = 1; a.S = 1; a.D = 1; a.G = 1; a.Ho = 1; a.Wo = 1; a.stride = 1;  // one "pixel" per row
  a.A = A; a.Wt = Wt; a.scale = scale; a.shift = shift; a.Out = Out; a.K = K; a.ldw = K; a.Ncols = ncols;
  a.lda = K; a.ldo = ncols; a.relu = relu; a.m_rows = (int)rows;
  return launch_gemm<M_SD1>(dtype, a, rows, 1, stream);
}

}  // namespace laud

using namespace laud;

extern "C" size_t laud_workspace_size(int op, laud_fmap fx, const laud_bottleneck* p, int S_or_D) {
  switch (op) {
    case LAUD_OP_MASK_GEN: {
      if (!valid_fmap(fx) || S_or_D <= 0 || fx.H % S_or_D || fx.W % S_or_D) return 0;
      return compact_ws_bytes((long long)fx.N * (fx.H / S_or_D) * (fx.W / S_or_D));
    }
    case LAUD_OP_COMPACT:
      return S_or_D >= 0 ? compact_ws_bytes(S_or_D) : 0;
    case LAUD_OP_GATHER:
      return 0;
    case LAUD_OP_DYN_BOTTLENECK:
      if (!valid_fmap(fx) || !p || p->c_mid <= 0) return 0;
      return dyn_ws_layout(fx, p->c_mid).bytes;
    case LAUD_OP_CHANNEL_SKIP:
      if (!valid_fmap(fx) || !p || p->c_mid <= 0) return 0;
      return cs_ws_layout(fx, p->c_mid).bytes;
    default:
      return 0;
  }
}

// Checks the group-convolution / SE extension of a block; hw = pixels per sample of the map h1 lives on.
static int validate_group_se(const laud_bottleneck* p, const laud_group_se* e, const laud_fmap& fx) {
  if (e->group_width <= 0 || p->c_mid % e->group_width || e->se_width < 0) return LAUD_ERR_INVALID_ARG;
  if (e->se_width > 0 && (!e->w_se1 || !e->b_se1 || !e->w_se2 || !e->b_se2)) return LAUD_ERR_INVALID_ARG;
  // a 64-channel output tile must hold whole groups, and a group whole 16-byte chunks
  const int g = e->group_width;
  if (!(g == 8 || g == 16 || g == 32 || g == 64)) return LAUD_ERR_UNSUPPORTED;
  if (e->se_width > kSeMaxHidden || (e->se_width > 0 && p->c_mid > kSeMaxC)) return LAUD_ERR_UNSUPPORTED;
  if (e->se_width > 0 && fx.N > 65535) return LAUD_ERR_UNSUPPORTED;  // one grid row of the squeeze per sample
  // the SE module's means, gates and hidden units are kept in the scratch region of h1 (N*H*W*c_mid elements)
  if (e->se_width > 0 && 4 * (2 * (size_t)p->c_mid + e->se_width) > (size_t)fx.H * fx.W * p->c_mid * elem_bytes(fx.dtype))
    return LAUD_ERR_UNSUPPORTED;
  return LAUD_OK;
}

// The 3x3 of a block on the active patches: `a` is set up for the plain convolution (w2 [c_mid][3][3][c_mid]);
// with `e` it runs as a group convolution (w2 [c_mid][3][3][g]; 64-channel output tiles read their own 64 input
// channels).
static int launch_conv2(int dtype, GemmArgs a, const laud_group_se* e, long long cap_rows, hipStream_t st) {
  if (!e) return launch_gemm<M_CONV2>(dtype, a, cap_rows, 1, st);
  a.gw = e->group_width;
  a.ldw = 9 * e->group_width;
  StageScope scope(LAUD_STAGE_CONV2, st);
  return dtype == LAUD_BF16 ? launch_gemm_t<M_G2, bf16_t, 64, 64, 2>(a, cap_rows, 1, st)
                            : launch_gemm_t<M_G2, float, 64, 64, 2>(a, cap_rows, 1, st);
}

// Whether conv2 -> conv3 -> residual add run as the one kernel of laud_tail.hip (h2 stays in LDS), and whether
// the dense first 1x1 (+ masker projection) runs as the kernel of laud_head.hip.
static bool tail_wanted(int dtype, const laud_bottleneck* p, const laud_group_se* e) {
#ifdef LAUD_TAIL_OFF
  return false;
#endif
  return !e && tail_supported(dtype, p->c_mid, p->c_out);
}
static bool head_wanted(int dtype, const laud_bottleneck* p) {
#ifdef LAUD_TAIL_OFF
  return false;
#endif
  return head_supported(dtype, p->c_in, p->c_mid);
}
// Where the two parts lie in a block's packed weights (laud_pack_weights, or the workspace copy of a call).
struct PackedLayout { size_t head, tail, bytes; };
static PackedLayout packed_layout(int dtype, const laud_bottleneck* p) {
  PackedLayout L{0, 0, 0};
  if (head_wanted(dtype, p)) L.bytes += head_packed_bytes(p->c_in);
  L.tail = L.bytes;
  if (tail_wanted(dtype, p, nullptr)) L.bytes += tail_packed_bytes(p->c_mid, p->c_out);
  return L;
}
static int pack_weights_into(int dtype, const laud_bottleneck* p, void* packed, bool head, bool tail, hipStream_t st) {
  const PackedLayout L = packed_layout(dtype, p);
  int rc = LAUD_OK;
  if (head && head_wanted(dtype, p)) rc = launch_head_pack(p->w1, p->c_in, (char*)packed + L.head, st);
  if (rc == LAUD_OK && tail && tail_wanted(dtype, p, nullptr))
    rc = launch_tail_pack(p->w2, p->w3, p->c_out, (char*)packed + L.tail, st);
  return rc;
}
// ... and then the first 1x1's launch carries the re-ordering of w2 / w3 for it in spare workgroups.
static void attach_tail_pack(GemmArgs& a, int dtype, const laud_bottleneck* p, const laud_group_se* e, void* wpack) {
  a.pk_out = nullptr;
  if (!tail_wanted(dtype, p, e) || p->packed) return;
  a.pk_w2 = p->w2; a.pk_w3 = p->w3; a.pk_out = (char*)wpack + packed_layout(dtype, p).tail;
  a.pk_chunks = tail::packed_slices(p->c_out) * tail::kSliceChunks;
}

// The first 1x1 over the dilated active set (rows = pixel ids from the per-group lists) with the register-weight
// kernel; without caller-packed weights both packed parts are made here, ahead of it.
static int launch_sparse_head(int dtype, const laud_bottleneck* p, const void* x, void* h1, const int32_t* pix,
                              const int32_t* need_counts, int group_rows, int ngroups, void* wpack, hipStream_t st) {
  int rc;
  if (!p->packed && (rc = pack_weights_into(dtype, p, wpack, true, true, st)) != LAUD_OK) return rc;
  HeadArgs h{};
  h.x = x; h.wpacked = (const char*)(p->packed ? p->packed : wpack) + packed_layout(dtype, p).head;
  h.s1 = p->s1; h.t1 = p->t1; h.h1 = h1; h.m_rows = ngroups; h.K = p->c_in;
  h.list = pix; h.counts = need_counts; h.group_rows = group_rows;
  return launch_head(h, st);
}

// conv2 -> conv3 -> residual add as one kernel where laud_tail.hip covers the shape (h2 stays in LDS).
// Returns 1 when that kernel was launched (*rc = its status), 0 when the caller has to run the two GEMMs.
static int try_tail(int dtype, const laud_bottleneck* p, const laud_group_se* e, const void* h1, const void* res,
                    void* out, const int32_t* idx, const int32_t* count, int H, int W, int S, int stride, int Ho, int Wo,
                    long long cap_rows, void* wpack, hipStream_t st, int* rc) {
  if (!tail_wanted(dtype, p, e)) return 0;
  TailArgs t{};
  t.h1 = h1; t.wpacked = (const char*)(p->packed ? p->packed : wpack) + packed_layout(dtype, p).tail; t.s2 = p->s2; t.t2 = p->t2; t.s3 = p->s3; t.t3 = p->t3;
  t.res = res; t.out = out; t.count = count; t.list = idx; t.H = H; t.W = W; t.S = S; t.stride = stride;
  t.Ho = Ho; t.Wo = Wo; t.cout = p->c_out; t.relu = p->relu_out ? 1 : 0;
  t.cap_patches = (int)(cap_rows / ((long long)S * S));
  *rc = launch_tail(t, cap_rows, st);
  return 1;
}

// The spatially adaptive block on an index list; `e` adds the group convolution / SE variant (or is null).
static int run_dyn_block(const void* x, laud_fmap fx, const laud_bottleneck* p, const laud_group_se* e, int S,
                         const int32_t* idx, const int32_t* count, void* out, void* ws, size_t ws_bytes,
                         void* stream) {
  int rc = validate_block(x, fx, p, out);
  if (rc != LAUD_OK) return rc;
  if (!idx || !count || S <= 0 || fx.H % S || fx.W % S) return LAUD_ERR_INVALID_ARG;
  const int Hp = fx.H / S, Wp = fx.W / S;
  if ((size_t)Hp * Wp > 60000) return LAUD_ERR_UNSUPPORTED;  // per-sample patch mask lives in LDS
  if (e && (rc = validate_group_se(p, e, fx)) != LAUD_OK) return rc;
  const DynWs L = dyn_ws_layout(fx, p->c_mid);
  if (!ws || ws_bytes < L.bytes) return LAUD_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  char* wsb = (char*)ws;
  int32_t* need_counts = (int32_t*)(wsb + L.need_counts);
  int32_t* pix = (int32_t*)(wsb + L.pix);
  void* h1 = wsb + L.h1;
  void* h2 = wsb + L.h2;
  const long long npix = (long long)fx.N * fx.H * fx.W;
  const int cpp = (int)((size_t)fx.C * elem_bytes(fx.dtype) / 16);

  if (x != out) {
    StageScope scope(LAUD_STAGE_COPY_INACTIVE, st);
    hipLaunchKernelGGL(k_copy_inactive, dim3((unsigned)(fx.N * Hp * Wp)), dim3(256), 0, st, (const uint4*)x,
                       (uint4*)out, fx.H, fx.W, S, cpp, idx, count);
    if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;
  }
  // samples per group of the dilated pixel lists: about 1.5k pixels, so that a group's ragged last
  // conv1 tile wastes little, and its patch masks fit in LDS
  const int hw = fx.H * fx.W, pps = Hp * Wp;
  int gs = (1536 + hw - 1) / hw;
  if (gs > fx.N) gs = fx.N;
  while (gs > 1 && (size_t)gs * pps > 60000) --gs;
  const int ngroups = (fx.N + gs - 1) / gs;
  {
    StageScope scope(LAUD_STAGE_NEED, st);
    hipLaunchKernelGGL(k_need, dim3(ngroups), dim3(kNeedThreads), align_up((size_t)gs * pps, 16), st, idx, count,
                       fx.N, fx.H, fx.W, S, 1, fx.H, fx.W, gs, need_counts, pix);
  }
  if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;

  GemmArgs a{};
  a.H = fx.H; a.W = fx.W; a.S = S; a.D = 1; a.G = 1; a.cmask = nullptr;
  // conv1: gathered 1x1 over the dilated active set -> h1 at pixel positions
  a.A = x; a.Wt = p->w1; a.scale = p->s1; a.shift = p->t1; a.Out = h1; a.Res = nullptr;
  a.count = need_counts; a.list = pix; a.group_rows = gs * hw; a.K = p->c_in; a.ldw = p->c_in; a.Ncols = p->c_mid;
  a.lda = p->c_in; a.ldo = p->c_mid; a.relu = 1;
  if (!e && head_wanted(fx.dtype, p)) {
    if ((rc = launch_sparse_head(fx.dtype, p, x, h1, pix, need_counts, gs * hw, ngroups, wsb + L.wpack, st)) != LAUD_OK) return rc;
  } else {
    attach_tail_pack(a, fx.dtype, p, e, wsb + L.wpack);
    if ((rc = launch_gemm<M_CONV1>(fx.dtype, a, (long long)gs * hw, ngroups, st)) != LAUD_OK) return rc;
    a.pk_out = nullptr;
  }
  if (try_tail(fx.dtype, p, e, h1, x, out, idx, count, fx.H, fx.W, S, 1, fx.H, fx.W, npix, wsb + L.wpack, st, &rc)) return rc;
  // conv2: 3x3 over active patches, A rows fetched from h1 by index -> dense h2
  a.A = h1; a.Wt = p->w2; a.scale = p->s2; a.shift = p->t2; a.Out = h2;
  a.count = count; a.list = idx; a.K = p->c_mid; a.ldw = 9 * p->c_mid; a.Ncols = p->c_mid;
  a.lda = p->c_mid; a.ldo = p->c_mid;
  if ((rc = launch_conv2(fx.dtype, a, e, npix, st)) != LAUD_OK) return rc;
  if (e && e->se_width > 0 &&
      (rc = launch_se(fx.dtype, fx.N, Hp * Wp, S * S, p->c_mid, e, h2, idx, count, (float*)h1, npix, st)) != LAUD_OK)
    return rc;
  // conv3: 1x1 on dense h2 with the scatter-add epilogue
  a.A = h2; a.Wt = p->w3; a.scale = p->s3; a.shift = p->t3; a.Out = out; a.Res = x;
  a.K = p->c_mid; a.ldw = p->c_mid; a.Ncols = p->c_out; a.lda = p->c_mid; a.ldo = p->c_out;
  a.relu = p->relu_out ? 1 : 0;
  return launch_gemm<M_CONV3>(fx.dtype, a, npix, 1, st);
}

extern "C" int laud_dyn_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p, int S, const int32_t* idx,
                                   const int32_t* count, void* out, void* ws, size_t ws_bytes, void* stream) {
  return run_dyn_block(x, fx, p, nullptr, S, idx, count, out, ws, ws_bytes, stream);
}

extern "C" int laud_dyn_group_se_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p,
                                            const laud_group_se* e, int S, const int32_t* idx, const int32_t* count,
                                            void* out, void* ws, size_t ws_bytes, void* stream) {
  if (!e) return LAUD_ERR_INVALID_ARG;
  return run_dyn_block(x, fx, p, e, S, idx, count, out, ws, ws_bytes, stream);
}

extern "C" int laud_masker_dyn_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p, int S,
                                          const float* w, float bias, const uint8_t* keep, uint8_t* mask,
                                          int32_t* idx, int32_t* count, int32_t* sample_offsets, float* logits,
                                          void* out, void* ws, size_t ws_bytes, void* stream) {
  int rc = validate_block(x, fx, p, out);
  if (rc != LAUD_OK) return rc;
  if (!w || !mask || !idx || !count || S <= 0 || fx.H % S || fx.W % S) return LAUD_ERR_INVALID_ARG;
  if (p->c_in > 4096) return LAUD_ERR_UNSUPPORTED;  // masker weights are held in LDS by conv1
  const int Hp = fx.H / S, Wp = fx.W / S;
  const DynWs L = dyn_ws_layout(fx, p->c_mid);
  if (!ws || ws_bytes < L.bytes) return LAUD_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  char* wsb = (char*)ws;
  float* proj = (float*)(wsb + L.pix);  // the pixel-list region is free in this variant
  void* h1 = wsb + L.h1;
  void* h2 = wsb + L.h2;
  const long long npix = (long long)fx.N * fx.H * fx.W;
  const int cpp = (int)((size_t)fx.C * elem_bytes(fx.dtype) / 16);

  GemmArgs a{};
  a.H = fx.H; a.W = fx.W; a.S = S; a.D = 1; a.G = 1; a.cmask = nullptr;
  // conv1 on every pixel + per-pixel masker projection, one read of x
  a.A = x; a.Wt = p->w1; a.scale = p->s1; a.shift = p->t1; a.Out = h1; a.Res = nullptr;
  a.count = nullptr; a.list = nullptr; a.K = p->c_in; a.ldw = p->c_in; a.Ncols = p->c_mid;
  a.lda = p->c_in; a.ldo = p->c_mid; a.relu = 1; a.m_rows = (int)npix; a.wmask = w; a.proj = proj;
  if (head_wanted(fx.dtype, p)) {
    // register-weight kernel; without caller-packed weights both parts are re-ordered here, ahead of it
    if (!p->packed && (rc = pack_weights_into(fx.dtype, p, wsb + L.wpack, true, true, st)) != LAUD_OK) return rc;
    HeadArgs h{};
    h.x = x; h.wpacked = (const char*)(p->packed ? p->packed : wsb + L.wpack) + packed_layout(fx.dtype, p).head;
    h.s1 = p->s1; h.t1 = p->t1; h.h1 = h1; h.m_rows = (int)npix; h.K = p->c_in; h.wmask = w; h.proj = proj;
    if (keep != nullptr && logits == nullptr) {
      // layer gate: the first 1x1 (and the projection) run on the kept samples only -- ordered compaction of the
      // gates, then rows = pixels of the listed samples.  (With `logits` wanted every sample's projection is needed.)
      int32_t* slist = (int32_t*)(wsb + L.need_counts);
      int32_t* scount = (int32_t*)(wsb + L.scnt);
      if ((rc = launch_compact(keep, fx.N, slist, scount, nullptr, 1, (int32_t*)(wsb + L.blocks), st)) != LAUD_OK) return rc;
      h.slist = slist; h.scount = scount; h.scap = fx.N; h.hw = fx.H * fx.W;
    }
    if ((rc = launch_head(h, st)) != LAUD_OK) return rc;
  } else {
    attach_tail_pack(a, fx.dtype, p, nullptr, wsb + L.wpack);
    if ((rc = launch_gemm<M_DENSE1>(fx.dtype, a, npix, 1, st)) != LAUD_OK) return rc;
    a.pk_out = nullptr;
  }
  // pooled logits -> threshold -> ascending index list (device-side count)
  if ((rc = launch_pool_compact(proj, fx.N, fx.H, fx.W, S, bias, keep, mask, logits, idx, count, sample_offsets,
                                (int32_t*)(wsb + L.blocks), st)) != LAUD_OK)
    return rc;
  if (x != out) {
    StageScope scope(LAUD_STAGE_COPY_INACTIVE, st);
    hipLaunchKernelGGL(k_copy_inactive, dim3((unsigned)(fx.N * Hp * Wp)), dim3(256), 0, st, (const uint4*)x,
                       (uint4*)out, fx.H, fx.W, S, cpp, idx, count);
    if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;
  }
  a.wmask = nullptr; a.proj = nullptr;
  if (try_tail(fx.dtype, p, nullptr, h1, x, out, idx, count, fx.H, fx.W, S, 1, fx.H, fx.W, npix, wsb + L.wpack, st, &rc)) return rc;
  // conv2 and conv3 exactly as in laud_dyn_bottleneck
  a.A = h1; a.Wt = p->w2; a.scale = p->s2; a.shift = p->t2; a.Out = h2;
  a.count = count; a.list = idx; a.K = p->c_mid; a.ldw = 9 * p->c_mid; a.Ncols = p->c_mid;
  a.lda = p->c_mid; a.ldo = p->c_mid;
  if ((rc = launch_gemm<M_CONV2>(fx.dtype, a, npix, 1, st)) != LAUD_OK) return rc;
  a.A = h2; a.Wt = p->w3; a.scale = p->s3; a.shift = p->t3; a.Out = out; a.Res = x;
  a.K = p->c_mid; a.ldw = p->c_mid; a.Ncols = p->c_out; a.lda = p->c_mid; a.ldo = p->c_out;
  a.relu = p->relu_out ? 1 : 0;
  return launch_gemm<M_CONV3>(fx.dtype, a, npix, 1, st);
}

// Unfused schedule, step 3 (Sec. 3.1): out[pixel] = act(x[pixel] + f[row]) for every pixel of every
// active patch; one wave per pixel row, 16-byte chunks.
template <typename ET>
__global__ __launch_bounds__(256) void k_scatter_add(const float* __restrict__ f, const ET* x, ET* out, int H, int W,
                                                     int S, int C, int relu, const int32_t* __restrict__ idx,
                                                     const int32_t* __restrict__ count, long long cap_rows) {
  constexpr int EPC = elem<ET>::per16;
  const long long rho = (long long)blockIdx.x * 4 + threadIdx.x / kWave;
  if (rho >= cap_rows) return;
  const int SS = S * S, p = (int)(rho / SS), j = (int)(rho - (long long)p * SS);
  if (p >= *count) return;
  const int Hp = H / S, Wp = W / S;
  const int q = idx[p];
  const int n = q / (Hp * Wp), r2 = q - n * (Hp * Wp);
  const size_t pix = ((size_t)n * H + (r2 / Wp) * S + j / S) * W + (r2 % Wp) * S + j % S;
  for (int c = lane_id() * EPC; c < C; c += kWave * EPC) {
    const float* fp = f + (size_t)rho * C + c;
    uint4 xv = *reinterpret_cast<const uint4*>(x + pix * C + c);
    ET xe[EPC], oe[EPC];
    float fe[EPC];
#pragma unroll
    for (int u = 0; u < EPC / 4; ++u) {
      const float4 t4 = reinterpret_cast<const float4*>(fp)[u];
      fe[4 * u] = t4.x; fe[4 * u + 1] = t4.y; fe[4 * u + 2] = t4.z; fe[4 * u + 3] = t4.w;
    }
    __builtin_memcpy(xe, &xv, 16);
#pragma unroll
    for (int e = 0; e < EPC; ++e) {
      float v = elem<ET>::load(&xe[e]) + fe[e];
      if (relu) v = fmaxf(v, 0.f);
      elem<ET>::store(&oe[e], v);
    }
    uint4 ov;
    __builtin_memcpy(&ov, oe, 16);
    *reinterpret_cast<uint4*>(out + pix * C + c) = ov;
  }
}

struct UnfusedWs { size_t xg, h1g, h2g, fg, bytes; };
static UnfusedWs unfused_ws_layout(const laud_fmap& fx, int c_mid, int S) {
  const size_t eb = elem_bytes(fx.dtype), E = (size_t)S + 2;
  const size_t npatch = (size_t)fx.N * (fx.H / S) * (fx.W / S), npix = (size_t)fx.N * fx.H * fx.W;
  UnfusedWs w;
  size_t o = 0;
  w.xg = o;  o += align_up(npatch * E * E * fx.C * eb, 256);
  w.h1g = o; o += align_up(npatch * E * E * c_mid * eb, 256);
  w.h2g = o; o += align_up(npix * c_mid * eb, 256);
  w.fg = o;  o += align_up(npix * fx.C * sizeof(float), 256);  // branch output stays float32
  w.bytes = o;
  return w;
}

extern "C" size_t laud_dyn_bottleneck_unfused_workspace(laud_fmap fx, const laud_bottleneck* p, int S) {
  if (!valid_fmap(fx) || !p || p->c_mid <= 0 || S <= 0 || fx.H % S || fx.W % S) return 0;
  return unfused_ws_layout(fx, p->c_mid, S).bytes;
}

extern "C" int laud_dyn_bottleneck_unfused(const void* x, laud_fmap fx, const laud_bottleneck* p, int S,
                                           const int32_t* idx, const int32_t* count, void* out, void* ws,
                                           size_t ws_bytes, void* stream) {
  int rc = validate_block(x, fx, p, out);
  if (rc != LAUD_OK) return rc;
  if (!idx || !count || S <= 0 || fx.H % S || fx.W % S) return LAUD_ERR_INVALID_ARG;
  const int Hp = fx.H / S, Wp = fx.W / S, E = S + 2;
  const long long npatch = (long long)fx.N * Hp * Wp, npix = (long long)fx.N * fx.H * fx.W;
  if (npatch * E * E > 0x7fffffffLL / 2) return LAUD_ERR_UNSUPPORTED;
  if (operand_too_big(npatch * E * E, fx.C > p->c_mid ? fx.C : p->c_mid, fx.dtype)) return LAUD_ERR_UNSUPPORTED;
  const UnfusedWs L = unfused_ws_layout(fx, p->c_mid, S);
  if (!ws || ws_bytes < L.bytes) return LAUD_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  char* wsb = (char*)ws;
  void *xg = wsb + L.xg, *h1g = wsb + L.h1g, *h2g = wsb + L.h2g, *fg = wsb + L.fg;
  const int cpp = (int)((size_t)fx.C * elem_bytes(fx.dtype) / 16);
  // step 1: gather (stand-alone kernel, zero fill outside the image)
  if ((rc = laud_gather_patches(x, fx, S, 1, idx, count, xg, stream)) != LAUD_OK) return rc;
  if (x != out) {
    StageScope scope(LAUD_STAGE_COPY_INACTIVE, st);
    hipLaunchKernelGGL(k_copy_inactive, dim3((unsigned)npatch), dim3(256), 0, st, (const uint4*)x, (uint4*)out, fx.H,
                       fx.W, S, cpp, idx, count);
    if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;
  }
  // step 2: the three convolutions on the gathered tiles
  GemmArgs a{};
  a.H = fx.H; a.W = fx.W; a.S = S; a.D = 1; a.G = 1; a.cmask = nullptr; a.count = count; a.list = idx;
  a.A = xg; a.Wt = p->w1; a.scale = p->s1; a.shift = p->t1; a.Out = h1g; a.Res = nullptr;
  a.K = p->c_in; a.ldw = p->c_in; a.Ncols = p->c_mid; a.lda = p->c_in; a.ldo = p->c_mid; a.relu = 1;
  if ((rc = launch_gemm<M_U1>(fx.dtype, a, npatch * E * E, 1, st)) != LAUD_OK) return rc;
  a.A = h1g; a.Wt = p->w2; a.scale = p->s2; a.shift = p->t2; a.Out = h2g;
  a.K = p->c_mid; a.ldw = 9 * p->c_mid; a.Ncols = p->c_mid; a.lda = p->c_mid; a.ldo = p->c_mid;
  if ((rc = launch_gemm<M_U2>(fx.dtype, a, npix, 1, st)) != LAUD_OK) return rc;
  a.A = h2g; a.Wt = p->w3; a.scale = p->s3; a.shift = p->t3; a.Out = fg;
  a.K = p->c_mid; a.ldw = p->c_mid; a.Ncols = p->c_out; a.lda = p->c_mid; a.ldo = p->c_out; a.relu = 0;
  if ((rc = launch_gemm<M_U3>(fx.dtype, a, npix, 1, st)) != LAUD_OK) return rc;
  // step 3: scatter + residual add
  {
    StageScope scope(LAUD_STAGE_SCATTER, st);
    const unsigned blocks = (unsigned)((npix + 3) / 4);
    if (fx.dtype == LAUD_BF16)
      hipLaunchKernelGGL((k_scatter_add<bf16_t>), dim3(blocks), dim3(256), 0, st, (const float*)fg, (const bf16_t*)x,
                         (bf16_t*)out, fx.H, fx.W, S, fx.C, p->relu_out ? 1 : 0, idx, count, npix);
    else
      hipLaunchKernelGGL((k_scatter_add<float>), dim3(blocks), dim3(256), 0, st, (const float*)fg, (const float*)x,
                         (float*)out, fx.H, fx.W, S, fx.C, p->relu_out ? 1 : 0, idx, count, npix);
  }
  return check_launch();
}

// ------------------------------------------------------------------------------------------------
// static first block of a stage (projection shortcut, optional stride on the 3x3)
// ------------------------------------------------------------------------------------------------
extern "C" size_t laud_static_bottleneck_workspace(laud_fmap fx, const laud_bottleneck* p, int stride) {
  if (!valid_fmap(fx) || !p || p->c_mid <= 0 || (stride != 1 && stride != 2)) return 0;
  const size_t eb = elem_bytes(fx.dtype), npix = (size_t)fx.N * fx.H * fx.W;
  const size_t nout = (size_t)fx.N * ((fx.H - 1) / stride + 1) * ((fx.W - 1) / stride + 1);
  return align_up(npix * p->c_mid * eb, 256) + align_up(nout * p->c_mid * eb, 256);
}

extern "C" int laud_static_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p, const void* w_sc,
                                      const float* s_sc, const float* t_sc, int stride, void* out, void* ws,
                                      size_t ws_bytes, void* stream) {
  if (!x || !out || !p || !w_sc || !s_sc || !t_sc || !valid_fmap(fx) || x == out) return LAUD_ERR_INVALID_ARG;
  if (!p->w1 || !p->w2 || !p->w3 || !p->s1 || !p->t1 || !p->s2 || !p->t2 || !p->s3 || !p->t3)
    return LAUD_ERR_INVALID_ARG;
  if (p->c_in != fx.C || p->c_mid <= 0 || p->c_out <= 0 || (stride != 1 && stride != 2)) return LAUD_ERR_INVALID_ARG;
  if (p->c_in % 8 || p->c_mid % 8 || p->c_out % 8) return LAUD_ERR_UNSUPPORTED;
  const int Ho = (fx.H - 1) / stride + 1, Wo = (fx.W - 1) / stride + 1;  // 3x3 pad 1 and 1x1 pad 0 agree on this
  const long long npix = (long long)fx.N * fx.H * fx.W, nout = (long long)fx.N * Ho * Wo;
  if (npix > 0x7fffffffLL / 2) return LAUD_ERR_UNSUPPORTED;
  if (operand_too_big(npix, p->c_in > p->c_mid ? p->c_in : p->c_mid, fx.dtype, fx.W)) return LAUD_ERR_UNSUPPORTED;
  if (misaligned16(x) || misaligned16(out) || misaligned16(w_sc) || block_params_misaligned(p)) return LAUD_ERR_UNSUPPORTED;
  if (partial_overlap(x, out, (size_t)npix * fx.C * elem_bytes(fx.dtype), (size_t)nout * p->c_out * elem_bytes(fx.dtype)))
    return LAUD_ERR_INVALID_ARG;
  if (!ws || ws_bytes < laud_static_bottleneck_workspace(fx, p, stride)) return LAUD_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  void* h1 = ws;
  void* h2 = (char*)ws + align_up((size_t)npix * p->c_mid * elem_bytes(fx.dtype), 256);
  int rc;
  GemmArgs a{};
  a.H = fx.H; a.W = fx.W; a.S = 1; a.D = 1; a.G = 1; a.Ho = Ho; a.Wo = Wo;
  // shortcut: strided 1x1 + affine, straight into the output buffer
  a.A = x; a.Wt = w_sc; a.scale = s_sc; a.shift = t_sc; a.Out = out; a.K = p->c_in; a.ldw = p->c_in;
  a.Ncols = p->c_out; a.lda = p->c_in; a.ldo = p->c_out; a.relu = 0; a.stride = stride; a.m_rows = (int)nout;
  if ((rc = launch_gemm<M_SD1>(fx.dtype, a, nout, 1, st)) != LAUD_OK) return rc;
  // conv1 on every input pixel
  a.Wt = p->w1; a.scale = p->s1; a.shift = p->t1; a.Out = h1; a.Ncols = p->c_mid; a.ldo = p->c_mid; a.relu = 1;
  a.stride = 1; a.Ho = fx.H; a.Wo = fx.W; a.m_rows = (int)npix;
  if ((rc = launch_gemm<M_SD1>(fx.dtype, a, npix, 1, st)) != LAUD_OK) return rc;
  // conv2: 3x3, pad 1, the block's stride
  a.A = h1; a.Wt = p->w2; a.scale = p->s2; a.shift = p->t2; a.Out = h2; a.K = p->c_mid; a.ldw = 9 * p->c_mid;
  a.lda = p->c_mid; a.stride = stride; a.Ho = Ho; a.Wo = Wo; a.m_rows = (int)nout;
  if ((rc = launch_gemm<M_SD2>(fx.dtype, a, nout, 1, st)) != LAUD_OK) return rc;
  // conv3 + shortcut (already in `out`) + ReLU
  a.A = h2; a.Wt = p->w3; a.scale = p->s3; a.shift = p->t3; a.Out = out; a.Res = out; a.K = p->c_mid;
  a.ldw = p->c_mid; a.Ncols = p->c_out; a.ldo = p->c_out; a.relu = 1;
  return launch_gemm<M_SD3>(fx.dtype, a, nout, 1, st);
}

namespace {
struct DynProjWs { size_t need_counts, pix, h1, h2, wpack, bytes; };
DynProjWs dyn_proj_ws_layout(const laud_fmap& fx, int c_mid, int c_out, int stride) {
  const size_t eb = elem_bytes(fx.dtype), npix = (size_t)fx.N * fx.H * fx.W;
  const size_t nout = (size_t)fx.N * ((fx.H - 1) / stride + 1) * ((fx.W - 1) / stride + 1);
  DynProjWs w;
  size_t o = 0;
  w.need_counts = o; o += align_up((size_t)fx.N * 4, 256);
  w.pix = o;         o += align_up(npix * 4, 256);
  w.h1 = o;          o += align_up(npix * c_mid * eb, 256);
  w.h2 = o;          o += align_up(nout * c_mid * eb, 256);
  w.wpack = o;       o += (head_supported(fx.dtype, fx.C, c_mid) ? head_packed_bytes(fx.C) : 0) +
                          (tail_supported(fx.dtype, c_mid, c_out) ? tail_packed_bytes(c_mid, c_out) : 0);
  w.bytes = o;
  return w;
}
}  // namespace

extern "C" size_t laud_dyn_projection_workspace(laud_fmap fx, const laud_bottleneck* p, int stride) {
  if (!valid_fmap(fx) || !p || p->c_mid <= 0 || (stride != 1 && stride != 2)) return 0;
  return dyn_proj_ws_layout(fx, p->c_mid, p->c_out, stride).bytes;
}

// Dynamic first block of a stage; `e` adds the group convolution / SE variant (or is null).
static int run_dyn_projection(const void* x, laud_fmap fx, const laud_bottleneck* p, const laud_group_se* e,
                              const void* w_sc, const float* s_sc, const float* t_sc, int stride, int S,
                              const int32_t* idx, const int32_t* count, void* out, void* ws, size_t ws_bytes,
                              void* stream) {
  if (!x || !out || !p || !w_sc || !s_sc || !t_sc || !idx || !count || !valid_fmap(fx) || x == out)
    return LAUD_ERR_INVALID_ARG;
  if (!p->w1 || !p->w2 || !p->w3 || !p->s1 || !p->t1 || !p->s2 || !p->t2 || !p->s3 || !p->t3)
    return LAUD_ERR_INVALID_ARG;
  if (p->c_in != fx.C || p->c_mid <= 0 || p->c_out <= 0 || (stride != 1 && stride != 2) || S <= 0)
    return LAUD_ERR_INVALID_ARG;
  if (p->c_in % 8 || p->c_mid % 8 || p->c_out % 8) return LAUD_ERR_UNSUPPORTED;
  const int Ho = (fx.H - 1) / stride + 1, Wo = (fx.W - 1) / stride + 1;
  if (Ho % S || Wo % S) return LAUD_ERR_INVALID_ARG;
  const int Hp = Ho / S, Wp = Wo / S;
  if ((size_t)Hp * Wp > 60000) return LAUD_ERR_UNSUPPORTED;  // per-sample patch mask lives in LDS
  const long long npix = (long long)fx.N * fx.H * fx.W, nout = (long long)fx.N * Ho * Wo;
  if (npix > 0x7fffffffLL / 2) return LAUD_ERR_UNSUPPORTED;
  if (operand_too_big(npix, p->c_in > p->c_mid ? p->c_in : p->c_mid, fx.dtype, fx.W)) return LAUD_ERR_UNSUPPORTED;
  if (misaligned16(x) || misaligned16(out) || misaligned16(w_sc) || block_params_misaligned(p)) return LAUD_ERR_UNSUPPORTED;
  if (partial_overlap(x, out, (size_t)npix * fx.C * elem_bytes(fx.dtype), (size_t)nout * p->c_out * elem_bytes(fx.dtype)))
    return LAUD_ERR_INVALID_ARG;
  int rc;
  if (e && (rc = validate_group_se(p, e, fx)) != LAUD_OK) return rc;
  const DynProjWs L = dyn_proj_ws_layout(fx, p->c_mid, p->c_out, stride);
  if (!ws || ws_bytes < L.bytes) return LAUD_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  char* wsb = (char*)ws;
  int32_t* need_counts = (int32_t*)(wsb + L.need_counts);
  int32_t* pix = (int32_t*)(wsb + L.pix);
  void* h1 = wsb + L.h1;
  void* h2 = wsb + L.h2;

  GemmArgs a{};
  a.H = fx.H; a.W = fx.W; a.S = S; a.D = 1; a.G = 1; a.Ho = Ho; a.Wo = Wo; a.stride = stride;
  // shortcut on every output pixel (the skip value of locations that are not selected), activated
  // only inside inactive patches
  a.A = x; a.Wt = w_sc; a.scale = s_sc; a.shift = t_sc; a.Out = out; a.K = p->c_in; a.ldw = p->c_in;
  a.Ncols = p->c_out; a.lda = p->c_in; a.ldo = p->c_out; a.relu = p->relu_out ? 1 : 0; a.m_rows = (int)nout;
  a.list = idx; a.count = count;
  if ((rc = launch_gemm<M_SD1>(fx.dtype, a, nout, 1, st)) != LAUD_OK) return rc;

  // input pixels the branch reads: the 3x3 windows (at the block's stride) of the active output pixels
  const int hw = fx.H * fx.W, pps = Hp * Wp;
  int gs = (1536 + hw - 1) / hw;
  if (gs > fx.N) gs = fx.N;
  while (gs > 1 && (size_t)gs * pps > 60000) --gs;
  const int ngroups = (fx.N + gs - 1) / gs;
  {
    StageScope scope(LAUD_STAGE_NEED, st);
    hipLaunchKernelGGL(k_need, dim3(ngroups), dim3(kNeedThreads), align_up((size_t)gs * pps, 16), st, idx, count,
                       fx.N, fx.H, fx.W, S, stride, Ho, Wo, gs, need_counts, pix);
  }
  if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;
  // conv1 over that set -> h1 at input pixel positions
  a.Wt = p->w1; a.scale = p->s1; a.shift = p->t1; a.Out = h1; a.Res = nullptr;
  a.count = need_counts; a.list = pix; a.group_rows = gs * hw; a.Ncols = p->c_mid; a.ldo = p->c_mid; a.relu = 1;
  if (!e && head_wanted(fx.dtype, p)) {
    if ((rc = launch_sparse_head(fx.dtype, p, x, h1, pix, need_counts, gs * hw, ngroups, wsb + L.wpack, st)) != LAUD_OK) return rc;
  } else {
    attach_tail_pack(a, fx.dtype, p, e, wsb + L.wpack);
    if ((rc = launch_gemm<M_CONV1>(fx.dtype, a, (long long)gs * hw, ngroups, st)) != LAUD_OK) return rc;
    a.pk_out = nullptr;
  }
  if (try_tail(fx.dtype, p, e, h1, out, out, idx, count, fx.H, fx.W, S, stride, Ho, Wo, nout, wsb + L.wpack, st, &rc)) return rc;
  // conv2: strided 3x3 at the active output pixels -> dense h2
  a.A = h1; a.Wt = p->w2; a.scale = p->s2; a.shift = p->t2; a.Out = h2;
  a.count = count; a.list = idx; a.K = p->c_mid; a.ldw = 9 * p->c_mid; a.Ncols = p->c_mid;
  a.lda = p->c_mid; a.ldo = p->c_mid;
  if ((rc = launch_conv2(fx.dtype, a, e, nout, st)) != LAUD_OK) return rc;
  if (e && e->se_width > 0 &&
      (rc = launch_se(fx.dtype, fx.N, pps, S * S, p->c_mid, e, h2, idx, count, (float*)h1, nout, st)) != LAUD_OK)
    return rc;
  // conv3 added onto the shortcut already in `out`, at the active output pixels
  a.A = h2; a.Wt = p->w3; a.scale = p->s3; a.shift = p->t3; a.Out = out; a.Res = out;
  a.K = p->c_mid; a.ldw = p->c_mid; a.Ncols = p->c_out; a.lda = p->c_mid; a.ldo = p->c_out;
  a.relu = p->relu_out ? 1 : 0;
  return launch_gemm<M_CONV3>(fx.dtype, a, nout, 1, st);
}

extern "C" int laud_dyn_projection_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p,
                                              const void* w_sc, const float* s_sc, const float* t_sc, int stride,
                                              int S, const int32_t* idx, const int32_t* count, void* out, void* ws,
                                              size_t ws_bytes, void* stream) {
  return run_dyn_projection(x, fx, p, nullptr, w_sc, s_sc, t_sc, stride, S, idx, count, out, ws, ws_bytes, stream);
}

extern "C" int laud_dyn_group_se_projection_bottleneck(const void* x, laud_fmap fx, const laud_bottleneck* p,
                                                       const laud_group_se* e, const void* w_sc, const float* s_sc,
                                                       const float* t_sc, int stride, int S, const int32_t* idx,
                                                       const int32_t* count, void* out, void* ws, size_t ws_bytes,
                                                       void* stream) {
  if (!e) return LAUD_ERR_INVALID_ARG;
  return run_dyn_projection(x, fx, p, e, w_sc, s_sc, t_sc, stride, S, idx, count, out, ws, ws_bytes, stream);
}

extern "C" int laud_channel_skip_conv(const void* x, laud_fmap fx, const laud_bottleneck* p, const uint8_t* cmask,
                                      int D, void* out, void* ws, size_t ws_bytes, void* stream) {
  int rc = validate_block(x, fx, p, out);
  if (rc != LAUD_OK) return rc;
  if (!cmask || D <= 0 || p->c_mid % D) return LAUD_ERR_INVALID_ARG;
  if (D > kMaxGroups || fx.N > 65535) return LAUD_ERR_UNSUPPORTED;
  const CsWs L = cs_ws_layout(fx, p->c_mid);
  if (!ws || ws_bytes < L.bytes) return LAUD_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  void* h1 = (char*)ws + L.h1;
  void* h2 = (char*)ws + L.h2;
  const long long hw = (long long)fx.H * fx.W;

  // 256-wide bf16 blocks with groups of whole 64-channel slices: the register-weight first 1x1 on every pixel (h1 zeroed
  // in the groups a sample drops) and the fused 3x3 -> last 1x1 kernel over the samples ordered by mask pattern, which
  // skips the input slices of groups no row of a tile keeps and zeroes h2 in the groups a row drops.
  const int G = p->c_mid / D;
  if (tail_wanted(fx.dtype, p, nullptr) && head_wanted(fx.dtype, p) && D <= 4 && G % 64 == 0 && fx.H == fx.W &&
      fx.N <= kCsSortMaxN) {
    char* wsb = (char*)ws;
    int32_t* perm = (int32_t*)(wsb + L.perm);
    uint8_t* sbits = (uint8_t*)(wsb + L.sbits);
    uint8_t* rbits = (uint8_t*)(wsb + L.rbits);
    int32_t* cnt = (int32_t*)(wsb + L.cnt);
    hipLaunchKernelGGL(k_cs_sort, dim3(1), dim3(kCsSortThreads), 0, st, cmask, fx.N, D, perm, sbits, rbits, cnt);
    if ((rc = check_launch()) != LAUD_OK) return rc;
    if (!p->packed && (rc = pack_weights_into(fx.dtype, p, wsb + L.wpack, true, true, st)) != LAUD_OK) return rc;
    const char* packed = (const char*)(p->packed ? p->packed : wsb + L.wpack);
    const PackedLayout PL = packed_layout(fx.dtype, p);
    HeadArgs h{};
    h.x = x; h.wpacked = packed + PL.head; h.s1 = p->s1; h.t1 = p->t1; h.h1 = h1;
    h.m_rows = (int)(fx.N * hw); h.K = p->c_in; h.rbits = rbits; h.hw = (int)hw; h.cs_group = G;
    if ((rc = launch_head(h, st)) != LAUD_OK) return rc;  // (stage timing books the two kernels as conv1 / conv2)
    TailArgs t{};
    t.h1 = h1; t.wpacked = packed + PL.tail; t.s2 = p->s2; t.t2 = p->t2; t.s3 = p->s3; t.t3 = p->t3;
    t.res = x; t.out = out; t.count = cnt; t.list = perm; t.cap_patches = fx.N;
    t.H = fx.H; t.W = fx.W; t.S = fx.H; t.stride = 1; t.Ho = fx.H; t.Wo = fx.W; t.cout = p->c_out;
    t.relu = p->relu_out ? 1 : 0; t.sbits = sbits; t.cs_group = G;
    return launch_tail(t, fx.N * hw, st);
  }

  GemmArgs a{};
  a.H = fx.H; a.W = fx.W; a.S = 1; a.D = D; a.G = p->c_mid / D; a.cmask = cmask;
  a.count = nullptr; a.list = nullptr;
  // conv1 with the kept output kernels only -> compact h1
  a.A = x; a.Wt = p->w1; a.scale = p->s1; a.shift = p->t1; a.Out = h1; a.Res = nullptr;
  a.K = p->c_in; a.ldw = p->c_in; a.Ncols = p->c_mid; a.lda = p->c_in; a.ldo = p->c_mid; a.relu = 1;
  if ((rc = launch_gemm<M_CS1>(fx.dtype, a, hw, fx.N, st)) != LAUD_OK) return rc;
  // conv2 with kept input and output kernels -> compact h2
  a.A = h1; a.Wt = p->w2; a.scale = p->s2; a.shift = p->t2; a.Out = h2;
  a.K = p->c_mid; a.ldw = 9 * p->c_mid; a.Ncols = p->c_mid; a.lda = p->c_mid; a.ldo = p->c_mid;
  if ((rc = launch_gemm<M_CS2>(fx.dtype, a, hw, fx.N, st)) != LAUD_OK) return rc;
  // conv3 with the kept input kernels, residual add on every pixel
  a.A = h2; a.Wt = p->w3; a.scale = p->s3; a.shift = p->t3; a.Out = out; a.Res = x;
  a.K = p->c_mid; a.ldw = p->c_mid; a.Ncols = p->c_out; a.lda = p->c_mid; a.ldo = p->c_out;
  a.relu = p->relu_out ? 1 : 0;
  return launch_gemm<M_CS3>(fx.dtype, a, hw, fx.N, st);
}

// ------------------------------------------------------------------------------------------------
// one-time set-up and the allocation-free entry point
// ------------------------------------------------------------------------------------------------
// Scratch memory of laud_dyn_bottleneck_noalloc: a fixed array in the library's device image instead of a
// caller workspace.  Every GPU the library runs on holds its own copy at its own address until the process ends.
static __device__ __align__(256) unsigned char scratch[LAUD_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
// Device address of `scratch` per device ordinal.  In host code the array's name is only a handle for
// hipGetSymbolAddress, never an address a kernel may receive.
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Resolves (once per device, with that device current) and returns the current device's scratch array.
int scratch_of_current_device(void** out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LAUD_ERR_HIP;
  void* ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (!ptr) {
    if (hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return LAUD_ERR_HIP;
    g_scratch_ptr[dev].store(ptr, std::memory_order_release);  // threads racing here store the same address
  }
  *out = ptr;
  return LAUD_OK;
}
}  // namespace

extern "C" int laud_init(void) {
  clear_stale_error();
  void* ptr = nullptr;
  int rc = scratch_of_current_device(&ptr);
  if (rc != LAUD_OK) return rc;
  rc = gemm_init_device();
  if (rc != LAUD_OK) return rc;
  if ((rc = tail_init_device()) != LAUD_OK) return rc;
  return head_init_device();
}

extern "C" int laud_dyn_bottleneck_noalloc(const void* x, laud_fmap fx, const laud_bottleneck* p, int S,
                                           const int32_t* idx, const int32_t* count, void* out, void* stream) {
  if (!p || !valid_fmap(fx) || p->c_mid <= 0) return LAUD_ERR_INVALID_ARG;
  const size_t need = dyn_ws_layout(fx, p->c_mid).bytes;
  if (need > (size_t)LAUD_NOALLOC_SCRATCH_BYTES) return LAUD_ERR_SCRATCH_LIMIT;
  void* ptr = nullptr;
  const int rc = scratch_of_current_device(&ptr);
  if (rc != LAUD_OK) return rc;
  // Nothing in this workspace has to start at zero: every region is written before it is read within the call.
  return run_dyn_block(x, fx, p, nullptr, S, idx, count, out, ptr, (size_t)LAUD_NOALLOC_SCRATCH_BYTES, stream);
}

extern "C" size_t laud_packed_weights_size(const laud_bottleneck* p, int dtype) {
  if (!p || p->c_in <= 0 || p->c_mid <= 0 || p->c_out <= 0) return 0;
  return packed_layout(dtype, p).bytes;
}

extern "C" int laud_pack_weights(const laud_bottleneck* p, int dtype, void* packed, void* stream) {
  if (!p || !packed || !p->w1 || !p->w2 || !p->w3 || p->c_in <= 0 || p->c_mid <= 0 || p->c_out <= 0)
    return LAUD_ERR_INVALID_ARG;
  if (packed_layout(dtype, p).bytes == 0) return LAUD_ERR_UNSUPPORTED;
  if (misaligned16(packed) || block_params_misaligned(p)) return LAUD_ERR_UNSUPPORTED;
  clear_stale_error();
  return pack_weights_into(dtype, p, packed, true, true, (hipStream_t)stream);
}
