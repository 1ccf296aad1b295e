// Shared host/device helpers of the gfx950 dynamic-bottleneck library (internal header).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "laud.h"

namespace laud {

constexpr int kWave = 64;  // CDNA wavefront width

// ---- workspace carving: every sub-buffer starts on a 256-byte boundary ------------------
__host__ __device__ inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

// ---- element types -----------------------------------------------------------------------
// bf16 is stored as its 16-bit pattern; arithmetic is always float32.
typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t b) { return __uint_as_float(((uint32_t)b) << 16); }

// Round-to-nearest-even, quiet NaN preserved.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (bf16_t)0x7fc0;
  u += 0x7fffu + ((u >> 16) & 1u);
  return (bf16_t)(u >> 16);
}

template <typename ET> struct elem;
template <> struct elem<float> {
  static constexpr int per16 = 4;  // elements per 16-byte chunk
  __device__ static __forceinline__ float load(const float* p) { return *p; }
  __device__ static __forceinline__ void store(float* p, float v) { *p = v; }
};
template <> struct elem<bf16_t> {
  static constexpr int per16 = 8;
  __device__ static __forceinline__ float load(const bf16_t* p) { return bf16_to_f32(*p); }
  __device__ static __forceinline__ void store(bf16_t* p, float v) { *p = f32_to_bf16(v); }
};

// ---- wave-level primitives ---------------------------------------------------------------
__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// Number of set bits of a 64-bit ballot below the calling lane.
__device__ __forceinline__ int ballot_prefix(unsigned long long b) {
  return (int)__builtin_amdgcn_mbcnt_hi((unsigned)(b >> 32), __builtin_amdgcn_mbcnt_lo((unsigned)b, 0u));
}

// Exclusive scan of one count per wave across the (at most 64) waves of a block: every wave leaves
// its count in wsum[wave], one barrier, then each wave scans the counts with wave shuffles (no thread
// walks the list alone).  Returns the sum of the counts of the waves before this one; *total gets the
// block's sum.  wsum must not be reused by the next call before another barrier: alternate two arrays.
__device__ __forceinline__ int scan_wave_counts(int count, int nwaves, int* wsum, int* total) {
  const int lane = lane_id(), wave = (int)threadIdx.x / kWave;
  if (lane == 0) wsum[wave] = count;
  __syncthreads();
  const int v = lane < nwaves ? wsum[lane] : 0;
  int incl = v;
#pragma unroll
  for (int o = 1; o < kWave; o <<= 1) {
    const int t = __shfl_up(incl, o, kWave);
    if (lane >= o) incl += t;
  }
  *total = __shfl(incl, kWave - 1, kWave);
  return __shfl(incl - v, wave, kWave);
}

// lower_bound over a sorted list by a whole wave: 64 probes per round instead of one, so a list of n entries
// takes ceil(log64 n) dependent round trips.  Every lane of the wave must call it; all get the result.
__device__ __forceinline__ int wave_lower_bound(const int32_t* v, int n, int key) {
  const int lane = lane_id();
  int lo = 0, hi = n;  // the answer lies in [lo, hi]
  while (hi > lo) {
    const int step = (hi - lo + kWave - 1) / kWave;
    const int pos = lo + lane * step;
    const bool below = pos < hi && v[pos] < key;  // true for a prefix of the lanes (sorted list)
    const int c = __popcll(__ballot(below));
    if (c == 0) {
      hi = lo;
    } else {
      const int nhi = min(lo + c * step, hi);
      lo = lo + (c - 1) * step + 1;
      hi = nhi;
    }
  }
  return lo;
}

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

__device__ __forceinline__ int wave_sum_int(int v) {
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

// ---- host-side launch checking -----------------------------------------------------------
// hipGetLastError() reports (and clears) the last error of ANY earlier HIP call of the thread,
// the caller's included; each entry point clears that state once, after validation and before
// its first launch, so that check_launch() sees only the library's own launches.
inline void clear_stale_error() { (void)hipGetLastError(); }
inline int check_launch() { return hipGetLastError() == hipSuccess ? LAUD_OK : LAUD_ERR_HIP; }

inline bool valid_fmap(const laud_fmap& f) {
  return f.N > 0 && f.H > 0 && f.W > 0 && f.C > 0 && (f.dtype == LAUD_F32 || f.dtype == LAUD_BF16);
}
inline size_t elem_bytes(int dtype) { return dtype == LAUD_BF16 ? 2 : 4; }

// Compaction works on blocks of this many mask bytes.
constexpr int kCompactBlock = 4096;
inline size_t compact_ws_bytes(long long n) {
  long long nb = (n + kCompactBlock - 1) / kCompactBlock;
  return align_up((size_t)(nb > 0 ? nb : 1) * sizeof(int32_t), 256);
}

// Launches the ordered compaction of `n` mask bytes on `stream` (see laud_mask.hip).
int launch_compact(const uint8_t* mask, int n, int32_t* idx, int32_t* count, int32_t* sample_offsets,
                   int per_sample, int32_t* block_counts, hipStream_t stream);

// Pools a per-pixel masker projection over S x S patches, thresholds, and launches the ordered
// compaction (one launch for small patch counts); see laud_mask.hip.
int launch_pool_compact(const float* proj, int N, int H, int W, int S, float bias, const uint8_t* keep, uint8_t* mask,
                        float* logits, int32_t* idx, int32_t* count, int32_t* sample_offsets, int32_t* block_counts,
                        hipStream_t stream);

// Dense GEMM + per-column affine (+ ReLU) on the MFMA kernels of laud_gemm.hip:
// Out[r][c] = act(scale[c] * sum_k A[r][k] * Wt[c][k] + shift[c]), A [rows][K], Wt [ncols][K], all of `dtype`.
int launch_dense_affine(int dtype, const void* A, const void* Wt, const float* scale, const float* shift, void* Out,
                        long long rows, int K, int ncols, int relu, hipStream_t stream);

// The SE module on the compact rows h2 [rows][C] of the active patches (pps patches per sample, SS pixels per
// patch, at most cap_rows rows); see laud_se.hip.  `scratch` holds N*(2*C + se_width) floats.
constexpr int kSeMaxC = 4096, kSeMaxHidden = 1024;  // widest layer / SE hidden layer the kernels keep in LDS
int launch_se(int dtype, int N, int pps, int SS, int C, const laud_group_se* e, void* h2, const int32_t* idx,
              const int32_t* count, float* scratch, long long cap_rows, hipStream_t stream);

// conv2 -> conv3 -> residual add in one kernel (laud_tail.hip), for the shapes tail_supported() names.
struct TailArgs {
  const void* h1;        // [pixels of the input grid][MID] bf16, conv1's output at pixel positions
  const void* wpacked;   // w2 and w3 in MFMA fragment order (launch_tail_pack), tail_packed_bytes() bytes
  const float* s2; const float* t2;  // [MID]
  const float* s3; const float* t3;  // [cout]
  const void* res;       // residual [output pixels][cout] (x, or the shortcut already in `out`)
  void* out;             // [output pixels][cout]; may alias res
  const int32_t* count;  // device: number of active patches
  const int32_t* list;   // device: ascending active patch ids
  int cap_patches;       // capacity of `list` (number of patches of the grid), > 0
  int H, W;              // input grid of h1
  int S;                 // patch size on the output grid
  int stride, Ho, Wo;    // spatial stride of the 3x3 and the output grid (stride 1: Ho = H, Wo = W)
  int cout;
  int relu;
  int pb;                // tile height in blocks of 32 pixels (1..3); 0 = chosen on the device from the count
  // channel skipping (Fig. 2(c)) on whole samples (S = H: a "patch" is a sample, `list` the samples in processing
  // order): sbits[i] = kept channel groups (bit g) of the i-th sample of the list, cs_group = channels per group (a
  // multiple of 64).  Input slices of groups no row of a tile keeps are skipped in the 3x3, and h2 is zeroed in the
  // groups a row drops.  Null: no channel mask.
  const uint8_t* sbits;
  int cs_group;
  int wg_target;         // workgroups that fill the device once (its compute units; set by launch_tail)
};

bool tail_supported(int dtype, int c_mid, int c_out);
int tail_init_device();
size_t tail_packed_bytes(int c_mid, int c_out);
// re-orders w2 [c_mid][3][3][c_mid] and w3 [c_out][c_mid] into the order the fused kernel streams them
int launch_tail_pack(const void* w2, const void* w3, int c_out, void* packed, hipStream_t stream);
// cap_rows: upper bound of the number of active pixels (grid size); the count itself stays on the device
int launch_tail(const TailArgs& a, long long cap_rows, hipStream_t stream);

// conv1 on every pixel (+ masker projection) with register-resident weights (laud_head.hip), for head_supported() shapes.
struct HeadArgs {
  const void* x;         // [m_rows][K] bf16
  const void* wpacked;   // w1 in MFMA fragment order (launch_head_pack), head_packed_bytes() bytes
  const float* s1; const float* t1;  // [256]
  void* h1;              // [m_rows][256] bf16
  int m_rows, K;
  const float* wmask;    // masker weights [K] or null
  float* proj;           // [m_rows] per-pixel projection (with wmask)
  // sparse form (the gather fused into the first 1x1): rows are pixel ids taken from per-group lists; list == null: dense
  const int32_t* list;   // [ngroups][group_rows] ascending pixel ids of the dilated active set
  const int32_t* counts; // [ngroups] device: valid entries per group
  int group_rows;        // capacity of one group's list
  // rows = the pixels of listed samples (layer gate ahead of a spatially static first 1x1): slist [scap] ascending kept
  // sample ids, *scount of them valid (device), hw pixels per sample; m_rows = scap * hw is the capacity.  Null: all rows.
  const int32_t* slist;
  const int32_t* scount;
  int scap;
  // channel skipping: rbits[n] = kept channel groups (bit g) of sample n, hw = pixels per sample, cs_group = channels per
  // group (a multiple of 32); h1 is written as zero in the groups a row's sample drops.  Null: no channel mask.
  const uint8_t* rbits;
  int hw, cs_group;
  int pb;                // tile height in blocks of 32 pixels (2 or 4); 0 = chosen by launch_head (dense rows) or on the device (lists)
  int wg_target;         // workgroups that fill the device once (its compute units; set by launch_head)
};
bool head_supported(int dtype, int c_in, int c_mid);
int head_init_device();
size_t head_packed_bytes(int c_in);
int launch_head_pack(const void* w1, int c_in, void* packed, hipStream_t stream);
int launch_head(const HeadArgs& a, hipStream_t stream);

// Stage timing (see laud_stage_timing_enable): RAII bracket around the launches of one stage.
extern bool g_stage_timing_on;
void stage_mark(int stage, hipStream_t stream, bool begin);
struct StageScope {
  int stage;
  hipStream_t stream;
  StageScope(int s, hipStream_t st) : stage(s), stream(st) {
    if (g_stage_timing_on) stage_mark(stage, stream, true);
  }
  ~StageScope() {
    if (g_stage_timing_on) stage_mark(stage, stream, false);
  }
};

}  // namespace laud
