// Spatial masker, ordered index generation and stand-alone gather for gfx950.
//
//   k_mask_logits   Sec. 3.2 "Masker design" + App. B item 1: pooled one-channel masker,
//                   threshold at 0; HBM-bound (reads x once, 16-byte loads).
//   k_block_counts / k_compact
//                   App. B item 2: the masker emits the ascending list of active patch
//                   indices; wave64 ballot + mbcnt prefix inside a wave, LDS scan across
//                   the 16 waves of a block, per-block counts for the cross-block base.
//                   No atomics: the order is the ascending flat index, bit-exact.
//   k_gather        Sec. 3.1 step 1: copy of active patches (+1 halo) to a dense buffer.
#include "laud_common.h"

namespace laud {

// ------------------------------------------------------------------------------------------
// ordered compaction
// ------------------------------------------------------------------------------------------
constexpr int kCompactThreads = 1024;                            // 16 waves
constexpr int kCompactChunks = kCompactBlock / kCompactThreads;  // 4 sub-chunks per block

__global__ __launch_bounds__(kCompactThreads) void k_block_counts(const uint8_t* __restrict__ mask, int n,
                                                                  int32_t* __restrict__ block_counts) {
  __shared__ int wcnt[kCompactThreads / kWave];
  const int base = blockIdx.x * kCompactBlock;
  int c = 0;
#pragma unroll
  for (int k = 0; k < kCompactChunks; ++k) {
    int i = base + k * kCompactThreads + (int)threadIdx.x;
    bool f = (i < n) && mask[i] != 0;
    c += __popcll(__ballot(f));  // identical in every lane of the wave
  }
  if (lane_id() == 0) wcnt[threadIdx.x / kWave] = c;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < kCompactThreads / kWave; ++w) t += wcnt[w];
    block_counts[blockIdx.x] = t;
  }
}

// Each block recomputes its base as the sum of the counts of the blocks before it (a few
// hundred values at most), then writes its own indices in ascending order.
__global__ __launch_bounds__(kCompactThreads) void k_compact(const uint8_t* __restrict__ mask, int n,
                                                             int32_t* __restrict__ idx, int32_t* __restrict__ count,
                                                             int32_t* __restrict__ sample_offsets, int per_sample,
                                                             const int32_t* __restrict__ block_counts, int nblocks) {
  __shared__ int wsum[kCompactThreads / kWave];
  __shared__ int scan[2][kCompactThreads / kWave];
  __shared__ int s_base;
  const int wave = threadIdx.x / kWave, lane = lane_id();

  // base = sum of block_counts[0 .. blockIdx.x)
  int part = 0;
  for (int b = threadIdx.x; b < (int)blockIdx.x; b += kCompactThreads) part += block_counts[b];
#pragma unroll
  for (int o = kWave / 2; o > 0; o >>= 1) part += __shfl_xor(part, o, kWave);
  if (lane == 0) wsum[wave] = part;
  __syncthreads();
  if (threadIdx.x == 0) {
    int t = 0;
    for (int w = 0; w < kCompactThreads / kWave; ++w) t += wsum[w];
    s_base = t;
  }
  __syncthreads();
  int running = s_base;

  const int base = blockIdx.x * kCompactBlock;
  for (int k = 0; k < kCompactChunks; ++k) {
    const int i = base + k * kCompactThreads + (int)threadIdx.x;
    const bool f = (i < n) && mask[i] != 0;
    const unsigned long long b = __ballot(f);
    const int lp = ballot_prefix(b);
    int tot;
    const int wo = scan_wave_counts(__popcll(b), kCompactThreads / kWave, scan[k & 1], &tot);
    const int pos = running + wo + lp;  // number of set entries before i
    if (f) idx[pos] = i;
    if (sample_offsets && i < n && (i % per_sample) == 0) sample_offsets[i / per_sample] = pos;
    running += tot;
  }
  if ((int)blockIdx.x == nblocks - 1 && threadIdx.x == 0) {
    *count = running;
    if (sample_offsets) sample_offsets[n / per_sample] = running;
  }
}

// Small masks (a few thousand entries: one stage's patch grid, a batch of layer gates): one block
// does the whole ordered compaction in one launch.  Each thread owns four consecutive entries per
// pass; four ballots give the in-wave prefix (mbcnt), an LDS scan over the 16 waves the rest.
constexpr int kSmallCompactMax = 8 * kCompactBlock;  // 32768 entries
// Pooling of the per-pixel masker projection (Masker-Conv1x1 fusion, App. B item 1): patch logit =
// bias + mean over the S x S patch of proj; active iff logit > 0 (and the sample's gate, if any).
struct PoolArgs {
  const float* proj;    // [N*H*W] per-pixel projection, or null: the mask bytes are the input
  const uint8_t* keep;  // [N] or null
  float* logits;        // [npatch] or null
  int H, W, S;
  float bias;
};
__device__ __forceinline__ bool pooled_decision(const PoolArgs& pa, int q, uint8_t* mask) {
  const int Hp = pa.H / pa.S, Wp = pa.W / pa.S;
  const int n = q / (Hp * Wp), r = q - n * (Hp * Wp);
  const int py = r / Wp, px = r - py * Wp;
  float acc = 0.f;
  const float* base = pa.proj + ((size_t)n * pa.H + py * pa.S) * pa.W + px * pa.S;
  if (pa.S == 2) {  // all loads in flight at once; fixed summation order (row major)
    const float a0 = base[0], a1 = base[1], a2 = base[pa.W], a3 = base[pa.W + 1];
    acc = ((a0 + a1) + a2) + a3;
  } else if (pa.S == 4) {
    float v[16];
#pragma unroll
    for (int k = 0; k < 16; ++k) v[k] = base[(k >> 2) * pa.W + (k & 3)];
#pragma unroll
    for (int k = 0; k < 16; ++k) acc += v[k];
  } else {
    for (int dy = 0; dy < pa.S; ++dy)
      for (int dx = 0; dx < pa.S; ++dx) acc += base[dy * pa.W + dx];
  }
  const float logit = acc / (float)(pa.S * pa.S) + pa.bias;
  bool on = logit > 0.f;
  if (pa.keep && pa.keep[n] == 0) on = false;
  mask[q] = on ? 1 : 0;
  if (pa.logits) pa.logits[q] = logit;
  return on;
}

__global__ __launch_bounds__(256) void k_pool_mask(PoolArgs pa, int npatch, uint8_t* __restrict__ mask) {
  const int q = blockIdx.x * 256 + threadIdx.x;
  if (q < npatch) pooled_decision(pa, q, mask);
}

__global__ __launch_bounds__(kCompactThreads) void k_compact_small(const uint8_t* __restrict__ mask, int n,
                                                                   int32_t* __restrict__ idx,
                                                                   int32_t* __restrict__ count,
                                                                   int32_t* __restrict__ sample_offsets,
                                                                   int per_sample) {
  __shared__ int scan[2][kCompactThreads / kWave];
  // A thread owns entries 4*tid .. 4*tid+3 of each 4096-entry pass.  All of its mask bytes (at most eight
  // passes: n <= 32768) are requested before the first pass runs, so the kernel pays one far-memory round trip
  // instead of one per pass.
  constexpr int kMaxPass = kSmallCompactMax / (4 * kCompactThreads);
  unsigned m4[kMaxPass];
  // Every load is unconditional (clamped index, value dropped past the end): conditional loads would be waited for
  // one by one.  Whole words when the base is word-aligned and n a multiple of four (uniform), bytes otherwise.
  const bool words = (reinterpret_cast<unsigned long long>(mask) & 3ull) == 0 && (n & 3) == 0 && n > 0;
  if (words) {
#pragma unroll
    for (int p = 0; p < kMaxPass; ++p) {
      const int i0 = p * 4 * kCompactThreads + 4 * (int)threadIdx.x;
      const unsigned v = *reinterpret_cast<const unsigned*>(mask + min(i0, n - 4));
      m4[p] = i0 < n ? v : 0u;
    }
  } else if (n > 0) {
#pragma unroll
    for (int p = 0; p < kMaxPass; ++p) {
      const int i0 = p * 4 * kCompactThreads + 4 * (int)threadIdx.x;
      unsigned v = 0;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const unsigned byte = mask[min(i0 + j, n - 1)];
        v |= (i0 + j < n ? byte : 0u) << (8 * j);
      }
      m4[p] = v;
    }
  } else {
#pragma unroll
    for (int p = 0; p < kMaxPass; ++p) m4[p] = 0u;
  }
  int running = 0;
#pragma unroll
  for (int p = 0; p < kMaxPass; ++p) {
    const int base = p * 4 * kCompactThreads;
    if (base >= n) break;  // uniform
    const int i0 = base + 4 * (int)threadIdx.x;
    bool f[4];
    unsigned long long b[4];
    int before = 0, mine = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      f[j] = ((m4[p] >> (8 * j)) & 0xffu) != 0;  // entries past n were read as 0
      b[j] = __ballot(f[j]);
      before += ballot_prefix(b[j]);  // set entries of lower lanes at position j
    }
    int wtot = 0, tot;
#pragma unroll
    for (int j = 0; j < 4; ++j) wtot += __popcll(b[j]);
    const int wo = scan_wave_counts(wtot, kCompactThreads / kWave, scan[p & 1], &tot);
    int pos = running + wo + before;  // set entries before (this thread, position 0)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int i = i0 + j;
      if (sample_offsets && i < n && (i % per_sample) == 0) sample_offsets[i / per_sample] = pos + mine;
      if (f[j]) { idx[pos + mine] = i; ++mine; }
    }
    running += tot;
  }
  if (threadIdx.x == 0) {
    *count = running;
    if (sample_offsets) sample_offsets[n / per_sample] = running;
  }
}

// Pooling, threshold and ordered compaction in ONE launch for S = 2 and at most 8192 patches (a stage-3
// batch of 128 images): the two dependent kernels cost two launch-plus-far-latency chains for a few kilobytes
// of work.  One patch per thread, up to eight blocks of 1024; a block needs the number of active patches
// before its own and gets it by deciding those patches itself (at most seven more per thread: four adds and a
// compare each), so the blocks neither wait for each other nor share anything, and no block runs more than one
// compaction pass (a single block doing all passes is bound by instruction issue on its one CU).  Every
// projection read of a thread (two 8-byte loads per patch) is requested before any is used.  Same summation
// order as pooled_decision, hence the same decisions in every block.
constexpr int kPoolFusedMax = 2 * kCompactBlock;
constexpr int kPoolFusedBlocks = kPoolFusedMax / kCompactThreads;
__global__ __launch_bounds__(kCompactThreads) void k_pool_compact_s2(PoolArgs pa, int n, uint8_t* __restrict__ mask,
                                                                     int32_t* __restrict__ idx,
                                                                     int32_t* __restrict__ count,
                                                                     int32_t* __restrict__ sample_offsets,
                                                                     int per_sample) {
  __shared__ int scan[2][kCompactThreads / kWave];
  const int Hp = pa.H / 2, Wp = pa.W / 2;
  const int b = blockIdx.x, tid = threadIdx.x;
  float2 top[kPoolFusedBlocks], bot[kPoolFusedBlocks];
  int kept[kPoolFusedBlocks];
#pragma unroll
  for (int u = 0; u < kPoolFusedBlocks; ++u) {
    // slot u < b: the patch of block u at this thread's position; slots from b on: the thread's own patch
    const int q = min(min(u, b) * kCompactThreads + tid, n - 1);  // past the end: the last patch, result unused
    const int s = q / (Hp * Wp), r = q - s * (Hp * Wp);
    const int py = r / Wp, px = r - py * Wp;
    const float* base = pa.proj + ((size_t)s * pa.H + py * 2) * pa.W + px * 2;
    top[u] = *reinterpret_cast<const float2*>(base);
    bot[u] = *reinterpret_cast<const float2*>(base + pa.W);
    kept[u] = pa.keep ? (int)pa.keep[s] : 1;
  }
  int before_blocks = 0;
  bool own_on = false;
  float own_logit = 0.f;
#pragma unroll
  for (int u = 0; u < kPoolFusedBlocks; ++u) {
    const float acc = ((top[u].x + top[u].y) + bot[u].x) + bot[u].y;
    const float logit = acc / 4.0f + pa.bias;
    const bool on = logit > 0.f && kept[u] != 0;  // false for NaN
    before_blocks += (u < b && on) ? 1 : 0;         // blocks before this one are full: every slot is a patch
    if (u == b) { own_on = on; own_logit = logit; }
  }
  int base_cnt;
  (void)scan_wave_counts(wave_sum_int(before_blocks), kCompactThreads / kWave, scan[0], &base_cnt);
  const int q = b * kCompactThreads + tid;
  const bool f = q < n && own_on;
  if (q < n) {
    mask[q] = own_on ? 1 : 0;
    if (pa.logits) pa.logits[q] = own_logit;
  }
  const unsigned long long bal = __ballot(f);
  int tot;
  const int wo = scan_wave_counts(__popcll(bal), kCompactThreads / kWave, scan[1], &tot);
  const int pos = base_cnt + wo + ballot_prefix(bal);
  if (sample_offsets && q < n && (q % per_sample) == 0) sample_offsets[q / per_sample] = pos;
  if (f) idx[pos] = q;
  if (b == (int)gridDim.x - 1 && tid == 0) {
    *count = base_cnt + tot;
    if (sample_offsets) sample_offsets[n / per_sample] = base_cnt + tot;
  }
}

// The same in one launch for any S when one block holds all patches (coarse granularities: S = 7 on a 14 x 14 map
// gives 512 patches for 128 images): one patch per thread, decision by pooled_decision (so the masks are those of
// the two-launch path, bit for bit), ordered compaction with one ballot and one scan of the wave counts.
__global__ __launch_bounds__(kCompactThreads) void k_pool_compact_one_block(PoolArgs pa, int n, uint8_t* __restrict__ mask,
                                                                            int32_t* __restrict__ idx,
                                                                            int32_t* __restrict__ count,
                                                                            int32_t* __restrict__ sample_offsets,
                                                                            int per_sample) {
  __shared__ int scan[kCompactThreads / kWave];
  const int q = threadIdx.x;
  const bool on = q < n ? pooled_decision(pa, q, mask) : false;
  const unsigned long long bal = __ballot(on);
  int tot;
  const int pos = scan_wave_counts(__popcll(bal), kCompactThreads / kWave, scan, &tot) + ballot_prefix(bal);
  if (sample_offsets && q < n && (q % per_sample) == 0) sample_offsets[q / per_sample] = pos;
  if (on) idx[pos] = q;
  if (q == 0) {
    *count = tot;
    if (sample_offsets) sample_offsets[n / per_sample] = tot;
  }
}

// Ordered compaction of up to 64 x 4096 entries in ONE launch of several blocks: block b owns entries
// [4096 b, 4096 b + 4096) and first counts the set entries of all blocks before it by itself (one 4-byte load
// per thread and preceding block, eight in flight) instead of waiting for anybody: no second launch, no
// inter-block dependency, and each block's own pass runs on a CU of its own.  Needs a word-aligned mask and n a
// multiple of four (whole-word loads); the launcher checks.
constexpr int kCompactOneLaunchMax = 64 * kCompactBlock;
__global__ __launch_bounds__(kCompactThreads) void k_compact_blocks(const uint8_t* __restrict__ mask, int n,
                                                                    int32_t* __restrict__ idx,
                                                                    int32_t* __restrict__ count,
                                                                    int32_t* __restrict__ sample_offsets,
                                                                    int per_sample) {
  __shared__ int scan[2][kCompactThreads / kWave];
  const int b = blockIdx.x, tid = threadIdx.x;
  const unsigned* words = reinterpret_cast<const unsigned*>(mask);
  // own entries: 4 tid .. 4 tid + 3 of the block's range (requested first, used last)
  const int i0 = b * kCompactBlock + 4 * tid;
  const unsigned own = words[min(i0, n - 4) >> 2];
  // set entries of the blocks before this one
  int before_blocks = 0;
  for (int p0 = 0; p0 < b; p0 += 8) {
    unsigned v[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) v[u] = words[min(p0 + u, b - 1) * (kCompactBlock / 4) + tid];
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      unsigned t = (v[u] | (v[u] >> 4)) & 0x0f0f0f0fu;  // per byte: non-zero -> one bit
      t = (t | (t >> 2)) & 0x03030303u;
      t = (t | (t >> 1)) & 0x01010101u;
      before_blocks += p0 + u < b ? __popc(t) : 0;
    }
  }
  int base;
  (void)scan_wave_counts(wave_sum_int(before_blocks), kCompactThreads / kWave, scan[0], &base);
  // own pass, as in k_compact_small
  const unsigned m4 = i0 < n ? own : 0u;
  bool f[4];
  unsigned long long bal[4];
  int before = 0, mine = 0, wtot = 0, tot;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    f[j] = ((m4 >> (8 * j)) & 0xffu) != 0;
    bal[j] = __ballot(f[j]);
    before += ballot_prefix(bal[j]);
    wtot += __popcll(bal[j]);
  }
  const int wo = scan_wave_counts(wtot, kCompactThreads / kWave, scan[1], &tot);
  const int pos = base + wo + before;
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int i = i0 + j;
    if (sample_offsets && i < n && (i % per_sample) == 0) sample_offsets[i / per_sample] = pos + mine;
    if (f[j]) { idx[pos + mine] = i; ++mine; }
  }
  if (b == (int)gridDim.x - 1 && tid == 0) {
    *count = base + tot;
    if (sample_offsets) sample_offsets[n / per_sample] = base + tot;
  }
}

__global__ void k_write_zero_count(int32_t* count, int32_t* sample_offsets) {
  *count = 0;
  if (sample_offsets) sample_offsets[0] = 0;
}

int launch_compact(const uint8_t* mask, int n, int32_t* idx, int32_t* count, int32_t* sample_offsets,
                   int per_sample, int32_t* block_counts, hipStream_t stream) {
  StageScope scope(LAUD_STAGE_COMPACT, stream);
  if (n == 0) {
    hipLaunchKernelGGL(k_write_zero_count, dim3(1), dim3(1), 0, stream, count, sample_offsets);
    return check_launch();
  }
  if (n > kCompactBlock && n <= kCompactOneLaunchMax && (n & 3) == 0 &&
      (reinterpret_cast<unsigned long long>(mask) & 3ull) == 0) {
    hipLaunchKernelGGL(k_compact_blocks, dim3((n + kCompactBlock - 1) / kCompactBlock), dim3(kCompactThreads), 0, stream,
                       mask, n, idx, count, sample_offsets, per_sample > 0 ? per_sample : 1);
    return check_launch();
  }
  if (n <= kSmallCompactMax) {
    hipLaunchKernelGGL(k_compact_small, dim3(1), dim3(kCompactThreads), 0, stream, mask, n, idx, count,
                       sample_offsets, per_sample > 0 ? per_sample : 1);
    return check_launch();
  }
  const int nb = (n + kCompactBlock - 1) / kCompactBlock;
  if (nb > 1) {
    hipLaunchKernelGGL(k_block_counts, dim3(nb - 1), dim3(kCompactThreads), 0, stream, mask, n, block_counts);
    if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;
  }
  hipLaunchKernelGGL(k_compact, dim3(nb), dim3(kCompactThreads), 0, stream, mask, n, idx, count, sample_offsets,
                     per_sample > 0 ? per_sample : 1, block_counts, nb);
  return check_launch();
}

int launch_pool_compact(const float* proj, int N, int H, int W, int S, float bias, const uint8_t* keep, uint8_t* mask,
                        float* logits, int32_t* idx, int32_t* count, int32_t* sample_offsets, int32_t* block_counts,
                        hipStream_t stream) {
  const int pps = (H / S) * (W / S), npatch = N * pps;
  PoolArgs pa{proj, keep, logits, H, W, S, bias};
  if (S == 2 && npatch > 0 && npatch <= kPoolFusedMax) {
    StageScope scope(LAUD_STAGE_COMPACT, stream);
    hipLaunchKernelGGL(k_pool_compact_s2, dim3((npatch + kCompactThreads - 1) / kCompactThreads), dim3(kCompactThreads), 0,
                       stream, pa, npatch, mask, idx, count, sample_offsets, pps);
    return check_launch();
  }
  if (npatch > 0 && npatch <= kCompactThreads) {
    StageScope scope(LAUD_STAGE_COMPACT, stream);
    hipLaunchKernelGGL(k_pool_compact_one_block, dim3(1), dim3(kCompactThreads), 0, stream, pa, npatch, mask, idx, count,
                       sample_offsets, pps);
    return check_launch();
  }
  // One thread per patch over a wide grid: the S*S projection reads of a patch are independent, and a
  // single block walking all patches would serialise their latency.
  {
    StageScope scope(LAUD_STAGE_MASK_LOGITS, stream);
    hipLaunchKernelGGL(k_pool_mask, dim3((npatch + 255) / 256), dim3(256), 0, stream, pa, npatch, mask);
  }
  if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;
  return launch_compact(mask, npatch, idx, count, sample_offsets, pps, block_counts, stream);
}

// ------------------------------------------------------------------------------------------
// masker logits + threshold
// ------------------------------------------------------------------------------------------
// One "team" (a wave, or the whole 256-thread block for big patches) per patch.  The team
// walks the S*S pixel rows of the patch in 16-byte chunks; float32 accumulation.
template <typename ET, int TEAM, bool WLDS>
__global__ __launch_bounds__(256) void k_mask_logits(const ET* __restrict__ x, int N, int H, int W, int C, int S,
                                                     const float* __restrict__ w, float bias,
                                                     const uint8_t* __restrict__ keep, uint8_t* __restrict__ mask,
                                                     float* __restrict__ logits) {
  constexpr int EPC = elem<ET>::per16;
  constexpr int TEAMS = 256 / TEAM;
  __shared__ float red[256 / kWave];
  // The masker weights are read once per 16-byte chunk of x; from global memory they would double the
  // number of vector-memory instructions of a kernel that should only stream x, so the block keeps
  // them in LDS (C floats) when they fit.
  extern __shared__ __align__(16) float s_w[];
  const int Hp = H / S, Wp = W / S;
  const int npatch = N * Hp * Wp;
  const int team = threadIdx.x / TEAM, tl = threadIdx.x % TEAM;
  const int q = blockIdx.x * TEAMS + team;
  const bool live = q < npatch;  // uniform per team
  float acc = 0.f;
  int n = 0;
  {
    // a team past the end reads the last patch (valid addresses) and writes nothing
    const int qq = live ? q : npatch - 1;
    n = qq / (Hp * Wp);
    const int r = qq - n * (Hp * Wp);
    const int py = r / Wp, px = r - py * Wp;
    const int cpr = C / EPC;          // chunks per pixel row
    const int total = S * S * cpr;    // chunks per patch
    // Eight (then four) 16-byte loads of x are put in flight before any of them is consumed: the kernel is a pure
    // stream over x and what bounds it is the number of bytes in flight per CU.  A thread's chunks are TEAM apart;
    // their position (pixel of the patch, chunk inside the pixel) is advanced incrementally -- one division at the
    // start instead of four per load, which at eight loads per lane delayed the last request of a wave by
    // about a thousand instructions.
    const size_t pix0 = ((size_t)n * H + (size_t)py * S) * W + (size_t)px * S;  // first pixel of the patch
    int cv, dy, dx;  // position of the next chunk: chunk column inside the pixel, pixel row / column inside the patch
    {
      const int j = tl / cpr;
      cv = tl - j * cpr;
      dy = j / S;
      dx = j - dy * S;
    }
    auto next_ptr = [&](int& cv_out) -> const uint4* {
      // chunks past the end of the patch (the last, partial round of a team) re-read the patch's last chunk
      const bool in = dy < S;
      const int ddy = in ? dy : S - 1, ddx = in ? dx : S - 1, ccv = in ? cv : cpr - 1;
      cv_out = ccv;
      const uint4* p = reinterpret_cast<const uint4*>(x + (pix0 + (size_t)ddy * W + ddx) * C + (size_t)ccv * EPC);
      cv += TEAM;
      while (cv >= cpr) {
        cv -= cpr;
        if (++dx == S) { dx = 0; ++dy; }
      }
      return p;
    };
    auto dot = [&](const uint4& raw, int cvv) -> float {
      float4 w0, w1 = make_float4(0.f, 0.f, 0.f, 0.f);
      if constexpr (WLDS) {
        const float4* wp = reinterpret_cast<const float4*>(s_w + cvv * EPC);
        w0 = wp[0];
        if constexpr (EPC == 8) w1 = wp[1];
      } else {
        const float4* wp = reinterpret_cast<const float4*>(w + cvv * EPC);
        w0 = wp[0];
        if constexpr (EPC == 8) w1 = wp[1];
      }
      if constexpr (EPC == 4) {
        return __uint_as_float(raw.x) * w0.x + __uint_as_float(raw.y) * w0.y + __uint_as_float(raw.z) * w0.z +
               __uint_as_float(raw.w) * w0.w;
      } else {
        return __uint_as_float(raw.x << 16) * w0.x + __uint_as_float(raw.x & 0xffff0000u) * w0.y +
               __uint_as_float(raw.y << 16) * w0.z + __uint_as_float(raw.y & 0xffff0000u) * w0.w +
               __uint_as_float(raw.z << 16) * w1.x + __uint_as_float(raw.z & 0xffff0000u) * w1.y +
               __uint_as_float(raw.w << 16) * w1.z + __uint_as_float(raw.w & 0xffff0000u) * w1.w;
      }
    };
    // The first eight loads of x are issued before the block fetches the weights, so the two
    // far-memory latencies overlap instead of adding up (the kernel lives for only a few of them).
    uint4 first[8];
    int fcv[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) first[u] = *next_ptr(fcv[u]);
    if constexpr (WLDS) {
      for (int k = threadIdx.x; k < C; k += 256) s_w[k] = w[k];
      __syncthreads();
    }
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      const float d = dot(first[u], fcv[u]);
      acc += tl + u * TEAM < total ? d : 0.f;
    }
    int c = tl + 8 * TEAM;
    for (; c + 7 * TEAM < total; c += 8 * TEAM) {
      uint4 r[8];
      int rcv[8];
#pragma unroll
      for (int u = 0; u < 8; ++u) r[u] = *next_ptr(rcv[u]);
#pragma unroll
      for (int u = 0; u < 8; ++u) acc += dot(r[u], rcv[u]);
    }
    for (; c + 3 * TEAM < total; c += 4 * TEAM) {
      uint4 r[4];
      int rcv[4];
#pragma unroll
      for (int u = 0; u < 4; ++u) r[u] = *next_ptr(rcv[u]);
#pragma unroll
      for (int u = 0; u < 4; ++u) acc += dot(r[u], rcv[u]);
    }
    for (; c < total; c += TEAM) {
      int cvv;
      const uint4 r = *next_ptr(cvv);
      acc += dot(r, cvv);
    }
  }
  acc = wave_sum(acc);
  if constexpr (TEAM > kWave) {
    if (lane_id() == 0) red[threadIdx.x / kWave] = acc;
    __syncthreads();
    acc = 0.f;
    for (int k = 0; k < 256 / kWave; ++k) acc += red[k];
  }
  if (live && tl == 0) {
    const float logit = acc / (float)(S * S) + bias;
    bool on = logit > 0.f;  // false for NaN
    if (keep && keep[n] == 0) on = false;
    mask[q] = on ? 1 : 0;
    if (logits) logits[q] = logit;
  }
}

// Small patches (at most 4 KB): one wave takes PPW patches at once and requests all of their chunks -- PPW x LPP =
// 16 loads of 16 bytes per lane -- before it touches any of them, so a wave keeps 16 KB in flight however small
// the patch is, and a block's weight fill and barrier are paid once per 4 x PPW patches.  (Measured: 2 to 5 times
// the rate of one patch per wave at 0.5 - 4 KB per patch; at 8 KB one patch per wave is as fast or faster.)
template <typename ET, int PPW, int LPP>
__global__ __launch_bounds__(256) void k_mask_logits_multi(const ET* __restrict__ x, int N, int H, int W, int C, int S,
                                                           const float* __restrict__ w, float bias,
                                                           const uint8_t* __restrict__ keep,
                                                           uint8_t* __restrict__ mask, float* __restrict__ logits) {
  constexpr int EPC = elem<ET>::per16;
  extern __shared__ __align__(16) float s_w[];  // the masker weights, [C]
  const int Hp = H / S, Wp = W / S, pps = Hp * Wp;
  const int npatch = N * pps;
  const int wave = threadIdx.x / kWave, lane = lane_id();
  const int q0 = (blockIdx.x * (256 / kWave) + wave) * PPW;
  const int cpr = C / EPC;        // chunks per pixel row
  const int total = S * S * cpr;  // chunks per patch (at most 64 * LPP)
  uint4 r[PPW][LPP];
#pragma unroll
  for (int p = 0; p < PPW; ++p) {
    // a patch past the end re-reads the last one (valid addresses); nothing is written for it
    const int qq = min(q0 + p, npatch - 1);
    const int n = qq / pps, rr = qq - n * pps;
    const int py = rr / Wp, px = rr - py * Wp;
#pragma unroll
    for (int u = 0; u < LPP; ++u) {
      const int c = min(lane + u * kWave, total - 1);
      const int j = c / cpr, cv = c - j * cpr;
      const int dy = j / S, dx = j - dy * S;
      const size_t pix = ((size_t)n * H + (py * S + dy)) * W + (px * S + dx);
      r[p][u] = *reinterpret_cast<const uint4*>(x + pix * C + (size_t)cv * EPC);
    }
  }
  for (int k = threadIdx.x; k < C; k += 256) s_w[k] = w[k];
  __syncthreads();
  float acc[PPW];
#pragma unroll
  for (int p = 0; p < PPW; ++p) {
    acc[p] = 0.f;
#pragma unroll
    for (int u = 0; u < LPP; ++u) {
      const int c = lane + u * kWave;
      const int cv = min(c, total - 1) % cpr;
      const float4* wp = reinterpret_cast<const float4*>(s_w + cv * EPC);
      const float4 w0 = wp[0];
      const uint4 raw = r[p][u];
      float d;
      if constexpr (EPC == 4) {
        d = __uint_as_float(raw.x) * w0.x + __uint_as_float(raw.y) * w0.y + __uint_as_float(raw.z) * w0.z +
            __uint_as_float(raw.w) * w0.w;
      } else {
        const float4 w1 = wp[1];
        d = __uint_as_float(raw.x << 16) * w0.x + __uint_as_float(raw.x & 0xffff0000u) * w0.y +
            __uint_as_float(raw.y << 16) * w0.z + __uint_as_float(raw.y & 0xffff0000u) * w0.w +
            __uint_as_float(raw.z << 16) * w1.x + __uint_as_float(raw.z & 0xffff0000u) * w1.y +
            __uint_as_float(raw.w << 16) * w1.z + __uint_as_float(raw.w & 0xffff0000u) * w1.w;
      }
      acc[p] += c < total ? d : 0.f;
    }
  }
#pragma unroll
  for (int p = 0; p < PPW; ++p) acc[p] = wave_sum(acc[p]);
  // lane p writes patch p
  float mine = 0.f;
#pragma unroll
  for (int p = 0; p < PPW; ++p) mine = lane == p ? acc[p] : mine;
  const int q = q0 + lane;
  if (lane < PPW && q < npatch) {
    const float logit = mine / (float)(S * S) + bias;
    bool on = logit > 0.f;  // false for NaN
    if (keep && keep[q / pps] == 0) on = false;
    mask[q] = on ? 1 : 0;
    if (logits) logits[q] = logit;
  }
}

// ------------------------------------------------------------------------------------------
// stand-alone gather
// ------------------------------------------------------------------------------------------
// One team of `team` lanes (a power of two, 8 .. 64: the pixel's 16-byte chunks rounded up, so that narrow maps do
// not leave most of a wave idle) per (patch, dy, dx) slot of the gathered buffer; 16-byte copies, zero fill outside.
__global__ __launch_bounds__(256) void k_gather(const uint4* __restrict__ x, int H, int W, int S, int halo,
                                                int chunks_per_pixel, const int32_t* __restrict__ idx,
                                                const int32_t* __restrict__ count, uint4* __restrict__ out,
                                                long long cap_slots, int team) {
  const int E = S + 2 * halo;
  const int Hp = H / S, Wp = W / S;
  const long long slot = ((long long)blockIdx.x * 256 + threadIdx.x) / team;
  const int tl = (int)threadIdx.x & (team - 1);
  if (slot >= cap_slots) return;
  const int p = (int)(slot / (E * E));
  if (p >= *count) return;
  const int e = (int)(slot - (long long)p * (E * E));
  const int dy = e / E, dx = e - dy * E;
  const int q = idx[p];
  const int n = q / (Hp * Wp);
  const int r = q - n * (Hp * Wp);
  const int py = r / Wp, px = r - py * Wp;
  const int yy = py * S - halo + dy, xx = px * S - halo + dx;
  const bool inside = yy >= 0 && yy < H && xx >= 0 && xx < W;
  uint4* dst = out + (size_t)slot * chunks_per_pixel;
  const uint4* src = x + (((size_t)n * H + (inside ? yy : 0)) * W + (inside ? xx : 0)) * chunks_per_pixel;
  const uint4 zero = make_uint4(0, 0, 0, 0);
  for (int c = tl; c < chunks_per_pixel; c += team) dst[c] = inside ? src[c] : zero;
}

}  // namespace laud

using namespace laud;

// ------------------------------------------------------------------------------------------
// C ABI
// ------------------------------------------------------------------------------------------
extern "C" int laud_layer_skip_compact(const uint8_t* keep, int n, int32_t* idx, int32_t* count, void* ws,
                                       size_t ws_bytes, void* stream) {
  if (n < 0 || !count || (n > 0 && (!keep || !idx))) return LAUD_ERR_INVALID_ARG;
  if (n > kSmallCompactMax && (!ws || ws_bytes < compact_ws_bytes(n))) return LAUD_ERR_WORKSPACE;
  clear_stale_error();
  return launch_compact(keep, n, idx, count, nullptr, 1, (int32_t*)ws, (hipStream_t)stream);
}

extern "C" int laud_mask_gen(const void* x, laud_fmap fx, int S, const float* w, float bias, const uint8_t* keep,
                             uint8_t* mask, int32_t* idx, int32_t* count, int32_t* sample_offsets, float* logits,
                             void* ws, size_t ws_bytes, void* stream) {
  if (!x || !w || !mask || !idx || !count || !valid_fmap(fx) || S <= 0) return LAUD_ERR_INVALID_ARG;
  if (fx.H % S || fx.W % S) return LAUD_ERR_INVALID_ARG;
  if (fx.C % 8) return LAUD_ERR_UNSUPPORTED;
  const long long npatch = (long long)fx.N * (fx.H / S) * (fx.W / S);
  if (npatch > 0x7fffffffLL || (long long)fx.N * fx.H * fx.W > 0x7fffffffLL) return LAUD_ERR_UNSUPPORTED;
  if (npatch > kSmallCompactMax && (!ws || ws_bytes < compact_ws_bytes(npatch))) return LAUD_ERR_WORKSPACE;
  hipStream_t st = (hipStream_t)stream;
  clear_stale_error();
  const size_t patch_bytes = (size_t)S * S * fx.C * elem_bytes(fx.dtype);
  const bool big = patch_bytes >= 32768;  // a whole block per patch
  const int teams = big ? 1 : 256 / kWave;
  const unsigned grid = (unsigned)((npatch + teams - 1) / teams);
  const int w_lds = fx.C <= 8192 ? 1 : 0;
  {
    StageScope scope(LAUD_STAGE_MASK_LOGITS, st);
#define LAUD_LAUNCH_MASK(ET, TEAM)                                                                            \
  do {                                                                                                        \
    if (w_lds)                                                                                                \
      hipLaunchKernelGGL((k_mask_logits<ET, TEAM, true>), dim3(grid), dim3(256), (size_t)fx.C * 4, st,        \
                         (const ET*)x, fx.N, fx.H, fx.W, fx.C, S, w, bias, keep, mask, logits);                \
    else                                                                                                      \
      hipLaunchKernelGGL((k_mask_logits<ET, TEAM, false>), dim3(grid), dim3(256), 0, st, (const ET*)x, fx.N,  \
                         fx.H, fx.W, fx.C, S, w, bias, keep, mask, logits);                                   \
  } while (0)
  // small patches, enough of them to fill the chip with waves of PPW patches each: the multi-patch kernel
  const int chunks = (int)(patch_bytes / 16);
  const int lpp = chunks <= 64 ? 1 : chunks <= 128 ? 2 : 4;
  if (chunks <= 256 && w_lds && npatch / (16 / lpp) >= 1024) {
    const int ppw = 16 / lpp;
    const unsigned g2 = (unsigned)((npatch + 4 * ppw - 1) / (4 * ppw));
#define LAUD_LAUNCH_MULTI(ET, PPW, LPP)                                                                          \
  hipLaunchKernelGGL((k_mask_logits_multi<ET, PPW, LPP>), dim3(g2), dim3(256), (size_t)fx.C * 4, st, (const ET*)x, \
                     fx.N, fx.H, fx.W, fx.C, S, w, bias, keep, mask, logits)
#define LAUD_PICK_MULTI(ET)                                                    \
  do {                                                                         \
    if (lpp == 1) LAUD_LAUNCH_MULTI(ET, 16, 1);                                \
    else if (lpp == 2) LAUD_LAUNCH_MULTI(ET, 8, 2);                            \
    else LAUD_LAUNCH_MULTI(ET, 4, 4);                                          \
  } while (0)
    if (fx.dtype == LAUD_BF16) LAUD_PICK_MULTI(bf16_t); else LAUD_PICK_MULTI(float);
#undef LAUD_PICK_MULTI
#undef LAUD_LAUNCH_MULTI
  } else if (fx.dtype == LAUD_BF16) {
    if (big) LAUD_LAUNCH_MASK(bf16_t, 256); else LAUD_LAUNCH_MASK(bf16_t, 64);
  } else {
    if (big) LAUD_LAUNCH_MASK(float, 256); else LAUD_LAUNCH_MASK(float, 64);
  }
#undef LAUD_LAUNCH_MASK
  }
  if (check_launch() != LAUD_OK) return LAUD_ERR_HIP;
  return launch_compact(mask, (int)npatch, idx, count, sample_offsets, (fx.H / S) * (fx.W / S), (int32_t*)ws, st);
}

extern "C" int laud_gather_patches(const void* x, laud_fmap fx, int S, int halo, const int32_t* idx,
                                   const int32_t* count, void* out, void* stream) {
  if (!x || !idx || !count || !out || !valid_fmap(fx) || S <= 0 || halo < 0 || halo > 1) return LAUD_ERR_INVALID_ARG;
  if (fx.H % S || fx.W % S) return LAUD_ERR_INVALID_ARG;
  if (fx.C % 8) return LAUD_ERR_UNSUPPORTED;
  const long long npatch = (long long)fx.N * (fx.H / S) * (fx.W / S);
  if (npatch > 0x7fffffffLL) return LAUD_ERR_UNSUPPORTED;
  const int E = S + 2 * halo;
  const long long slots = npatch * E * E;
  const int cpp = (int)((size_t)fx.C * elem_bytes(fx.dtype) / 16);
  int team = 8;
  while (team < kWave && team < cpp) team <<= 1;
  const long long blocks = (slots * team + 255) / 256;
  if (blocks > 0x7fffffffLL) return LAUD_ERR_UNSUPPORTED;
  clear_stale_error();
  StageScope scope(LAUD_STAGE_GATHER, (hipStream_t)stream);
  hipLaunchKernelGGL(k_gather, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream, (const uint4*)x, fx.H, fx.W,
                     S, halo, cpp, idx, count, (uint4*)out, slots, team);
  return check_launch();
}
