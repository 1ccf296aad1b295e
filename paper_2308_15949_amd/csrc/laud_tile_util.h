// Device helpers shared by the register-weight MFMA kernels (laud_head.hip, laud_tail.hip): LDS-direct loads,
// explicit counter waits, the transposed 32x32x16 bf16 MFMA tile and its lane-swap epilogue.
#pragma once

#include "laud_common.h"

namespace laud {

typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef unsigned int u32x4 __attribute__((ext_vector_type(4)));

// LDS-direct load of 16 bytes per lane: lane l's chunk lands at LDS byte address lds_base + 16*l.
__device__ __forceinline__ void dma16(__amdgpu_buffer_rsrc_t rsrc, unsigned voff, unsigned soff, unsigned lds_base) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tbuffer_load_dwordx4 %1, %2, %3 offen lds"
               :
               : "s"(lds_base), "v"(voff), "s"(rsrc), "s"(soff)
               : "memory");
}
template <int N>
__device__ __forceinline__ void vm_wait() {
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}
__device__ __forceinline__ void wg_barrier() { asm volatile("s_barrier" ::: "memory"); }
__device__ __forceinline__ void lds_wait() { asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory"); }

__device__ __forceinline__ f32x16 mma_bf16(const u32x4& first, const uint4& second, f32x16 acc) {
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

}  // namespace laud
