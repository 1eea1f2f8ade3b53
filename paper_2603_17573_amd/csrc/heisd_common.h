// Shared device helpers of the HeiSD verify kernels (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace heisd {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

constexpr int kWave = 64;

// fp32 -> bf16 bit pattern, round to nearest even; NaN stays NaN.
__device__ __forceinline__ uint32_t f32_to_bf16_bits(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}

__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }

// Split x into a bf16 head and a bf16 tail: x ~= hi + lo with about 16 mantissa bits kept.
__device__ __forceinline__ void split_bf16(float x, uint32_t &hi, uint32_t &lo) {
  hi = f32_to_bf16_bits(x);
  lo = f32_to_bf16_bits(x - bf16_bits_to_f32(hi));
}

// Workgroup barrier that orders LDS traffic only: outstanding global loads (prefetched weight
// tiles) keep flying across it, which __syncthreads() would wait for.
__device__ __forceinline__ void lds_barrier() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
  __builtin_amdgcn_s_barrier();
  __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// One 16-byte-per-lane transfer global -> LDS that passes through no register: lane l's bytes land
// at lds_addr + 16*l (lds_addr: LDS byte address, wave-uniform).  Completion is counted by vmcnt
// like a load, in issue order with the wave's other vector memory operations.  Written as
// assembly on purpose: the compiler would make every later LDS read wait for it.
__device__ __forceinline__ void lds_dma16(const void *gptr, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off" ::"s"(lds_addr), "v"(gptr) : "memory");
}
// The same transfer with the address split into a wave-uniform 64-bit base (scalar registers) and a
// 32-bit per-lane byte offset: a run of transfers that differ only in the base costs no vector
// address arithmetic.
__device__ __forceinline__ void lds_dma16_s(const void *sbase, uint32_t lane_off, uint32_t lds_addr) {
  asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(lds_addr), "v"(lane_off), "s"(sbase)
               : "memory");
}
// s_waitcnt vmcnt(N) and nothing else, as a compiler-level memory barrier too: no load or store of
// the surrounding code may be moved across it (the count is only right for the written order).
template <int N>
__device__ __forceinline__ void wait_vmcnt() {
  static_assert(N >= 0 && N <= 63, "vmcnt range");
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(N) : "memory");
}

// vmcnt(0) in the form the compiler's own wait placement reads.  A wave that is about to issue
// lds_dma16 transfers calls this first: the compiler cannot see the transfers, and a wait it places
// later for one of ITS OWN earlier loads (one it moved up from code both kinds of wave share, say)
// would land between the transfers and wait for them too, one round trip per transfer.  After this
// call it knows of nothing pending.
__device__ __forceinline__ void wait_vmcnt_all() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_waitcnt(0x0F70);                 // vmcnt 0; expcnt and lgkmcnt left at their maxima
  asm volatile("" ::: "memory");
}

// Does episode b sit this step out?  Either its verify-skip flag is set (Sec. 4.1), or its new rows
// would not fit its cache (prefix_len[b] < 0 or prefix_len[b] + rows > capacity) - a caller's error
// that the host cannot see.  Every kernel that touches per-episode state treats both alike: nothing
// of the episode's cache is read or written.  The acceptance kernels tell them apart again and report
// the second kind (accepted_len = -1, error word).
__device__ __forceinline__ bool episode_overflows(const int32_t *prefix_len, int b, int rows, int cap) {
  const int P = prefix_len[b];
  return P < 0 || P > cap - rows;
}
__device__ __forceinline__ bool episode_sits_out(const uint8_t *skip, const int32_t *prefix_len, int b, int rows, int cap) {
  return (skip && skip[b]) || episode_overflows(prefix_len, b, rows, cap);
}
constexpr unsigned kErrBarrier = 1u, kErrOverflow = 2u;      // bits of the device error word

__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
  return v;
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
  return v;
}

}  // namespace heisd
