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

// Lane exchanges inside a row of 16 lanes run in the vector ALU (DPP operand modifiers, a few cycles each);
// a general lane exchange goes through the LDS crossbar and costs an LDS round trip, and a butterfly of six
// of them is a chain of six such round trips - most of the time of a wave-wide sum.  CTRL: quad_perm
// selectors (0x00-0xFF), 0x140 row_mirror (lane i <-> 15 - i), 0x141 row_half_mirror (i <-> 7 - i).
template <int CTRL>
__device__ __forceinline__ float dpp_move(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
constexpr int kDppXor1 = 0xB1;           // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;           // quad_perm [2,3,0,1]
constexpr int kDppNext = 0xF5;           // quad_perm [1,1,3,3]: an even lane reads its odd neighbour
constexpr int kDppHalfMirror = 0x141, kDppMirror = 0x140;

// Sum over each aligned group of 8 (16) adjacent lanes, in every lane of the group.  After the two quad
// steps the four lanes of a quad hold the same value, so a mirror delivers the other quad's (half's) sum.
__device__ __forceinline__ float sum8(float v) {
  v += dpp_move<kDppXor1>(v);
  v += dpp_move<kDppXor2>(v);
  v += dpp_move<kDppHalfMirror>(v);
  return v;
}
__device__ __forceinline__ float sum16(float v) {
  v = sum8(v);
  v += dpp_move<kDppMirror>(v);
  return v;
}
__device__ __forceinline__ float lane_value(float v, int lane) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), lane));
}

// Sum (maximum) over the wave, the same value in every lane: the four rows of 16, then the rows' results
// through scalar registers, in a fixed order.
__device__ __forceinline__ float wave_sum(float v) {
  v = sum16(v);
  return (lane_value(v, 0) + lane_value(v, 16)) + (lane_value(v, 32) + lane_value(v, 48));
}

__device__ __forceinline__ float wave_max(float v) {
  v = fmaxf(v, dpp_move<kDppXor1>(v));
  v = fmaxf(v, dpp_move<kDppXor2>(v));
  v = fmaxf(v, dpp_move<kDppHalfMirror>(v));
  v = fmaxf(v, dpp_move<kDppMirror>(v));
  return fmaxf(fmaxf(lane_value(v, 0), lane_value(v, 16)), fmaxf(lane_value(v, 32), lane_value(v, 48)));
}

}  // namespace heisd
