// Direct global->LDS tile loads and the swizzled 256-byte-row tile layout shared by the
// bf16 MFMA kernels (gfx950 only).
#pragma once

#include "common.h"

namespace pc {

typedef __attribute__((address_space(3))) uint8_t lds_u8;

// Exchange between lane i and lane i ^ 32 with v_permlane32_swap (one vector instruction, no
// LDS round trip).  Given the same value in both operands it returns r[0] = the lower half's
// value in both halves and r[1] = the upper half's value in both halves.
struct HalfPair {
  float lo, hi;  // value held by lane (i & 31) and by lane (i & 31) + 32
};
__device__ __forceinline__ HalfPair wave_halves(float v) {
  const auto r = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
  return {__uint_as_float(r[0]), __uint_as_float(r[1])};
}
__device__ __forceinline__ float wave_half_max(float v) {
  const HalfPair p = wave_halves(v);
  return fmaxf(p.lo, p.hi);
}
__device__ __forceinline__ float wave_half_sum(float v) {
  const HalfPair p = wave_halves(v);
  return p.lo + p.hi;
}
// the value of the partner lane i ^ 32
__device__ __forceinline__ float wave_half_swap(float v) {
  const HalfPair p = wave_halves(v);
  return (threadIdx.x & 32) ? p.lo : p.hi;
}

// Tiles are filled by direct global->LDS loads: a wave-wide load writes lane i's 16 bytes at
// base + 16 i, i.e. four whole 256-byte rows back to back, so rows cannot be padded.  Bank
// conflicts are avoided by choosing WHICH 16-byte chunk of the row each lane fetches: for an
// operand read as MFMA fragments (16 rows, one chunk each per quarter wave) chunk c of row r
// is stored at chunk position c ^ (r & 15).  The map is an involution.
__device__ __forceinline__ int k_chunk_pos(int row, int chunk) { return chunk ^ (row & 15); }

// The LDS base of a direct load travels in M0, a register the compiler reserves for itself and
// does not accept on a clobber list: the statements below put back what they found in it, so
// they are neutral to whatever the compiler keeps there (two scalar moves per load).
// One wave-wide 1-KB direct load: lane i's 16 bytes from `src` land at lds_base + 16 i.
__device__ __forceinline__ void dma_16B(const void* src, uint32_t lds_base) {
  uint32_t saved_m0;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %2, off\n\ts_mov_b32 m0, %0"
      : "=&s"(saved_m0)
      : "s"(lds_base), "v"(src)
      : "memory");
}
// One wave-wide 256-byte direct load: lane i's 4 bytes from `src` land at lds_base + 4 i.
__device__ __forceinline__ void dma_4B(const void* src, uint32_t lds_base) {
  uint32_t saved_m0;
  asm volatile(
      "s_mov_b32 %0, m0\n\ts_mov_b32 m0, %1\n\ts_nop 0\n\tglobal_load_lds_dword %2, off\n\ts_mov_b32 m0, %0"
      : "=&s"(saved_m0)
      : "s"(lds_base), "v"(src)
      : "memory");
}

__device__ __forceinline__ bf16x8 lds_frag(const lds_u8* p) {
  return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(p);
}

}  // namespace pc
