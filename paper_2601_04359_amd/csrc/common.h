// Internal helpers shared by the libpackcache translation units (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>

#include <atomic>
#include <stdarg.h>
#include <stdint.h>
#include <stdio.h>

#include "packcache.h"

namespace pc {

// ---- error reporting -------------------------------------------------------------------
void set_detail(const char* fmt, ...);  // thread-local message for pc_last_error_detail()

#define PC_FAIL(code, ...)        \
  do {                            \
    ::pc::set_detail(__VA_ARGS__); \
    return (code);                \
  } while (0)

#define PC_REQUIRE(cond, code, ...) \
  do {                              \
    if (!(cond)) PC_FAIL(code, __VA_ARGS__); \
  } while (0)

// Checks the launch that was just enqueued (no synchronisation).
#define PC_CHECK_LAUNCH(what)                                                       \
  do {                                                                              \
    hipError_t e_ = hipGetLastError();                                              \
    if (e_ != hipSuccess) PC_FAIL(PC_ERR_HIP, "%s: %s", what, hipGetErrorString(e_)); \
  } while (0)

// Raises a kernel's dynamic-LDS limit once per device; `done` is the caller's per-kernel
// bit mask of devices already served.  Safe to call from several host threads.
inline int allow_dynamic_lds(const void* kernel, size_t bytes, std::atomic<uint64_t>& done, const char* who) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) dev = 0;
  const uint64_t bit = 1ull << dev;
  if (done.load(std::memory_order_acquire) & bit) return PC_OK;
  const hipError_t e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, static_cast<int>(bytes));
  if (e != hipSuccess) PC_FAIL(PC_ERR_HIP, "%s: LDS attribute: %s", who, hipGetErrorString(e));
  done.fetch_or(bit, std::memory_order_release);
  return PC_OK;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }
inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// ---- device-side types -----------------------------------------------------------------
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(4 * sizeof(__bf16)))) __bf16 bf16x4;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef __attribute__((__vector_size__(4 * sizeof(float)))) float f32x4;
typedef __attribute__((__vector_size__(4 * sizeof(uint32_t)))) uint32_t u32x4;
typedef __attribute__((__vector_size__(2 * sizeof(uint32_t)))) uint32_t u32x2;

__device__ __forceinline__ float bf16_to_f32(uint16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}
// Round to nearest even; the compiler selects v_cvt_pk_bf16_f32 on gfx950.
__device__ __forceinline__ uint16_t f32_to_bf16(float f) {
  __bf16 h = static_cast<__bf16>(f);
  return __builtin_bit_cast(uint16_t, h);
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return static_cast<uint32_t>(f32_to_bf16(lo)) | (static_cast<uint32_t>(f32_to_bf16(hi)) << 16);
}

// Work-group index -> logical index such that work-groups that land on the same XCD
// (the hardware deals consecutive work-group ids round-robin over the 8 XCDs, each with
// its own L2) receive a contiguous range of logical indices.
__device__ __forceinline__ int xcd_contiguous_index(int b, int n) {
  constexpr int kXcd = 8;
  const int x = b % kXcd, r = b / kXcd;
  const int q = n / kXcd, rem = n % kXcd;
  return x * q + (x < rem ? x : rem) + r;
}

}  // namespace pc
