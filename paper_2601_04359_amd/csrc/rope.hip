// pc_rope3d: in-place 3D rotary embedding (the operator R of Eq. 2 with the (t, h, w)
// coordinates of Sec. 3.1 / Sec. 3.4).  HBM-bound: every element is read and written
// once; sin/cos of a (token, pair) are computed once and shared by all heads.
#include <math.h>

#include "common.h"

namespace pc {
namespace {

constexpr int kMaxPairs = 128;    // D <= 256
constexpr int kTokPerBlock = 16;  // tokens per work-group
constexpr int kThreads = 256;

struct RopeFreq {
  double inv_freq[kMaxPairs];  // base^(-2i/s) of every pair, section by section
  uint8_t axis[kMaxPairs];     // which coordinate (0 = t, 1 = h, 2 = w) turns the pair
};

// Phase 1: cos/sin of the kTokPerBlock x (D/2) angles of this work-group, angle formed
// and reduced in fp64 (positions reach hundreds of radians), kept as fp32 in LDS.
// Phase 2: every thread rotates 16 bytes (8 bf16 = 4 pairs, or 4 fp32 = 2 pairs) per head.
template <typename T>
__global__ __launch_bounds__(kThreads) void rope3d_kernel(T* __restrict__ x, int H, int n, int D,
                                                          int64_t stride_h,
                                                          const int32_t* __restrict__ pos,
                                                          RopeFreq fr) {
  __shared__ float2 cs[kTokPerBlock][kMaxPairs];
  const int tok0 = blockIdx.x * kTokPerBlock;
  const int pairs = D / 2;
  for (int e = threadIdx.x; e < kTokPerBlock * pairs; e += kThreads) {
    const int t = e / pairs, p = e % pairs;
    const int tok = tok0 + t;
    float2 v = make_float2(1.f, 0.f);
    if (tok < n) {
      const double ang = static_cast<double>(pos[static_cast<int64_t>(tok) * 3 + fr.axis[p]]) *
                         fr.inv_freq[p];
      double s, c;
      sincos(ang, &s, &c);
      v = make_float2(static_cast<float>(c), static_cast<float>(s));
    }
    cs[t][p] = v;
  }
  __syncthreads();

  constexpr int kElems = 16 / sizeof(T);  // elements per 16-byte chunk
  const int chunks_per_row = D / kElems;
  const int total = kTokPerBlock * chunks_per_row;
  for (int h = 0; h < H; ++h) {
    T* xh = x + h * stride_h;
    for (int e = threadIdx.x; e < total; e += kThreads) {
      const int t = e / chunks_per_row, c = e % chunks_per_row;
      const int tok = tok0 + t;
      if (tok >= n) continue;
      u32x4* p = reinterpret_cast<u32x4*>(xh + static_cast<int64_t>(tok) * D + c * kElems);
      u32x4 raw = *p;
      if constexpr (sizeof(T) == 2) {
#pragma unroll
        for (int k = 0; k < 4; ++k) {
          const float2 r = cs[t][c * 4 + k];
          const float x0 = bf16_to_f32(static_cast<uint16_t>(raw[k] & 0xFFFFu));
          const float x1 = bf16_to_f32(static_cast<uint16_t>(raw[k] >> 16));
          raw[k] = pack_bf16x2(x0 * r.x - x1 * r.y, x0 * r.y + x1 * r.x);
        }
      } else {
#pragma unroll
        for (int k = 0; k < 2; ++k) {
          const float2 r = cs[t][c * 2 + k];
          const float x0 = __uint_as_float(raw[2 * k]), x1 = __uint_as_float(raw[2 * k + 1]);
          raw[2 * k] = __float_as_uint(x0 * r.x - x1 * r.y);
          raw[2 * k + 1] = __float_as_uint(x0 * r.y + x1 * r.x);
        }
      }
      *p = raw;
    }
  }
}

}  // namespace
}  // namespace pc

using namespace pc;

extern "C" int pc_rope3d(void* x, int dtype, int H, int n, int D, int64_t stride_h,
                         const int32_t* pos, int sec_t, int sec_h, int sec_w, double base,
                         void* stream) {
  PC_REQUIRE(dtype == PC_F32 || dtype == PC_BF16, PC_ERR_DTYPE, "pc_rope3d: dtype %d", dtype);
  PC_REQUIRE(H >= 0 && n >= 0 && D > 0, PC_ERR_SHAPE, "pc_rope3d: H=%d n=%d D=%d", H, n, D);
  const int secs[3] = {sec_t, sec_h, sec_w};
  for (int a = 0; a < 3; ++a)
    PC_REQUIRE(secs[a] >= 0 && secs[a] % 2 == 0, PC_ERR_SHAPE,
               "pc_rope3d: section %d has width %d (must be even, >= 0)", a, secs[a]);
  PC_REQUIRE(sec_t + sec_h + sec_w == D, PC_ERR_SHAPE, "pc_rope3d: sections %d+%d+%d != D=%d",
             sec_t, sec_h, sec_w, D);
  PC_REQUIRE(D <= 2 * kMaxPairs && D % 8 == 0, PC_ERR_SHAPE,
             "pc_rope3d: D=%d must be a multiple of 8 and <= %d", D, 2 * kMaxPairs);
  PC_REQUIRE(base > 0.0, PC_ERR_SHAPE, "pc_rope3d: base %g", base);
  if (H == 0 || n == 0) return PC_OK;
  PC_REQUIRE(x && pos, PC_ERR_NULL, "pc_rope3d: x or pos is NULL");
  PC_REQUIRE(stride_h >= static_cast<int64_t>(n) * D || H == 1, PC_ERR_SHAPE,
             "pc_rope3d: head stride %lld < n*D", static_cast<long long>(stride_h));
  PC_REQUIRE((stride_h * (dtype == PC_BF16 ? 2 : 4)) % 16 == 0 &&
                 reinterpret_cast<uintptr_t>(x) % 16 == 0,
             PC_ERR_SHAPE, "pc_rope3d: x and its head stride must be 16-byte aligned");

  RopeFreq fr;
  int p = 0;
  for (int a = 0; a < 3; ++a)
    for (int i = 0; i < secs[a] / 2; ++i, ++p) {
      fr.inv_freq[p] = pow(base, -2.0 * i / secs[a]);
      fr.axis[p] = static_cast<uint8_t>(a);
    }
  for (; p < kMaxPairs; ++p) {
    fr.inv_freq[p] = 0.0;
    fr.axis[p] = 0;
  }
  const dim3 grid(ceil_div(n, kTokPerBlock));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == PC_BF16)
    rope3d_kernel<uint16_t><<<grid, kThreads, 0, s>>>(static_cast<uint16_t*>(x), H, n, D, stride_h, pos, fr);
  else
    rope3d_kernel<float><<<grid, kThreads, 0, s>>>(static_cast<float*>(x), H, n, D, stride_h, pos, fr);
  PC_CHECK_LAUNCH("pc_rope3d");
  return PC_OK;
}
