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
                                                          RopeFreq fr, double out_scale) {
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
      // the output scale rides on the rotation: no instruction per element, one rounding of the result
      v = make_float2(static_cast<float>(c * out_scale), static_cast<float>(s * out_scale));
    }
    cs[t][p] = v;
  }
  __syncthreads();

  constexpr int kElems = 16 / sizeof(T);  // elements per 16-byte chunk
  constexpr int kHeadsInFlight = 4;       // loads of several heads are issued before any is used
  const int chunks_per_row = D / kElems;
  const int total = kTokPerBlock * chunks_per_row;
  for (int e = threadIdx.x; e < total; e += kThreads) {
    const int t = e / chunks_per_row, c = e % chunks_per_row;
    const int tok = tok0 + t;
    if (tok >= n) continue;
    T* x0 = x + static_cast<int64_t>(tok) * D + c * kElems;
    for (int h0 = blockIdx.y * kHeadsInFlight; h0 < H; h0 += gridDim.y * kHeadsInFlight) {
      u32x4 raw[kHeadsInFlight];
#pragma unroll
      for (int i = 0; i < kHeadsInFlight; ++i)
        if (h0 + i < H) raw[i] = *reinterpret_cast<const u32x4*>(x0 + (h0 + i) * stride_h);
#pragma unroll
      for (int i = 0; i < kHeadsInFlight; ++i) {
        if constexpr (sizeof(T) == 2) {
#pragma unroll
          for (int k = 0; k < 4; ++k) {
            const float2 r = cs[t][c * 4 + k];
            const float a0 = bf16_to_f32(static_cast<uint16_t>(raw[i][k] & 0xFFFFu));
            const float a1 = bf16_to_f32(static_cast<uint16_t>(raw[i][k] >> 16));
            raw[i][k] = pack_bf16x2(a0 * r.x - a1 * r.y, a0 * r.y + a1 * r.x);
          }
        } else {
#pragma unroll
          for (int k = 0; k < 2; ++k) {
            const float2 r = cs[t][c * 2 + k];
            const float a0 = __uint_as_float(raw[i][2 * k]), a1 = __uint_as_float(raw[i][2 * k + 1]);
            raw[i][2 * k] = __float_as_uint(a0 * r.x - a1 * r.y);
            raw[i][2 * k + 1] = __float_as_uint(a0 * r.y + a1 * r.x);
          }
        }
      }
#pragma unroll
      for (int i = 0; i < kHeadsInFlight; ++i)
        if (h0 + i < H) *reinterpret_cast<u32x4*>(x0 + (h0 + i) * stride_h) = raw[i];
    }
  }
}

// pc_rebase: every row turns by the same angles, so the host passes cos/sin of the temporal
// pairs (fp64 angles, fp32 values) by value; a thread rewrites one 16-byte chunk of the
// temporal section of one row, the other sections are not touched.
struct RebaseTable {
  float2 cs[kMaxPairs];
};

template <typename T>
__global__ __launch_bounds__(kThreads) void rebase_kernel(T* __restrict__ K, int Hkv, int D, int64_t k_stride_h,
                                                          int32_t* __restrict__ pos, int Hsel,
                                                          int64_t pos_stride_h, int row0, int n_rows, int delta_t,
                                                          int chunks_t, RebaseTable tab) {
  constexpr int kElems = 16 / sizeof(T);
  const int64_t e = static_cast<int64_t>(blockIdx.x) * kThreads + threadIdx.x;
  const int64_t per_head = static_cast<int64_t>(n_rows) * chunks_t;
  if (e >= per_head * Hkv) return;
  const int h = static_cast<int>(e / per_head);
  const int r = static_cast<int>((e % per_head) / chunks_t), c = static_cast<int>(e % chunks_t);
  const int row = row0 + r;
  u32x4* p = reinterpret_cast<u32x4*>(K + h * k_stride_h + static_cast<int64_t>(row) * D + c * kElems);
  u32x4 raw = *p;
  if constexpr (sizeof(T) == 2) {
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const float2 t = tab.cs[c * 4 + k];
      const float x0 = bf16_to_f32(static_cast<uint16_t>(raw[k] & 0xFFFFu));
      const float x1 = bf16_to_f32(static_cast<uint16_t>(raw[k] >> 16));
      raw[k] = pack_bf16x2(x0 * t.x - x1 * t.y, x0 * t.y + x1 * t.x);
    }
  } else {
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const float2 t = tab.cs[c * 2 + k];
      const float x0 = __uint_as_float(raw[2 * k]), x1 = __uint_as_float(raw[2 * k + 1]);
      raw[2 * k] = __float_as_uint(x0 * t.x - x1 * t.y);
      raw[2 * k + 1] = __float_as_uint(x0 * t.y + x1 * t.x);
    }
  }
  *p = raw;
  if (c == 0 && h < Hsel) pos[h * pos_stride_h + static_cast<int64_t>(row) * 3] -= delta_t;
}

}  // namespace
}  // namespace pc

using namespace pc;

extern "C" int pc_rope3d(void* x, int dtype, int H, int n, int D, int64_t stride_h,
                         const int32_t* pos, int sec_t, int sec_h, int sec_w, double base,
                         double out_scale, void* stream) {
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
  PC_REQUIRE(out_scale > 0.0 && isfinite(out_scale), PC_ERR_SHAPE, "pc_rope3d: out_scale %g must be > 0", out_scale);
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
  // heads are dealt to grid.y in groups of four when there are many: more work-groups in flight
  // for the price of recomputing the (shared) sines and cosines
  const dim3 grid(ceil_div(n, kTokPerBlock), H >= 8 ? 2 : 1);
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == PC_BF16)
    rope3d_kernel<uint16_t><<<grid, kThreads, 0, s>>>(static_cast<uint16_t*>(x), H, n, D, stride_h, pos, fr, out_scale);
  else
    rope3d_kernel<float><<<grid, kThreads, 0, s>>>(static_cast<float*>(x), H, n, D, stride_h, pos, fr, out_scale);
  PC_CHECK_LAUNCH("pc_rope3d");
  return PC_OK;
}

extern "C" int pc_rebase(void* K, int dtype, int Hkv, int D, int64_t k_stride_h, int32_t* pos, int Hsel,
                         int64_t pos_stride_h, int row0, int n_rows, int delta_t, int sec_t, int sec_h,
                         int sec_w, double base, void* stream) {
  PC_REQUIRE(dtype == PC_F32 || dtype == PC_BF16, PC_ERR_DTYPE, "pc_rebase: dtype %d", dtype);
  PC_REQUIRE(Hkv >= 1 && Hsel >= 1 && Hsel <= Hkv && D > 0 && row0 >= 0 && n_rows >= 0, PC_ERR_SHAPE,
             "pc_rebase: Hkv=%d Hsel=%d D=%d row0=%d n_rows=%d", Hkv, Hsel, D, row0, n_rows);
  PC_REQUIRE(sec_t >= 0 && sec_h >= 0 && sec_w >= 0 && sec_t % 2 == 0 && sec_t + sec_h + sec_w == D, PC_ERR_SHAPE,
             "pc_rebase: sections %d+%d+%d must add up to D=%d, temporal width even", sec_t, sec_h, sec_w, D);
  const int elems = dtype == PC_BF16 ? 8 : 4;  // per 16-byte chunk
  PC_REQUIRE(sec_t % elems == 0 && D % elems == 0 && sec_t <= 2 * kMaxPairs, PC_ERR_UNSUPPORTED,
             "pc_rebase: temporal section of %d elements is not a whole number of 16-byte chunks", sec_t);
  PC_REQUIRE(base > 0.0, PC_ERR_SHAPE, "pc_rebase: base %g", base);
  if (n_rows == 0 || delta_t == 0) return PC_OK;
  PC_REQUIRE(K && pos, PC_ERR_NULL, "pc_rebase: K or pos is NULL");
  PC_REQUIRE((k_stride_h >= static_cast<int64_t>(row0 + n_rows) * D || Hkv == 1) &&
                 (pos_stride_h >= static_cast<int64_t>(row0 + n_rows) * 3 || Hsel == 1),
             PC_ERR_SHAPE, "pc_rebase: a head stride is smaller than the rows it must hold");
  PC_REQUIRE((k_stride_h * (dtype == PC_BF16 ? 2 : 4)) % 16 == 0 && reinterpret_cast<uintptr_t>(K) % 16 == 0,
             PC_ERR_SHAPE, "pc_rebase: K and its head stride must be 16-byte aligned");
  RebaseTable tab;
  for (int i = 0; i < kMaxPairs; ++i) {
    double ang = 0.0;
    if (i < sec_t / 2) ang = -static_cast<double>(delta_t) * pow(base, -2.0 * i / sec_t);
    tab.cs[i] = make_float2(static_cast<float>(cos(ang)), static_cast<float>(sin(ang)));
  }
  const int chunks_t = sec_t / elems;
  if (chunks_t == 0) return PC_OK;  // no temporal section: positions only would change nothing the keys encode
  const int64_t total = static_cast<int64_t>(Hkv) * n_rows * chunks_t;
  const dim3 grid(static_cast<unsigned>((total + kThreads - 1) / kThreads));
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (dtype == PC_BF16)
    rebase_kernel<uint16_t><<<grid, kThreads, 0, s>>>(static_cast<uint16_t*>(K), Hkv, D, k_stride_h, pos, Hsel,
                                                      pos_stride_h, row0, n_rows, delta_t, chunks_t, tab);
  else
    rebase_kernel<float><<<grid, kThreads, 0, s>>>(static_cast<float*>(K), Hkv, D, k_stride_h, pos, Hsel,
                                                   pos_stride_h, row0, n_rows, delta_t, chunks_t, tab);
  PC_CHECK_LAUNCH("pc_rebase");
  return PC_OK;
}
