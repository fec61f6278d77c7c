// pc_score: importance of every cached key = the softmax probability (Eq. 2) it receives,
// summed over the scoring queries and the query heads of its KV group.
//
// Two passes over Q K^T, both on the 32x32x16 bf16 MFMA and both free of atomics so the
// result is bit-reproducible:
//   1. row pass:    log-sum-exp of every scoring query over all keys (keys split over
//                   work-groups, partial (max, sum) pairs merged in a fixed order);
//   2. column pass: key-stationary.  A work-group owns 256 keys (staged once in LDS),
//                   streams all scoring queries of the KV group past them, forms
//                   p = exp2(c*s - lse2) with the FINAL normaliser, un-rounded, in fp32,
//                   and sums p down the query axis.
// A caller that already has the log-sum-exp skips pass 1.
#include <math.h>

#include <algorithm>

#include "common.h"

namespace pc {
namespace {

constexpr int kD = 128;
constexpr int kThreads = 256;
constexpr int kKStride = kD + 8;  // bf16 per key row in LDS
constexpr int kMaxSplits = 32;

__device__ __forceinline__ float wave_half_swap(float v) { return __shfl_xor(v, 32, 64); }

// ---- pass 1: per-query (max, sum) over a slice of the keys ---------------------------------
constexpr int kRowBN = 64;
constexpr int kRowBM = 256;

__global__ __launch_bounds__(kThreads, 1) void score_rowpass_bf16(
    const uint16_t* __restrict__ Qs, const int32_t* __restrict__ q_rows,
    const uint16_t* __restrict__ K, float2* __restrict__ part, int Hq, int rep, int n_qs, int Nk, int64_t q_stride_h, int64_t k_stride_h, float c,
    int n_row_tiles, int n_splits) {
  __shared__ __align__(16) uint16_t ks[2][kRowBN * kKStride];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int split = blockIdx.y;
  const int h = blockIdx.x / n_row_tiles, tile = blockIdx.x % n_row_tiles;
  const int kvh = h / rep;
  const int row0 = tile * kRowBM + wave * 64;
  const bool active = row0 < n_qs;
  const uint16_t* Qh = Qs + h * q_stride_h;
  const uint16_t* Kh = K + kvh * k_stride_h;

  bf16x8 qf[2][8];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    int row = min(row0 + qb * 32 + l32, n_qs - 1);
    if (q_rows) row = q_rows[row];
#pragma unroll
    for (int s = 0; s < 8; ++s)
      qf[qb][s] = *reinterpret_cast<const bf16x8*>(Qh + static_cast<int64_t>(row) * kD + s * 16 + g * 8);
  }
  const int n_tiles = (Nk + kRowBN - 1) / kRowBN;
  const int per = (n_tiles + n_splits - 1) / n_splits;
  const int t_begin = min(split * per, n_tiles), t_end = min(t_begin + per, n_tiles);

  float m_run[2] = {-INFINITY, -INFINITY}, l_run[2] = {0.f, 0.f};
  const int kc = threadIdx.x & 15, kr = threadIdx.x >> 4;
  u32x4 regs[4];
  auto load = [&](int t) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int key = min(t * kRowBN + kr + 16 * i, Nk - 1);
      regs[i] = *reinterpret_cast<const u32x4*>(Kh + static_cast<int64_t>(key) * kD + kc * 8);
    }
  };
  auto store = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
      *reinterpret_cast<u32x4*>(&ks[buf][(kr + 16 * i) * kKStride + kc * 8]) = regs[i];
  };
  if (t_begin < t_end) {
    load(t_begin);
    store(0);
  }
  __syncthreads();
  for (int t = t_begin; t < t_end; ++t) {
    const int buf = (t - t_begin) & 1;
    const bool more = t + 1 < t_end;
    if (more) load(t + 1);
    if (active) {
      f32x16 acc[2][2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[kb][qb][i] = 0.f;
#pragma unroll
      for (int s = 0; s < 8; ++s)
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const bf16x8 kf =
              *reinterpret_cast<const bf16x8*>(&ks[buf][(kb * 32 + l32) * kKStride + s * 16 + g * 8]);
#pragma unroll
          for (int qb = 0; qb < 2; ++qb)
            acc[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][s], acc[kb][qb], 0, 0, 0);
        }
      const int k0 = t * kRowBN;
      if (k0 + kRowBN > Nk) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (k0 + kb * 32 + (i >> 2) * 8 + g * 4 + (i & 3) >= Nk) {
              acc[kb][0][i] = -INFINITY;
              acc[kb][1][i] = -INFINITY;
            }
      }
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        float mx = acc[0][qb][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc[kb][qb][i]);
        mx = fmaxf(mx, wave_half_swap(mx));
        const float m_new = fmaxf(m_run[qb], mx * c);
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) psum += __builtin_amdgcn_exp2f(fmaf(acc[kb][qb][i], c, -m_new));
        l_run[qb] = l_run[qb] * __builtin_amdgcn_exp2f(m_run[qb] - m_new) + psum;
        m_run[qb] = m_new;
      }
    }
    if (more) store(buf ^ 1);
    __syncthreads();
  }
  if (!active) return;
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const float l_tot = l_run[qb] + wave_half_swap(l_run[qb]);
    const int row = row0 + qb * 32 + l32;
    if (g == 0 && row < n_qs)
      part[(static_cast<int64_t>(split) * Hq + h) * n_qs + row] = make_float2(m_run[qb], l_tot);
  }
}

// merge the per-split (max, sum) pairs in split order: lse2 = log2 sum_j 2^(c * s_j)
__global__ void score_merge_rows(const float2* __restrict__ part, float* __restrict__ lse2,
                                 int n_rows, int n_splits) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= n_rows) return;
  float m = -INFINITY;
  for (int s = 0; s < n_splits; ++s) m = fmaxf(m, part[static_cast<int64_t>(s) * n_rows + r].x);
  float l = 0.f;
  for (int s = 0; s < n_splits; ++s) {
    const float2 p = part[static_cast<int64_t>(s) * n_rows + r];
    if (p.y > 0.f) l += p.y * exp2f(p.x - m);
  }
  lse2[r] = m + log2f(l);
}

// ---- pass 2: key-stationary column mass ---------------------------------------------------
constexpr int kColKeys = 256;
constexpr size_t kColSmem = kColKeys * kKStride * sizeof(uint16_t) + 4 * kColKeys * sizeof(float);

__global__ __launch_bounds__(kThreads, 2) void score_colpass_bf16(
    const uint16_t* __restrict__ Qs, const int32_t* __restrict__ q_rows,
    const uint16_t* __restrict__ K, const float* __restrict__ lse, float lse_mul, float* __restrict__ score, int64_t score_stride_h, int rep, int n_qs, int Nk,
    int64_t q_stride_h, int64_t k_stride_h, float c) {
  extern __shared__ __align__(16) uint8_t smem_raw[];
  uint16_t* ks = reinterpret_cast<uint16_t*>(smem_raw);
  float* red = reinterpret_cast<float*>(smem_raw + kColKeys * kKStride * sizeof(uint16_t));

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  const int kvh = blockIdx.y;
  const int key0 = blockIdx.x * kColKeys;
  const uint16_t* Kh = K + kvh * k_stride_h;
  {
    const int kc = threadIdx.x & 15, kr = threadIdx.x >> 4;
#pragma unroll 4
    for (int i = 0; i < kColKeys / 16; ++i) {
      const int key = min(key0 + kr + 16 * i, Nk - 1);
      *reinterpret_cast<u32x4*>(ks + (kr + 16 * i) * kKStride + kc * 8) =
          *reinterpret_cast<const u32x4*>(Kh + static_cast<int64_t>(key) * kD + kc * 8);
    }
  }
  __syncthreads();

  float colsum[8];
#pragma unroll
  for (int kb = 0; kb < 8; ++kb) colsum[kb] = 0.f;

  const int chunks_per_head = (n_qs + 63) / 64;
  const int n_chunks = rep * chunks_per_head;
  for (int chunk = wave; chunk < n_chunks; chunk += 4) {
    const int h = kvh * rep + chunk / chunks_per_head;
    const int row0 = (chunk % chunks_per_head) * 64;
    const uint16_t* Qh = Qs + h * q_stride_h;
    const float* lh = lse + static_cast<int64_t>(h) * n_qs;
    bf16x8 qf[2][8];
    float lq[2][16];
#pragma unroll
    for (int qb = 0; qb < 2; ++qb) {
      int row = min(row0 + qb * 32 + l32, n_qs - 1);
      if (q_rows) row = q_rows[row];
#pragma unroll
      for (int s = 0; s < 8; ++s)
        qf[qb][s] = *reinterpret_cast<const bf16x8*>(Qh + static_cast<int64_t>(row) * kD + s * 16 + g * 8);
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        const int r = row0 + qb * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
        lq[qb][i] = r < n_qs ? lh[r] * lse_mul : INFINITY;  // rows past the end add nothing
      }
    }
#pragma unroll
    for (int kb = 0; kb < 8; ++kb) {
      f32x16 acc[2];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[qb][i] = 0.f;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
        const bf16x8 kf =
            *reinterpret_cast<const bf16x8*>(ks + (kb * 32 + l32) * kKStride + s * 16 + g * 8);
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
          acc[qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(qf[qb][s], kf, acc[qb], 0, 0, 0);
      }
      float sum = 0.f;
#pragma unroll
      for (int qb = 0; qb < 2; ++qb)
#pragma unroll
        for (int i = 0; i < 16; ++i) sum += __builtin_amdgcn_exp2f(fmaf(acc[qb][i], c, -lq[qb][i]));
      colsum[kb] += sum;
    }
  }
#pragma unroll
  for (int kb = 0; kb < 8; ++kb) {
    const float v = colsum[kb] + wave_half_swap(colsum[kb]);
    if (g == 0) red[wave * kColKeys + kb * 32 + l32] = v;
  }
  __syncthreads();
  const int key = key0 + threadIdx.x;
  if (key < Nk) {
    const int t = threadIdx.x;
    score[kvh * score_stride_h + key] =
        ((red[t] + red[kColKeys + t]) + red[2 * kColKeys + t]) + red[3 * kColKeys + t];
  }
}

// sum the per-KV-head mass over heads, head 0 first
__global__ void score_share_heads(const float* __restrict__ per_head, float* __restrict__ out,
                                  int Hkv, int Nk) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= Nk) return;
  float s = 0.f;
  for (int g = 0; g < Hkv; ++g) s += per_head[static_cast<int64_t>(g) * Nk + j];
  out[j] = s;
}

// ---- fp32 correctness tier ------------------------------------------------------------------
constexpr int kF32Tile = 16;

template <int D>
__global__ __launch_bounds__(64) void score_rowpass_f32(const float* __restrict__ Qs,
                                                        const int32_t* __restrict__ q_rows,
                                                        const float* __restrict__ K,
                                                        float* __restrict__ lse, int rep, int n_qs,
                                                        int Nk, int64_t q_stride_h,
                                                        int64_t k_stride_h, float scale) {
  __shared__ float ks[kF32Tile][D];
  const int h = blockIdx.y, kvh = h / rep;
  const int row = blockIdx.x * 64 + threadIdx.x;
  int qr = min(row, n_qs - 1);
  if (q_rows) qr = q_rows[qr];
  const float* qrow = Qs + h * q_stride_h + static_cast<int64_t>(qr) * D;
  float q[D];
#pragma unroll
  for (int d = 0; d < D; ++d) q[d] = qrow[d];
  const float* Kh = K + kvh * k_stride_h;
  float m = -INFINITY, l = 0.f;
  for (int k0 = 0; k0 < Nk; k0 += kF32Tile) {
    const int nt = min(kF32Tile, Nk - k0);
    __syncthreads();
    for (int e = threadIdx.x; e < nt * D; e += 64) ks[e / D][e % D] = Kh[static_cast<int64_t>(k0) * D + e];
    __syncthreads();
    float s[kF32Tile], mt = m;
#pragma unroll
    for (int j = 0; j < kF32Tile; ++j) {
      s[j] = -INFINITY;
      if (j < nt) {
        float dot = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) dot = fmaf(q[d], ks[j][d], dot);
        s[j] = dot * scale;
        mt = fmaxf(mt, s[j]);
      }
    }
    l *= expf(m - mt);
#pragma unroll
    for (int j = 0; j < kF32Tile; ++j)
      if (j < nt) l += expf(s[j] - mt);
    m = mt;
  }
  if (row < n_qs) lse[static_cast<int64_t>(h) * n_qs + row] = m + logf(l);
}

template <int D>
__global__ __launch_bounds__(64) void score_colpass_f32(const float* __restrict__ Qs,
                                                        const int32_t* __restrict__ q_rows,
                                                        const float* __restrict__ K,
                                                        const float* __restrict__ lse,
                                                        float* __restrict__ score,
                                                        int64_t score_stride_h, int rep, int n_qs,
                                                        int Nk, int64_t q_stride_h,
                                                        int64_t k_stride_h, float scale) {
  __shared__ float qs[kF32Tile][D];
  __shared__ float ls[kF32Tile];
  const int kvh = blockIdx.y;
  const int key = blockIdx.x * 64 + threadIdx.x;
  const float* krow = K + kvh * k_stride_h + static_cast<int64_t>(min(key, Nk - 1)) * D;
  float k[D];
#pragma unroll
  for (int d = 0; d < D; ++d) k[d] = krow[d];
  float sum = 0.f;
  for (int r = 0; r < rep; ++r) {
    const int h = kvh * rep + r;
    const float* Qh = Qs + h * q_stride_h;
    for (int r0 = 0; r0 < n_qs; r0 += kF32Tile) {
      const int nt = min(kF32Tile, n_qs - r0);
      __syncthreads();
      for (int e = threadIdx.x; e < nt * D; e += 64) {
        const int qr = q_rows ? q_rows[r0 + e / D] : r0 + e / D;
        qs[e / D][e % D] = Qh[static_cast<int64_t>(qr) * D + e % D];
      }
      if (threadIdx.x < nt) ls[threadIdx.x] = lse[static_cast<int64_t>(h) * n_qs + r0 + threadIdx.x];
      __syncthreads();
      for (int j = 0; j < nt; ++j) {
        float dot = 0.f;
#pragma unroll
        for (int d = 0; d < D; ++d) dot = fmaf(qs[j][d], k[d], dot);
        sum += expf(dot * scale - ls[j]);
      }
    }
  }
  if (key < Nk) score[kvh * score_stride_h + key] = sum;
}

struct WsLayout {
  size_t lse_off, part_off, heads_off, total;
};

WsLayout ws_layout(int Hq, int Hkv, int n_qs, int Nk, int share_heads) {
  WsLayout w;
  size_t at = 0;
  w.lse_off = at;
  at += align_up(sizeof(float) * static_cast<size_t>(Hq) * n_qs, 256);
  w.part_off = at;
  at += align_up(sizeof(float2) * static_cast<size_t>(kMaxSplits) * Hq * n_qs, 256);
  w.heads_off = at;
  if (share_heads) at += align_up(sizeof(float) * static_cast<size_t>(Hkv) * Nk, 256);
  w.total = at;
  return w;
}

}  // namespace
}  // namespace pc

using namespace pc;

extern "C" size_t pc_score_workspace_bytes(int Hq, int Hkv, int n_qs, int Nk, int share_heads) {
  if (Hq <= 0 || Hkv <= 0 || n_qs <= 0 || Nk <= 0) return 0;
  return ws_layout(Hq, Hkv, n_qs, Nk, share_heads).total;
}

extern "C" int pc_score(const void* Qs, const void* K, int dtype, int Hq, int Hkv, int n_qs,
                        int Nk, int D, int64_t q_stride_h, int64_t k_stride_h,
                        const int32_t* q_rows, float scale, const float* lse, float* score, int64_t score_stride_h, int share_heads,
                        void* ws, size_t ws_bytes, void* stream) {
  PC_REQUIRE(dtype == PC_F32 || dtype == PC_BF16, PC_ERR_DTYPE, "pc_score: dtype %d", dtype);
  PC_REQUIRE(Hq > 0 && Hkv > 0 && Hq % Hkv == 0, PC_ERR_SHAPE,
             "pc_score: Hq=%d must be a positive multiple of Hkv=%d", Hq, Hkv);
  PC_REQUIRE(n_qs >= 1 && Nk >= 1, PC_ERR_SHAPE, "pc_score: n_qs=%d Nk=%d must be >= 1", n_qs, Nk);
  PC_REQUIRE(scale > 0.f && isfinite(scale), PC_ERR_SHAPE, "pc_score: scale %g must be > 0", scale);
  PC_REQUIRE(Qs && K && score, PC_ERR_NULL, "pc_score: Qs, K or score is NULL");
  PC_REQUIRE((q_rows != nullptr || q_stride_h >= static_cast<int64_t>(n_qs) * D || Hq == 1) &&
                 (k_stride_h >= static_cast<int64_t>(Nk) * D || Hkv == 1),
             PC_ERR_SHAPE, "pc_score: a head stride is smaller than rows*D");
  PC_REQUIRE(share_heads || Hkv == 1 || score_stride_h >= Nk, PC_ERR_SHAPE,
             "pc_score: score head stride %lld < Nk", static_cast<long long>(score_stride_h));
  const WsLayout lay = ws_layout(Hq, Hkv, n_qs, Nk, share_heads);
  PC_REQUIRE(ws != nullptr && ws_bytes >= lay.total, PC_ERR_WORKSPACE,
             "pc_score: workspace %zu bytes, need %zu", ws_bytes, lay.total);
  PC_REQUIRE(reinterpret_cast<uintptr_t>(ws) % 16 == 0, PC_ERR_WORKSPACE, "pc_score: workspace not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* wsb = static_cast<uint8_t*>(ws);
  float* ws_lse = reinterpret_cast<float*>(wsb + lay.lse_off);
  float2* ws_part = reinterpret_cast<float2*>(wsb + lay.part_off);
  float* per_head = share_heads ? reinterpret_cast<float*>(wsb + lay.heads_off) : score;
  const int64_t per_head_stride = share_heads ? Nk : score_stride_h;
  const int rep = Hq / Hkv;

  if (dtype == PC_BF16) {
    PC_REQUIRE(D == kD, PC_ERR_UNSUPPORTED, "pc_score: bf16 tier needs D=128, got %d", D);
    const uintptr_t al = reinterpret_cast<uintptr_t>(Qs) | reinterpret_cast<uintptr_t>(K);
    PC_REQUIRE(al % 16 == 0 && q_stride_h % 8 == 0 && k_stride_h % 8 == 0, PC_ERR_SHAPE,
               "pc_score: bf16 tensors and head strides must be 16-byte aligned");
    const float c = scale * 1.4426950408889634f;
    const float* lse_in = lse;
    float lse_mul = 1.4426950408889634f;  // caller's natural-log LSE -> base 2
    if (lse == nullptr) {
      const int n_row_tiles = ceil_div(n_qs, kRowBM);
      const int n_tiles = ceil_div(Nk, kRowBN);
      int n_splits = ceil_div(1024, n_row_tiles * Hq);
      n_splits = std::max(1, std::min(std::min(n_splits, kMaxSplits), n_tiles));
      score_rowpass_bf16<<<dim3(n_row_tiles * Hq, n_splits), kThreads, 0, s>>>(
          static_cast<const uint16_t*>(Qs), q_rows, static_cast<const uint16_t*>(K), ws_part, Hq, rep, n_qs, Nk,
          q_stride_h, k_stride_h, c, n_row_tiles, n_splits);
      PC_CHECK_LAUNCH("pc_score row pass");
      const int n_rows = Hq * n_qs;
      score_merge_rows<<<ceil_div(n_rows, 256), 256, 0, s>>>(ws_part, ws_lse, n_rows, n_splits);
      PC_CHECK_LAUNCH("pc_score merge");
      lse_in = ws_lse;
      lse_mul = 1.f;
    }
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(score_colpass_bf16),
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         static_cast<int>(kColSmem));
      if (e != hipSuccess) PC_FAIL(PC_ERR_HIP, "pc_score: LDS attribute: %s", hipGetErrorString(e));
      attr_set = true;
    }
    score_colpass_bf16<<<dim3(ceil_div(Nk, kColKeys), Hkv), kThreads, kColSmem, s>>>(
        static_cast<const uint16_t*>(Qs), q_rows, static_cast<const uint16_t*>(K), lse_in, lse_mul, per_head,
        per_head_stride, rep, n_qs, Nk, q_stride_h, k_stride_h, c);
    PC_CHECK_LAUNCH("pc_score column pass");
  } else {
    PC_REQUIRE(D == 64 || D == 128, PC_ERR_UNSUPPORTED, "pc_score: fp32 tier needs D=64 or 128, got %d", D);
    const float* q = static_cast<const float*>(Qs);
    const float* k = static_cast<const float*>(K);
    const float* lse_in = lse;
    if (lse == nullptr) {
      const dim3 grid(ceil_div(n_qs, 64), Hq);
      if (D == 64)
        score_rowpass_f32<64><<<grid, 64, 0, s>>>(q, q_rows, k, ws_lse, rep, n_qs, Nk, q_stride_h, k_stride_h, scale);
      else
        score_rowpass_f32<128><<<grid, 64, 0, s>>>(q, q_rows, k, ws_lse, rep, n_qs, Nk, q_stride_h, k_stride_h, scale);
      PC_CHECK_LAUNCH("pc_score row pass");
      lse_in = ws_lse;
    }
    const dim3 grid(ceil_div(Nk, 64), Hkv);
    if (D == 64)
      score_colpass_f32<64><<<grid, 64, 0, s>>>(q, q_rows, k, lse_in, per_head, per_head_stride, rep, n_qs, Nk,
                                                  q_stride_h, k_stride_h, scale);
    else
      score_colpass_f32<128><<<grid, 64, 0, s>>>(q, q_rows, k, lse_in, per_head, per_head_stride, rep, n_qs, Nk,
                                                   q_stride_h, k_stride_h, scale);
    PC_CHECK_LAUNCH("pc_score column pass");
  }
  if (share_heads) {
    score_share_heads<<<ceil_div(Nk, 256), 256, 0, s>>>(per_head, score, Hkv, Nk);
    PC_CHECK_LAUNCH("pc_score head sum");
  }
  return PC_OK;
}
