// pc_frame_attn: attention of one frame's queries over the keys presented (Eq. 2).
//
// bf16 tier (D = 128): flash-style kernel on the gfx950 32x32x16 bf16 MFMA.
//   * A work-group is 4 waves; each wave owns 64 query rows (two 32-row blocks) of one
//     query head, so a K/V tile staged in LDS is reused by 256 rows.
//   * Scores are formed transposed, S^T = K Q^T: in the MFMA result layout a lane then
//     holds ONE query column and 16 keys per 32-key block.  The running max / sum of a
//     query are per-lane scalars (one cross-lane exchange per tile), and the probabilities
//     are already laid out as the B operand of the second product O^T += V^T P^T, so P
//     never goes through LDS.
//   * V is transposed on its way into LDS (4 keys x 8 dims per thread, register
//     shuffle, 8-byte LDS stores) so that the A operand of V^T P^T is one 16-byte LDS read.
//   * Softmax in fp32 with base-2 exponentials; accumulators are rescaled only when a
//     row maximum moves.
// fp32 tier (D = 64 or 128): one query row per thread, plain FMA; the correctness tier.
#include <math.h>

#include "common.h"

namespace pc {
namespace {

constexpr int kD = 128;
constexpr int kWaves = 4;
constexpr int kThreads = kWaves * 64;
constexpr int kRowsPerWave = 64;
constexpr int kBM = kWaves * kRowsPerWave;  // 256 query rows per work-group
constexpr int kBN = 64;                     // keys per tile
constexpr int kKStride = kD + 8;            // bf16 per K row in LDS (272 B: conflict-free 16-B reads)
constexpr int kVStride = kBN + 8;           // bf16 per V^T row in LDS (144 B)
constexpr int kKTile = kBN * kKStride;      // elements
constexpr int kVTile = kD * kVStride;
constexpr size_t kSmemBytes = 2 * (kKTile + kVTile) * sizeof(uint16_t);

__device__ __forceinline__ float wave_half_swap(float v) { return __shfl_xor(v, 32, 64); }

// Position, inside its 16-key step, at which key offset o (0..15) is stored in the V^T
// tile: the lane group g = bit 2 and the register half a = bit 3 of the MFMA result
// layout trade places, so a lane's 8 contraction slots are contiguous in LDS.
__device__ __forceinline__ int vt_slot(int o) {
  return (o & ~12) | ((o & 4) << 1) | ((o & 8) >> 1);
}

// ------------------------------------------------------------------------------------------
// Ping-pong kernel: 8 waves, two per SIMD, 32 query rows each.  The two waves of a SIMD
// are kept half an iteration apart by the work-group barrier: while one group of four
// waves is in its MFMA phase (O^T += V^T P^T of the previous tile, then S^T = K Q^T of
// the current one) the other is in its VALU phase (softmax of its current tile, staging
// of the next tile into LDS), so the matrix pipe and the vector ALU overlap.
// Group 0 stages K, group 1 stages V.  LDS buffers alternate per tile.
// ------------------------------------------------------------------------------------------
constexpr int kPPThreads = 512;
constexpr float kLazyRescale = 8.f;  // base-2 exponent range allowed before re-referencing

// One MFMA phase of the ping-pong kernel: the 16 products of O^T += V^T P^T (key step
// i/4, output block i%4) interleaved one-for-one with the 16 of S^T = K Q^T (contraction
// step i/2, key block i%2), which gives six independent accumulator chains.  LDS fragment
// reads run kRing products ahead of their use so the matrix pipe does not wait on LDS.
__device__ __forceinline__ void pp_mfma_phase(const uint16_t* __restrict__ vt_lane,
                                              const uint16_t* __restrict__ ks_lane, f32x16 (&o)[4],
                                              f32x16 (&acc)[2], const bf16x8 (&pf)[4],
                                              const bf16x8 (&qf)[8]) {
  constexpr int kRing = 6;
  auto frag = [&](int k) -> bf16x8 {
    const int i = k >> 1;
    if ((k & 1) == 0)
      return *reinterpret_cast<const bf16x8*>(vt_lane + (i & 3) * 32 * kVStride + (i >> 2) * 16);
    return *reinterpret_cast<const bf16x8*>(ks_lane + (i & 1) * 32 * kKStride + (i >> 1) * 16);
  };
  bf16x8 ring[kRing];
#pragma unroll
  for (int r = 0; r < kRing; ++r) ring[r] = frag(r);
  f32x16 zero;
#pragma unroll
  for (int i = 0; i < 16; ++i) zero[i] = 0.f;
#pragma unroll
  for (int k = 0; k < 32; ++k) {
    const int r = k % kRing, i = k >> 1;
    if ((k & 1) == 0) {
      o[i & 3] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[r], pf[i >> 2], o[i & 3], 0, 0, 0);
    } else {
      const int st = i >> 1, kb = i & 1;
      acc[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ring[r], qf[st], st == 0 ? zero : acc[kb], 0, 0, 0);
    }
    if (k + kRing < 32) ring[r] = frag(k + kRing);
  }
  // pin the issue order: kRing LDS reads up front, then one read behind every product
  __builtin_amdgcn_sched_group_barrier(0x100, kRing, 0);
#pragma unroll
  for (int k = 0; k < 32 - kRing; ++k) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
  }
  __builtin_amdgcn_sched_group_barrier(0x008, kRing, 0);
}

__global__ __launch_bounds__(kPPThreads, 1) void attn_bf16_pp_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    uint16_t* __restrict__ O, float* __restrict__ lse, int rep, int Nq, int Nk, int64_t q_stride_h,
    int64_t kv_stride_h, int64_t o_stride_h, float c, int n_tiles_q, int group_shift) {
  extern __shared__ __align__(16) uint8_t smem_raw[];
  uint16_t* ks_base = reinterpret_cast<uint16_t*>(smem_raw);
  uint16_t* vt_base = ks_base + 2 * kKTile;

  const int lane = threadIdx.x & 63;
  const int wave = threadIdx.x >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  // the two waves that share a SIMD must land in different groups
  const int group = group_shift ? (wave >> 2) : (wave & 1);
  const int wsub = group_shift ? (wave & 3) : (wave >> 1);
  const int L = xcd_contiguous_index(blockIdx.x, gridDim.x);
  const int h = L / n_tiles_q, tile = L % n_tiles_q;
  const int kvh = h / rep;
  const int row0 = tile * kBM + wave * 32;
  const bool active = row0 < Nq;  // wave-uniform

  const uint16_t* Qh = Q + h * q_stride_h;
  const uint16_t* Kh = K + kvh * kv_stride_h;
  const uint16_t* Vh = V + kvh * kv_stride_h;

  bf16x8 qf[8];
  {
    const int row = min(row0 + l32, Nq - 1);
#pragma unroll
    for (int s = 0; s < 8; ++s)
      qf[s] = *reinterpret_cast<const bf16x8*>(Qh + static_cast<int64_t>(row) * kD + s * 16 + g * 8);
  }
  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  f32x16 acc[2];
  bf16x8 pf[4];
#pragma unroll
  for (int k4 = 0; k4 < 4; ++k4)
#pragma unroll
    for (int e = 0; e < 8; ++e) pf[k4][e] = static_cast<__bf16>(0.f);
  float m_ref = -INFINITY, l_run = 0.f;
  // V^T buffer 1 is read (against zero probabilities) before its first tile arrives
  for (int e = threadIdx.x; e < kVTile / 8; e += kPPThreads)
    reinterpret_cast<u32x4*>(vt_base + kVTile)[e] = u32x4{0u, 0u, 0u, 0u};

  // staging roles: group 0 moves K rows, group 1 moves (and transposes) V
  const int t256 = wsub * 64 + lane;
  const int kc = t256 & 15, kr = t256 >> 4;
  const int kg = lane & 15, dc = wsub * 4 + (lane >> 4);
  const int vslot = ((kg * 4) & ~15) | vt_slot((kg * 4) & 15);
  // Two register sets: tile t travels in set t & 1, loaded two tiles ahead of its LDS store.
  u32x4 pre0[4], pre1[4];
  auto stage_load = [&](u32x4 (&pre)[4], int t) {
    const int k0 = t * kBN;
    if (group == 0) {
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int key = min(k0 + kr + 16 * i, Nk - 1);
        pre[i] = *reinterpret_cast<const u32x4*>(Kh + static_cast<int64_t>(key) * kD + kc * 8);
      }
    } else {
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const int key = min(k0 + kg * 4 + j, Nk - 1);
        pre[j] = *reinterpret_cast<const u32x4*>(Vh + static_cast<int64_t>(key) * kD + dc * 8);
      }
    }
  };
  auto stage_store = [&](const u32x4 (&pre)[4], int t) {
    const int buf = t & 1;
    if (group == 0) {
      uint16_t* ks = ks_base + buf * kKTile;
#pragma unroll
      for (int i = 0; i < 4; ++i)
        *reinterpret_cast<u32x4*>(ks + (kr + 16 * i) * kKStride + kc * 8) = pre[i];
    } else {
      uint16_t* vt = vt_base + buf * kVTile;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int w = e >> 1;
        u32x2 out;
        if (e & 1) {
          out[0] = (pre[0][w] >> 16) | (pre[1][w] & 0xFFFF0000u);
          out[1] = (pre[2][w] >> 16) | (pre[3][w] & 0xFFFF0000u);
        } else {
          out[0] = (pre[0][w] & 0xFFFFu) | (pre[1][w] << 16);
          out[1] = (pre[2][w] & 0xFFFFu) | (pre[3][w] << 16);
        }
        *reinterpret_cast<u32x2*>(vt + (dc * 8 + e) * kVStride + vslot) = out;
      }
    }
  };

  const int n = (Nk + kBN - 1) / kBN;
  stage_load(pre0, 0);
  if (n > 1) stage_load(pre1, 1);
  if (group == 0) {
    stage_store(pre0, 0);
    if (n > 2) stage_load(pre0, 2);
  }
  __syncthreads();

  for (int p = 0; p < 2 * n + 2; ++p) {
    const int j = (p - group) >> 1;  // tile this group works on (-1 / n: nothing to compute)
    if (((p + group) & 1) == 0) {
      // ---------------- MFMA phase: PV of tile j-1, then S of tile j ----------------
      if (active) {
        __builtin_amdgcn_s_setprio(1);
        const uint16_t* vt_lane = vt_base + ((j - 1) & 1) * kVTile + l32 * kVStride + g * 8;
        const uint16_t* ks_lane = ks_base + (j & 1) * kKTile + l32 * kKStride + g * 8;
        // Always both products: at j = 0 the P fragments are zero and the V^T buffer was
        // zero-filled, at j = n the scores computed from a stale K buffer are never used.
        pp_mfma_phase(vt_lane, ks_lane, o, acc, pf, qf);
        __builtin_amdgcn_s_setprio(0);
      }
    } else {
      // ---------------- VALU phase: softmax of tile j, stage tile j+1 ----------------
      if (active && j >= 0 && j < n) {
        const int k0 = j * kBN;
        if (k0 + kBN > Nk) {
          const int lim = Nk - k0 - g * 4;  // first invalid key offset, seen from this lane
#pragma unroll
          for (int kb = 0; kb < 2; ++kb)
#pragma unroll
            for (int i = 0; i < 16; ++i)
              if (kb * 32 + (i >> 2) * 8 + (i & 3) >= lim) acc[kb][i] = -INFINITY;
        }
        float mx = acc[0][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc[kb][i]);
        mx = fmaxf(mx, wave_half_swap(mx)) * c;
        if (__any(mx > m_ref + kLazyRescale)) {
          const float m_new = mx > m_ref + kLazyRescale ? mx : m_ref;
          const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
          l_run *= alpha;
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
          m_ref = m_new;
        }
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          float pv[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            pv[i] = __builtin_amdgcn_exp2f(fmaf(acc[kb][i], c, -m_ref));
            psum += pv[i];
          }
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            bf16x8 f;
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = static_cast<__bf16>(pv[half * 8 + e]);
            pf[kb * 2 + half] = f;
          }
        }
        l_run += psum;
      }
      const int t = j + 1;
      if (t & 1) {
        if (t < n) stage_store(pre1, t);
        if (t + 2 < n) stage_load(pre1, t + 2);
      } else {
        if (t < n) stage_store(pre0, t);
        if (t + 2 < n) stage_load(pre0, t + 2);
      }
    }
    __syncthreads();
  }

  if (!active) return;
  const float l_tot = l_run + wave_half_swap(l_run);
  const float inv = 1.f / l_tot;
  const int row = row0 + l32;
  if (row < Nq) {
    uint16_t* orow = O + h * o_stride_h + static_cast<int64_t>(row) * kD;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        u32x2 out;
        out[0] = pack_bf16x2(o[db][a * 4 + 0] * inv, o[db][a * 4 + 1] * inv);
        out[1] = pack_bf16x2(o[db][a * 4 + 2] * inv, o[db][a * 4 + 3] * inv);
        *reinterpret_cast<u32x2*>(orow + db * 32 + a * 8 + g * 4) = out;
      }
    if (lse != nullptr && g == 0)
      lse[static_cast<int64_t>(h) * Nq + row] = (m_ref + log2f(l_tot)) * 0.6931471805599453f;
  }
}

// ------------------------------------------------------------------------------------------
// fp32 correctness tier: one query row per thread, K/V tiles broadcast from LDS.
// ------------------------------------------------------------------------------------------
constexpr int kF32Threads = 64;
constexpr int kF32Tile = 16;

template <int D>
__global__ __launch_bounds__(kF32Threads) void attn_f32_kernel(
    const float* __restrict__ Q, const float* __restrict__ K, const float* __restrict__ V,
    float* __restrict__ O, float* __restrict__ lse, int rep, int Nq, int Nk, int64_t q_stride_h,
    int64_t kv_stride_h, int64_t o_stride_h, float scale) {
  __shared__ float ks[kF32Tile][D];
  __shared__ float vs[kF32Tile][D];
  const int h = blockIdx.y, kvh = h / rep;
  const int row = blockIdx.x * kF32Threads + threadIdx.x;
  const int rowc = min(row, Nq - 1);
  const float* qrow = Q + h * q_stride_h + static_cast<int64_t>(rowc) * D;
  float q[D], acc[D];
#pragma unroll
  for (int d = 0; d < D; ++d) {
    q[d] = qrow[d];
    acc[d] = 0.f;
  }
  float m = -INFINITY, l = 0.f;
  const float* Kh = K + kvh * kv_stride_h;
  const float* Vh = V + kvh * kv_stride_h;
  for (int k0 = 0; k0 < Nk; k0 += kF32Tile) {
    const int nt = min(kF32Tile, Nk - k0);
    __syncthreads();
    for (int e = threadIdx.x; e < nt * D; e += kF32Threads) {
      ks[e / D][e % D] = Kh[static_cast<int64_t>(k0) * D + e];
      vs[e / D][e % D] = Vh[static_cast<int64_t>(k0) * D + e];
    }
    __syncthreads();
    float s[kF32Tile];
    float mt = m;
#pragma unroll
    for (int j = 0; j < kF32Tile; ++j) {
      float dot = 0.f;
      if (j < nt) {
#pragma unroll
        for (int d = 0; d < D; ++d) dot = fmaf(q[d], ks[j][d], dot);
        s[j] = dot * scale;
        mt = fmaxf(mt, s[j]);
      } else {
        s[j] = -INFINITY;
      }
    }
    const float alpha = expf(m - mt);  // exp(-inf) = 0 on the first tile
    l *= alpha;
#pragma unroll
    for (int d = 0; d < D; ++d) acc[d] *= alpha;
#pragma unroll
    for (int j = 0; j < kF32Tile; ++j) {
      if (j < nt) {
        const float p = expf(s[j] - mt);
        l += p;
#pragma unroll
        for (int d = 0; d < D; ++d) acc[d] = fmaf(p, vs[j][d], acc[d]);
      }
    }
    m = mt;
  }
  if (row < Nq) {
    float* orow = O + h * o_stride_h + static_cast<int64_t>(row) * D;
    const float inv = 1.f / l;
#pragma unroll
    for (int d = 0; d < D; ++d) orow[d] = acc[d] * inv;
    if (lse) lse[static_cast<int64_t>(h) * Nq + row] = m + logf(l);
  }
}

}  // namespace
}  // namespace pc

using namespace pc;

extern "C" size_t pc_frame_attn_workspace_bytes(int, int, int, int) { return 0; }

extern "C" int pc_frame_attn(const void* Q, const void* K, const void* V, int dtype, int Hq,
                             int Hkv, int Nq, int Nk, int D, int64_t q_stride_h,
                             int64_t kv_stride_h, int64_t o_stride_h, float scale, void* O,
                             float* lse, void* /*ws*/, size_t /*ws_bytes*/, void* stream) {
  PC_REQUIRE(dtype == PC_F32 || dtype == PC_BF16, PC_ERR_DTYPE, "pc_frame_attn: dtype %d", dtype);
  PC_REQUIRE(Hq > 0 && Hkv > 0 && Hq % Hkv == 0, PC_ERR_SHAPE,
             "pc_frame_attn: Hq=%d must be a positive multiple of Hkv=%d", Hq, Hkv);
  PC_REQUIRE(Nq >= 1 && Nk >= 1, PC_ERR_SHAPE, "pc_frame_attn: Nq=%d Nk=%d must be >= 1", Nq, Nk);
  PC_REQUIRE(scale > 0.f && isfinite(scale), PC_ERR_SHAPE, "pc_frame_attn: scale %g must be > 0", scale);
  PC_REQUIRE(Q && K && V && O, PC_ERR_NULL, "pc_frame_attn: Q, K, V or O is NULL");
  PC_REQUIRE(q_stride_h >= static_cast<int64_t>(Nq) * D && o_stride_h >= static_cast<int64_t>(Nq) * D &&
                 kv_stride_h >= static_cast<int64_t>(Nk) * D,
             PC_ERR_SHAPE, "pc_frame_attn: a head stride is smaller than rows*D");
  hipStream_t s = static_cast<hipStream_t>(stream);
  const int rep = Hq / Hkv;
  if (dtype == PC_BF16) {
    PC_REQUIRE(D == kD, PC_ERR_UNSUPPORTED, "pc_frame_attn: bf16 tier needs D=128, got %d", D);
    const uintptr_t al = reinterpret_cast<uintptr_t>(Q) | reinterpret_cast<uintptr_t>(K) |
                         reinterpret_cast<uintptr_t>(V) | reinterpret_cast<uintptr_t>(O);
    PC_REQUIRE(al % 16 == 0 && q_stride_h % 8 == 0 && kv_stride_h % 8 == 0 && o_stride_h % 8 == 0,
               PC_ERR_SHAPE, "pc_frame_attn: bf16 tensors and head strides must be 16-byte aligned");
    static bool attr_set = false;
    if (!attr_set) {
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_pp_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         static_cast<int>(kSmemBytes));
      if (e != hipSuccess) PC_FAIL(PC_ERR_HIP, "pc_frame_attn: LDS attribute: %s", hipGetErrorString(e));
      attr_set = true;
    }
    const int n_tiles_q = ceil_div(Nq, kBM);
    const float c = scale * 1.4426950408889634f;
    attn_bf16_pp_kernel<<<dim3(n_tiles_q * Hq), kPPThreads, kSmemBytes, s>>>(
        static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
        static_cast<const uint16_t*>(V), static_cast<uint16_t*>(O), lse, rep, Nq, Nk, q_stride_h,
        kv_stride_h, o_stride_h, c, n_tiles_q, 1);
  } else {
    PC_REQUIRE(D == 64 || D == 128, PC_ERR_UNSUPPORTED, "pc_frame_attn: fp32 tier needs D=64 or 128, got %d", D);
    const dim3 grid(ceil_div(Nq, kF32Threads), Hq);
    if (D == 64)
      attn_f32_kernel<64><<<grid, kF32Threads, 0, s>>>(
          static_cast<const float*>(Q), static_cast<const float*>(K), static_cast<const float*>(V),
          static_cast<float*>(O), lse, rep, Nq, Nk, q_stride_h, kv_stride_h, o_stride_h, scale);
    else
      attn_f32_kernel<128><<<grid, kF32Threads, 0, s>>>(
          static_cast<const float*>(Q), static_cast<const float*>(K), static_cast<const float*>(V),
          static_cast<float*>(O), lse, rep, Nq, Nk, q_stride_h, kv_stride_h, o_stride_h, scale);
  }
  PC_CHECK_LAUNCH("pc_frame_attn");
  return PC_OK;
}
