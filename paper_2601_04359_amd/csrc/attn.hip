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

struct TileRegs {
  u32x4 k[4];
  u32x4 v[4];
};

__device__ __forceinline__ void load_tile(TileRegs& r, const uint16_t* __restrict__ Kh,
                                          const uint16_t* __restrict__ Vh, int k0, int Nk) {
  const int t = threadIdx.x;
  // K: 16 threads cover one 256-byte row
  const int kc = t & 15, kr = t >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int key = min(k0 + kr + 16 * i, Nk - 1);
    r.k[i] = *reinterpret_cast<const u32x4*>(Kh + static_cast<int64_t>(key) * kD + kc * 8);
  }
  // V: a thread takes 4 consecutive keys x 8 dims
  const int lane = t & 63, wave = t >> 6;
  const int kg = lane & 15, dc = wave * 4 + (lane >> 4);
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    const int key = min(k0 + kg * 4 + j, Nk - 1);
    r.v[j] = *reinterpret_cast<const u32x4*>(Vh + static_cast<int64_t>(key) * kD + dc * 8);
  }
}

__device__ __forceinline__ void store_tile(const TileRegs& r, uint16_t* ks, uint16_t* vt) {
  const int t = threadIdx.x;
  const int kc = t & 15, kr = t >> 4;
#pragma unroll
  for (int i = 0; i < 4; ++i)
    *reinterpret_cast<u32x4*>(ks + (kr + 16 * i) * kKStride + kc * 8) = r.k[i];
  const int lane = t & 63, wave = t >> 6;
  const int kg = lane & 15, dc = wave * 4 + (lane >> 4);
  const int o = kg * 4;
  const int slot = (o & ~15) | vt_slot(o & 15);
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    const int w = e >> 1;
    u32x2 out;
    if (e & 1) {
      out[0] = (r.v[0][w] >> 16) | (r.v[1][w] & 0xFFFF0000u);
      out[1] = (r.v[2][w] >> 16) | (r.v[3][w] & 0xFFFF0000u);
    } else {
      out[0] = (r.v[0][w] & 0xFFFFu) | (r.v[1][w] << 16);
      out[1] = (r.v[2][w] & 0xFFFFu) | (r.v[3][w] << 16);
    }
    *reinterpret_cast<u32x2*>(vt + (dc * 8 + e) * kVStride + slot) = out;
  }
}

__global__ __launch_bounds__(kThreads, 1) void attn_bf16_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    uint16_t* __restrict__ O, float* __restrict__ lse, int rep, int Nq, int Nk, int64_t q_stride_h,
    int64_t kv_stride_h, int64_t o_stride_h, float c, int n_tiles_q) {
  extern __shared__ __align__(16) uint8_t smem_raw[];
  uint16_t* ks_base = reinterpret_cast<uint16_t*>(smem_raw);
  uint16_t* vt_base = ks_base + 2 * kKTile;

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int l32 = lane & 31, g = lane >> 5;
  // logical order (head, query tile): heads of one KV group are adjacent, and the
  // XCD-contiguous mapping keeps a KV group's work-groups on as few L2s as possible.
  const int L = xcd_contiguous_index(blockIdx.x, gridDim.x);
  const int h = L / n_tiles_q, tile = L % n_tiles_q;
  const int kvh = h / rep;
  const int row0 = tile * kBM + wave * kRowsPerWave;
  const bool active = row0 < Nq;  // wave-uniform

  const uint16_t* Qh = Q + h * q_stride_h;
  const uint16_t* Kh = K + kvh * kv_stride_h;
  const uint16_t* Vh = V + kvh * kv_stride_h;

  // Q fragments (B operand of S^T = K Q^T): lane holds row l32 of each 32-row block,
  // dims s*16 + g*8 .. +8 of every 16-wide contraction step.
  bf16x8 qf[2][8];
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const int row = min(row0 + qb * 32 + l32, Nq - 1);
#pragma unroll
    for (int s = 0; s < 8; ++s)
      qf[qb][s] = *reinterpret_cast<const bf16x8*>(Qh + static_cast<int64_t>(row) * kD + s * 16 + g * 8);
  }

  f32x16 o[4][2];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int qb = 0; qb < 2; ++qb)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][qb][i] = 0.f;
  float m_run[2] = {-INFINITY, -INFINITY};  // running max of c * logit, per lane's query
  float l_run[2] = {0.f, 0.f};              // this lane's share of the running sum

  const int n_tiles = (Nk + kBN - 1) / kBN;
  TileRegs regs;
  load_tile(regs, Kh, Vh, 0, Nk);
  store_tile(regs, ks_base, vt_base);
  __syncthreads();

  for (int j = 0; j < n_tiles; ++j) {
    const int buf = j & 1;
    const uint16_t* ks = ks_base + buf * kKTile;
    const uint16_t* vt = vt_base + buf * kVTile;
    const bool more = j + 1 < n_tiles;
    if (more) load_tile(regs, Kh, Vh, (j + 1) * kBN, Nk);

    if (active) {
      // ---- S^T = K Q^T -----------------------------------------------------------------
      f32x16 acc[2][2];
#pragma unroll
      for (int kb = 0; kb < 2; ++kb)
#pragma unroll
        for (int qb = 0; qb < 2; ++qb)
#pragma unroll
          for (int i = 0; i < 16; ++i) acc[kb][qb][i] = 0.f;
#pragma unroll
      for (int s = 0; s < 8; ++s) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          const bf16x8 kf =
              *reinterpret_cast<const bf16x8*>(ks + (kb * 32 + l32) * kKStride + s * 16 + g * 8);
#pragma unroll
          for (int qb = 0; qb < 2; ++qb)
            acc[kb][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[qb][s], acc[kb][qb], 0, 0, 0);
        }
      }
      // keys past the end of the cache (last tile only) get probability zero
      const int k0 = j * kBN;
      if (k0 + kBN > Nk) {
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            const int key = k0 + kb * 32 + (i >> 2) * 8 + g * 4 + (i & 3);
            if (key >= Nk) {
              acc[kb][0][i] = -INFINITY;
              acc[kb][1][i] = -INFINITY;
            }
          }
      }
      // ---- online softmax (per lane: one query per 32-row block) ---------------------
      bf16x8 pf[2][4];
#pragma unroll
      for (int qb = 0; qb < 2; ++qb) {
        float mx = acc[0][qb][0];
#pragma unroll
        for (int kb = 0; kb < 2; ++kb)
#pragma unroll
          for (int i = 0; i < 16; ++i) mx = fmaxf(mx, acc[kb][qb][i]);
        mx = fmaxf(mx, wave_half_swap(mx));
        const float m_new = fmaxf(m_run[qb], mx * c);
        const float alpha = __builtin_amdgcn_exp2f(m_run[qb] - m_new);
        float psum = 0.f;
#pragma unroll
        for (int kb = 0; kb < 2; ++kb) {
          float p[16];
#pragma unroll
          for (int i = 0; i < 16; ++i) {
            p[i] = __builtin_amdgcn_exp2f(fmaf(acc[kb][qb][i], c, -m_new));
            psum += p[i];
          }
#pragma unroll
          for (int half = 0; half < 2; ++half) {
            bf16x8 f;
#pragma unroll
            for (int e = 0; e < 8; ++e) f[e] = static_cast<__bf16>(p[half * 8 + e]);
            pf[qb][kb * 2 + half] = f;
          }
        }
        l_run[qb] = l_run[qb] * alpha + psum;
        if (__any(m_new != m_run[qb])) {
#pragma unroll
          for (int db = 0; db < 4; ++db)
#pragma unroll
            for (int i = 0; i < 16; ++i) o[db][qb][i] *= alpha;
        }
        m_run[qb] = m_new;
      }
      // ---- O^T += V^T P^T ----------------------------------------------------------------
#pragma unroll
      for (int ks16 = 0; ks16 < 4; ++ks16) {
#pragma unroll
        for (int db = 0; db < 4; ++db) {
          const bf16x8 vf =
              *reinterpret_cast<const bf16x8*>(vt + (db * 32 + l32) * kVStride + ks16 * 16 + g * 8);
#pragma unroll
          for (int qb = 0; qb < 2; ++qb)
            o[db][qb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[qb][ks16], o[db][qb], 0, 0, 0);
        }
      }
    }

    if (more) store_tile(regs, ks_base + (buf ^ 1) * kKTile, vt_base + (buf ^ 1) * kVTile);
    __syncthreads();
  }

  if (!active) return;
  // ---- normalise and store: lane holds O^T[d = db*32 + a*8 + g*4 + b][query l32] ---------
#pragma unroll
  for (int qb = 0; qb < 2; ++qb) {
    const float l_tot = l_run[qb] + wave_half_swap(l_run[qb]);
    const float inv = 1.f / l_tot;
    const int row = row0 + qb * 32 + l32;
    if (row < Nq) {
      uint16_t* orow = O + h * o_stride_h + static_cast<int64_t>(row) * kD;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          u32x2 out;
          out[0] = pack_bf16x2(o[db][qb][a * 4 + 0] * inv, o[db][qb][a * 4 + 1] * inv);
          out[1] = pack_bf16x2(o[db][qb][a * 4 + 2] * inv, o[db][qb][a * 4 + 3] * inv);
          *reinterpret_cast<u32x2*>(orow + db * 32 + a * 8 + g * 4) = out;
        }
      if (lse != nullptr && g == 0)
        lse[static_cast<int64_t>(h) * Nq + row] = (m_run[qb] + log2f(l_tot)) * 0.6931471805599453f;
    }
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
      hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(attn_bf16_kernel),
                                         hipFuncAttributeMaxDynamicSharedMemorySize,
                                         static_cast<int>(kSmemBytes));
      if (e != hipSuccess) PC_FAIL(PC_ERR_HIP, "pc_frame_attn: LDS attribute: %s", hipGetErrorString(e));
      attr_set = true;
    }
    const int n_tiles_q = ceil_div(Nq, kBM);
    const float c = scale * 1.4426950408889634f;
    attn_bf16_kernel<<<dim3(n_tiles_q * Hq), kThreads, kSmemBytes, s>>>(
        static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
        static_cast<const uint16_t*>(V), static_cast<uint16_t*>(O), lse, rep, Nq, Nk, q_stride_h,
        kv_stride_h, o_stride_h, c, n_tiles_q);
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
