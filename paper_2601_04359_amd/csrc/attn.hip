// pc_frame_attn: attention of one frame's queries over the keys presented (Eq. 2).
//
// bf16 tier (D = 128): flash-style kernel on the gfx950 32x32x16 bf16 MFMA.
//   * Scores are formed transposed, S^T = K Q^T: in the MFMA result layout a lane then
//     holds ONE query column and 16 keys per 32-key block.  The reference maximum and the
//     running sum of a query are per-lane scalars, and the probabilities are already laid
//     out as the B operand of the second product O^T += V^T P^T, so P never goes through LDS.
//   * K and V tiles are fetched straight from global memory into LDS (no register
//     staging), four tiles deep; V stays row-major in LDS and is transposed by the LDS
//     transposing read on its way into the MFMA A operand.
//   * Softmax in fp32 with base-2 exponentials, interleaved instruction by instruction with
//     the products of the neighbouring half tiles.  No row maximum is taken on the fast path:
//     probabilities are formed against the standing reference, and a half tile is redone
//     (and the accumulators rescaled) only when one of its row sums runs away.
//   * With scale = ln 2 (the caller multiplied Q by scale * log2(e), e.g. while rotating it)
//     the affine step c*s - m is taken out of the loop: see kUnitC below.
// fp32 tier (D = 64 or 128): one query row per thread, plain FMA; the correctness tier.
#include <math.h>

#include <type_traits>

#include "lds_dma.h"

namespace pc {
namespace {

constexpr int kD = 128;
constexpr int kPPThreads = 512;      // 8 waves, two per SIMD
constexpr int kBM = 256;             // query rows per work-group (32 per wave)
constexpr int kBN = 64;              // keys per tile
constexpr int kRowBytes = kD * 2;    // a K or V row in LDS: 256 bytes, unpadded, chunk-swizzled
constexpr int kTileBytes = kBN * kRowBytes;
constexpr int kStages = 4;           // LDS slots per operand: tile t lives in slot t % kStages
constexpr size_t kSmemBytes = 2 * kStages * kTileBytes;
constexpr float kRescaleTrigger = 1024.f;  // row sum of a half tile that forces a new reference maximum
constexpr int kRing = 4;

// ---- LDS tile layout ---------------------------------------------------------------------------
// K tiles use the fragment-read swizzle of lds_dma.h.  V is read with transposing loads
// (4 rows x 32 bytes per quarter wave): chunk c of row r is stored at position c ^ (4 (r & 3)).
__device__ __forceinline__ int v_chunk_pos(int row, int chunk) { return chunk ^ ((row & 3) << 2); }

// Wait until at most 4 (kStages - 2) of this wave's direct loads are still in flight: every
// staging point issues exactly four, so all but the newest kStages - 2 points have landed.
__device__ __forceinline__ void dma_wait_older() { asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); }
static_assert(kStages == 4, "dma_wait_older encodes 4 * (kStages - 2)");

// Stage tile rows [k0, k0+64) of K or V: each of the 8 waves issues two 1-KB loads.
template <bool kIsV>
__device__ __forceinline__ void stage_tile(const uint16_t* __restrict__ base_h, int k0, int Nk, uint32_t lds_tile,
                                           int wave, int lane) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = (wave * 2 + i) * 4 + (lane >> 4);  // 4 rows per load
    const int pos = lane & 15;                          // chunk position inside the row
    const int chunk = kIsV ? v_chunk_pos(row, pos) : k_chunk_pos(row, pos);  // both maps are involutions
    const int key = min(k0 + row, Nk - 1);
    dma_16B(base_h + static_cast<int64_t>(key) * kD + chunk * 8, lds_tile + (wave * 2 + i) * 1024);
  }
}

// One phase of the software pipeline (see the kernel comment): 8 score products, then 8
// value products, with one element of the probability stage behind each.
// The probabilities are formed against the reference m_ref as it stands; no maximum is
// taken on the fast path.  If any row sum of the half tile comes out above kRescaleTrigger
// (a score outgrew the reference: rare, at most once per 2^10 of growth), the half tile is
// redone against its exact maximum and O, l are rescaled.
// kUnitC: the caller folded scale * log2(e) into Q (c == 1).  The score products then start
// from -m_ref instead of zero (neg_m: the reference in all 16 accumulator registers of the
// lane, which holds one query), so a score arrives as s - m_ref and the probability is a bare
// exp2: one vector instruction per element fewer.  When the reference moves, the scores that
// were started from the old one are shifted by the difference.
template <bool kUnitC>
__device__ __forceinline__ void pipeline_phase(
    const lds_u8* k_half, const int (&k_off)[8], const lds_u8* v_half, const int (&v_off)[4],
    const bf16x8 (&qf)[8], f32x16& s_nxt, const bf16x8 (&p_mm)[2], f32x16 (&o)[4], const f32x16& s_cur,
    bf16x8 (&p_cur)[2], float& m_ref, float& l_run, float c, f32x16& neg_m) {
  // fragment k: 0..7 -> K rows, contraction step k; 8..15 -> V^T (key step (k-8)/4, block (k-8)%4)
  auto frag = [&](int k) -> bf16x8 {
    if (k < 8) {
      return *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(k_half + k_off[k]);
    }
    const int ks = (k - 8) >> 2, db = (k - 8) & 3;
    // keys ks*16 + g*4 + {0..3} and + 8: two transposing reads of 4 keys each
    const lds_u8* p = v_half + v_off[db] + ks * 16 * kRowBytes;
    const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        reinterpret_cast<__attribute__((address_space(3))) bf16x4*>(const_cast<lds_u8*>(p)));
    const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
        reinterpret_cast<__attribute__((address_space(3))) bf16x4*>(const_cast<lds_u8*>(p + 8 * kRowBytes)));
    bf16x8 f;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      f[e] = lo[e];
      f[4 + e] = hi[e];
    }
    return f;
  };
  bf16x8 ring[kRing];
#pragma unroll
  for (int r = 0; r < kRing; ++r) ring[r] = frag(r);
  f32x16 zero;
#pragma unroll
  for (int i = 0; i < 16; ++i) zero[i] = 0.f;
  f32x16 s_acc = zero;
  float psum = 0.f;
  float pv[16];
  // The wave asks for issue priority over its SIMD neighbour while it is inside the interleaved
  // matrix / vector block, and gives it back for the bookkeeping behind it (measured: +0.5 %).
  __builtin_amdgcn_s_setprio(1);
#pragma unroll
  for (int k = 0; k < 16; ++k) {
    const bf16x8 f = ring[k % kRing];
    if (k < 8) {
      s_acc = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, qf[k], k == 0 ? (kUnitC ? neg_m : zero) : s_acc, 0, 0, 0);
    } else {
      const int ks = (k - 8) >> 2, db = (k - 8) & 3;
      o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f, p_mm[ks], o[db], 0, 0, 0);
    }
    if (k + kRing < 16) ring[k % kRing] = frag(k + kRing);
    pv[k] = kUnitC ? __builtin_amdgcn_exp2f(s_cur[k]) : __builtin_amdgcn_exp2f(fmaf(s_cur[k], c, -m_ref));
    psum += pv[k];
    if (k & 1) {
      p_cur[k >> 3][(k & 7) - 1] = static_cast<__bf16>(pv[k - 1]);
      p_cur[k >> 3][k & 7] = static_cast<__bf16>(pv[k]);
    }
    __builtin_amdgcn_sched_barrier(0);
  }
  __builtin_amdgcn_s_setprio(0);
  // keep the vector results in this basic block (otherwise they sink below the next branch)
#pragma unroll
  for (int half = 0; half < 2; ++half) asm volatile("" : "+v"(p_cur[half]));
  asm volatile("" : "+v"(psum));
  if (__any(!(psum <= kRescaleTrigger))) {  // also catches inf and NaN
    float mx = s_cur[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, s_cur[i]);
    // unit c: s_cur already holds s - m_ref, so the new reference lies max(0, max s_cur) above the old one
    const float m_new = kUnitC ? m_ref + fmaxf(0.f, wave_half_max(mx)) : fmaxf(m_ref, wave_half_max(mx) * c);
    const float alpha = __builtin_amdgcn_exp2f(m_ref - m_new);
    psum = 0.f;
#pragma unroll
    for (int i = 0; i < 16; ++i) {
      pv[i] = kUnitC ? __builtin_amdgcn_exp2f(s_cur[i] - (m_new - m_ref)) : __builtin_amdgcn_exp2f(fmaf(s_cur[i], c, -m_new));
      psum += pv[i];
    }
    if constexpr (kUnitC) {   // the scores just formed were started from the old reference
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        s_acc[i] -= m_new - m_ref;
        neg_m[i] = -m_new;
      }
    }
#pragma unroll
    for (int i = 0; i < 16; ++i) p_cur[i >> 3][i & 7] = static_cast<__bf16>(pv[i]);
    l_run *= alpha;
#pragma unroll
    for (int db = 0; db < 4; ++db)
#pragma unroll
      for (int i = 0; i < 16; ++i) o[db][i] *= alpha;
    m_ref = m_new;
  }
  l_run += psum;
  s_nxt = s_acc;
}

// ------------------------------------------------------------------------------------------
// bf16 frame attention.  8 waves (two per SIMD), 32 query rows each, 256 rows per
// work-group; keys in tiles of 64, processed as half tiles A (keys 0..31) and B (32..63).
// On this chip matrix and vector instructions overlap only inside one wave's instruction
// stream, so every wave interleaves, in one basic block per phase,
//     matrix:  S_nxt^T = K_half Q^T (8 products)  and  O^T += V_half^T P_mm^T (8 products)
//     vector:  P_cur = exp2(c S_cur - m_ref), its bf16 packing and its row sum
// where cur is the half tile scored one phase earlier and mm the one before that:
//     phase 1 of tile j:  S_B(j), O += V_B(j-1) P_B(j-1)  |  P_A(j)
//     phase 2 of tile j:  S_A(j+1), O += V_A(j) P_A(j)    |  P_B(j)
// One work-group barrier per tile, after phase 1: behind it K(j+4) and V(j+3) are fetched
// straight into the LDS slots just released (four slots per operand, 128 KB), three tiles
// ahead of their first use.
// ------------------------------------------------------------------------------------------
template <bool kUnitC>
__global__ __launch_bounds__(kPPThreads, 1) void attn_bf16_kernel(
    const uint16_t* __restrict__ Q, const uint16_t* __restrict__ K, const uint16_t* __restrict__ V,
    uint16_t* __restrict__ O, float* __restrict__ lse, int rep, int Nq, int Nk, int64_t q_stride_h,
    int64_t kv_stride_h, int64_t o_stride_h, float c, int n_tiles_q, int n_splits, float* __restrict__ part_o,
    float2* __restrict__ part_ml) {
  extern __shared__ __align__(16) uint8_t smem_raw[];
  lds_u8* smem = (lds_u8*)smem_raw;
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));
  auto k_slot = [&](int t) { return (t & (kStages - 1)) * kTileBytes; };
  auto v_slot = [&](int t) { return (kStages + (t & (kStages - 1))) * kTileBytes; };

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, g = lane >> 5;
  const int L = xcd_contiguous_index(blockIdx.x, gridDim.x);
  // logical order: key split slowest, then head, then row tile
  const int Hq_tiles = static_cast<int>(gridDim.x) / n_splits;
  const int split = L / Hq_tiles;
  const int h = (L % Hq_tiles) / n_tiles_q, tile = L % n_tiles_q;
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
    // Make the compiler retire these loads here: otherwise it guards every use of qf inside
    // the loop with s_waitcnt vmcnt(7..0), which also drains the direct K/V loads in flight.
#pragma unroll
    for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(qf[s]));
  }
  f32x16 o[4];
#pragma unroll
  for (int db = 0; db < 4; ++db)
#pragma unroll
    for (int i = 0; i < 16; ++i) o[db][i] = 0.f;
  f32x16 sA, sB;
  bf16x8 pA[2], pB[2];
#pragma unroll
  for (int ks = 0; ks < 2; ++ks)
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      pA[ks][e] = static_cast<__bf16>(0.f);
      pB[ks][e] = static_cast<__bf16>(0.f);
    }
  float m_ref = -INFINITY, l_run = 0.f;
  f32x16 neg_m;
#pragma unroll
  for (int i = 0; i < 16; ++i) neg_m[i] = 0.f;

  // per-lane byte offsets inside a half tile
  int k_off[8];  // K fragment of contraction step s: row l32, chunk 2s+g
#pragma unroll
  for (int s = 0; s < 8; ++s) k_off[s] = l32 * kRowBytes + k_chunk_pos(l32, 2 * s + g) * 16;
  int v_off[4];  // V^T fragment of output block db: this lane SUPPLIES row g*4 + r/4, dims db*32 + G*16 + 4(r%4)
  {
    const int r = lane & 15, G = (lane >> 4) & 1;
    const int row = g * 4 + (r >> 2);
#pragma unroll
    for (int db = 0; db < 4; ++db) {
      const int dim = db * 32 + G * 16 + 4 * (r & 3);
      v_off[db] = row * kRowBytes + v_chunk_pos(row, dim >> 3) * 16 + (dim & 7) * 2;
    }
  }

  // this work-group's share of the key tiles: [t0, t0 + n) of n_all (the host leaves no share empty)
  const int n_all = (Nk + kBN - 1) / kBN;
  const int per = (n_all + n_splits - 1) / n_splits;
  const int t0 = split * per;
  const int n = min(per, n_all - t0);
  const int key0 = t0 * kBN;
  const bool tail = (Nk % kBN) != 0 && t0 + n == n_all;   // the ragged last tile is in this share
  const int lim_a = Nk - (n_all - 1) * kBN - g * 4;  // last tile: first invalid key offset, half A
  const int lim_b = lim_a - 32;

  // the V slot of "tile -1" is read once against zero probabilities: clear it
  for (int e = threadIdx.x; e < kTileBytes / 16; e += kPPThreads)
    reinterpret_cast<__attribute__((address_space(3))) u32x4*>(smem + v_slot(-1))[e] = u32x4{0u, 0u, 0u, 0u};
  // Prologue, in order of need: K(0), V(0), K(1), then K(2), V(1), K(3), V(2).  Tiles past the
  // end of the cache are fetched too (clamped rows, never read) so that every staging point
  // issues the same number of loads and the in-flight count can be waited on.
  stage_tile<false>(Kh, key0, Nk, lds0 + k_slot(0), wave, lane);
  stage_tile<true>(Vh, key0, Nk, lds0 + v_slot(0), wave, lane);
  stage_tile<false>(Kh, key0 + kBN, Nk, lds0 + k_slot(1), wave, lane);
  stage_tile<false>(Kh, key0 + 2 * kBN, Nk, lds0 + k_slot(2), wave, lane);
  stage_tile<true>(Vh, key0 + kBN, Nk, lds0 + v_slot(1), wave, lane);
  stage_tile<false>(Kh, key0 + 3 * kBN, Nk, lds0 + k_slot(3), wave, lane);
  stage_tile<true>(Vh, key0 + 2 * kBN, Nk, lds0 + v_slot(2), wave, lane);
  dma_wait_older();
  __syncthreads();

  auto mask_tail = [&](f32x16& sc, int lim) {
#pragma unroll
    for (int i = 0; i < 16; ++i)
      if ((i >> 2) * 8 + (i & 3) >= lim) sc[i] = -INFINITY;
  };
  if (active) {  // S_A of tile 0 and the first reference maximum
    f32x16 zero;
#pragma unroll
    for (int i = 0; i < 16; ++i) zero[i] = 0.f;
#pragma unroll
    for (int s = 0; s < 8; ++s) {
      const bf16x8 kf = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(smem + k_slot(0) + k_off[s]);
      sA = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s == 0 ? zero : sA, 0, 0, 0);
    }
    float mx = sA[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) mx = fmaxf(mx, sA[i]);
    m_ref = wave_half_max(mx) * c;
    if constexpr (kUnitC) {
#pragma unroll
      for (int i = 0; i < 16; ++i) {
        sA[i] -= m_ref;
        neg_m[i] = -m_ref;
      }
    }
    if (tail && n == 1) mask_tail(sA, lim_a);
  }

  // Tile j lives in LDS slot j % 4.  The loop is unrolled four times so that every slot is a
  // compile-time constant and lands in the offset field of the LDS reads instead of costing a
  // vector add per fragment address.
  auto tile_body = [&](int j, auto slot_tag) {
    constexpr int u = decltype(slot_tag)::value;            // j % kStages
    constexpr int k_cur = u * kTileBytes, k_nxt = ((u + 1) & 3) * kTileBytes;
    constexpr int v_prev = (kStages + ((u + 3) & 3)) * kTileBytes, v_cur = (kStages + u) * kTileBytes;
    const bool last = j + 1 == n;
    // ---- phase 1: S_B(j), O += V_B(j-1) P_B(j-1)  |  P_A(j) ----
    if (active) {
      pipeline_phase<kUnitC>(smem + k_cur + 32 * kRowBytes, k_off, smem + v_prev + 32 * kRowBytes, v_off, qf, sB, pB, o, sA,
                     pA, m_ref, l_run, c, neg_m);
      if (last && tail) mask_tail(sB, lim_b);
    }
    // One barrier per tile: every wave is past K(j) and V(j-1), and K(j+1), V(j) (fetched
    // kStages - 1 tiles ago) have landed: each wave waited for its own share.
    dma_wait_older();
    __syncthreads();
    stage_tile<false>(Kh, key0 + (j + kStages) * kBN, Nk, lds0 + k_cur, wave, lane);
    stage_tile<true>(Vh, key0 + (j + kStages - 1) * kBN, Nk, lds0 + v_prev, wave, lane);
    // ---- phase 2: S_A(j+1), O += V_A(j) P_A(j)  |  P_B(j) ----
    // (after the last tile S_A is formed from a clamped tile and never used)
    if (active) {
      pipeline_phase<kUnitC>(smem + k_nxt, k_off, smem + v_cur, v_off, qf, sA, pA, o, sB, pB, m_ref, l_run, c, neg_m);
      if (j + 2 == n && tail) mask_tail(sA, lim_a);
    }
  };
  for (int j0 = 0; j0 < n; j0 += kStages) {
    tile_body(j0, std::integral_constant<int, 0>{});
    if (j0 + 1 >= n) break;
    tile_body(j0 + 1, std::integral_constant<int, 1>{});
    if (j0 + 2 >= n) break;
    tile_body(j0 + 2, std::integral_constant<int, 2>{});
    if (j0 + 3 >= n) break;
    tile_body(j0 + 3, std::integral_constant<int, 3>{});
  }
  if (!active) return;
  // ---- drain: O += V_B(n-1) P_B(n-1) ----
  {
    const lds_u8* v_half = smem + v_slot(n - 1) + 32 * kRowBytes;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int db = 0; db < 4; ++db) {
        const lds_u8* p = v_half + v_off[db] + ks * 16 * kRowBytes;
        const bf16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            reinterpret_cast<__attribute__((address_space(3))) bf16x4*>(const_cast<lds_u8*>(p)));
        const bf16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4bf16(
            reinterpret_cast<__attribute__((address_space(3))) bf16x4*>(const_cast<lds_u8*>(p + 8 * kRowBytes)));
        bf16x8 vf;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
          vf[e] = lo[e];
          vf[4 + e] = hi[e];
        }
        o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pB[ks], o[db], 0, 0, 0);
      }
  }
  const float l_tot = wave_half_sum(l_run);
  const int row = row0 + l32;
  if (part_o != nullptr) {  // one of several key shares: un-normalised O, reference and sum for the merge
    if (row < Nq) {
      const int64_t at = (static_cast<int64_t>(split) * gridDim.x / n_splits / n_tiles_q + h) * Nq + row;
      float* prow = part_o + at * kD;
#pragma unroll
      for (int db = 0; db < 4; ++db)
#pragma unroll
        for (int a = 0; a < 4; ++a) {
          f32x4 v;
#pragma unroll
          for (int e = 0; e < 4; ++e) v[e] = o[db][a * 4 + e];
          *reinterpret_cast<f32x4*>(prow + db * 32 + a * 8 + g * 4) = v;
        }
      if (g == 0) part_ml[at] = make_float2(m_ref, l_tot);
    }
    return;
  }
  const float inv = 1.f / l_tot;
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

// Merge of the key shares: O = sum_s 2^(m_s - M) O_s / sum_s 2^(m_s - M) l_s with M = max_s m_s.
// A thread owns four dims of one row.
__global__ __launch_bounds__(256) void attn_merge_kernel(const float* __restrict__ part_o,
                                                         const float2* __restrict__ part_ml,
                                                         uint16_t* __restrict__ O, float* __restrict__ lse,
                                                         int Hq, int Nq, int64_t o_stride_h, int n_splits) {
  const int64_t r = static_cast<int64_t>(blockIdx.x) * 8 + (threadIdx.x >> 5);
  const int c = threadIdx.x & 31;
  const int64_t n_rows = static_cast<int64_t>(Hq) * Nq;
  if (r >= n_rows) return;
  float M = -INFINITY;
  for (int s = 0; s < n_splits; ++s) M = fmaxf(M, part_ml[s * n_rows + r].x);
  float l = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int s = 0; s < n_splits; ++s) {
    const float2 ml = part_ml[s * n_rows + r];
    const float w = __builtin_amdgcn_exp2f(ml.x - M);
    l += w * ml.y;
    const f32x4 v = *reinterpret_cast<const f32x4*>(part_o + (s * n_rows + r) * kD + c * 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[e] += w * v[e];
  }
  const float inv = 1.f / l;
  const int h = static_cast<int>(r / Nq), row = static_cast<int>(r % Nq);
  u32x2 out;
  out[0] = pack_bf16x2(acc[0] * inv, acc[1] * inv);
  out[1] = pack_bf16x2(acc[2] * inv, acc[3] * inv);
  *reinterpret_cast<u32x2*>(O + h * o_stride_h + static_cast<int64_t>(row) * kD + c * 4) = out;
  if (lse != nullptr && c == 0) lse[r] = (M + log2f(l)) * 0.6931471805599453f;
}

// How many shares to cut the keys into: none unless it fills the 256 compute units in whole
// rounds noticeably better (e.g. 24 heads x 16 row tiles = 384 work-groups: 1.5 rounds -> 3 rounds
// of half the length), never so fine that a share's prologue shows.
int choose_key_splits(int base_blocks, int n_tiles) {
  int best = 1;
  double best_score = 0.0;
  for (int s = 1; s <= 4; ++s) {
    const int per = ceil_div(n_tiles, s);
    if (s > 1 && (per < 16 || ceil_div(n_tiles, per) != s)) continue;
    const int blocks = base_blocks * s, rounds = ceil_div(blocks, 256);
    const double score = static_cast<double>(blocks) / (rounds * 256.0) * per / (per + 2.0) * (s == 1 ? 1.08 : 1.0);
    if (score > best_score) {
      best_score = score;
      best = s;
    }
  }
  return best;
}

size_t attn_partial_bytes(int Hq, int Nq, int n_splits) {
  return n_splits <= 1 ? 0
                       : align_up(static_cast<size_t>(n_splits) * Hq * Nq * kD * sizeof(float), 256) +
                             align_up(static_cast<size_t>(n_splits) * Hq * Nq * sizeof(float2), 256);
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

extern "C" size_t pc_frame_attn_workspace_bytes(int Hq, int Nq, int Nk, int D) {
  if (D != kD || Hq <= 0 || Nq <= 0 || Nk <= 0) return 0;   // only the bf16 kernel splits the keys
  return attn_partial_bytes(Hq, Nq, choose_key_splits(Hq * ceil_div(Nq, kBM), ceil_div(Nk, kBN)));
}

extern "C" int pc_frame_attn(const void* Q, const void* K, const void* V, int dtype, int Hq,
                             int Hkv, int Nq, int Nk, int D, int64_t q_stride_h,
                             int64_t kv_stride_h, int64_t o_stride_h, float scale, void* O,
                             float* lse, void* ws, size_t ws_bytes, void* stream) {
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
    const bool unit_c = scale * 1.4426950408889634f == 1.0f;
    static std::atomic<uint64_t> lds_ok{0}, lds_ok_u{0};
    if (int rc = unit_c ? allow_dynamic_lds(reinterpret_cast<const void*>(attn_bf16_kernel<true>), kSmemBytes, lds_ok_u, "pc_frame_attn")
                        : allow_dynamic_lds(reinterpret_cast<const void*>(attn_bf16_kernel<false>), kSmemBytes, lds_ok, "pc_frame_attn"))
      return rc;
    const int n_tiles_q = ceil_div(Nq, kBM);
    const float c = scale * 1.4426950408889634f;
    // Key shares need the caller's workspace for the partial results; without it (or with one
    // that is too small or misaligned) the keys are not split, which is always valid.
    int n_splits = choose_key_splits(Hq * n_tiles_q, ceil_div(Nk, kBN));
    if (ws == nullptr || ws_bytes < attn_partial_bytes(Hq, Nq, n_splits) || reinterpret_cast<uintptr_t>(ws) % 16 != 0)
      n_splits = 1;
    float* part_o = nullptr;
    float2* part_ml = nullptr;
    if (n_splits > 1) {
      part_o = static_cast<float*>(ws);
      part_ml = reinterpret_cast<float2*>(static_cast<uint8_t*>(ws) +
                                          align_up(static_cast<size_t>(n_splits) * Hq * Nq * kD * sizeof(float), 256));
    }
    (unit_c ? attn_bf16_kernel<true> : attn_bf16_kernel<false>)<<<dim3(n_tiles_q * Hq * n_splits), kPPThreads, kSmemBytes, s>>>(
        static_cast<const uint16_t*>(Q), static_cast<const uint16_t*>(K),
        static_cast<const uint16_t*>(V), static_cast<uint16_t*>(O), lse, rep, Nq, Nk, q_stride_h,
        kv_stride_h, o_stride_h, c, n_tiles_q, n_splits, part_o, part_ml);
    if (n_splits > 1) {
      PC_CHECK_LAUNCH("pc_frame_attn");
      attn_merge_kernel<<<static_cast<unsigned>((static_cast<int64_t>(Hq) * Nq + 7) / 8), 256, 0, s>>>(
          part_o, part_ml, static_cast<uint16_t*>(O), lse, Hq, Nq, o_stride_h, n_splits);
    }
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
