// pc_score: importance of every cached key = the softmax probability (Eq. 2) it receives,
// summed over the scoring queries and the query heads of its KV group.
//
// Two passes over Q K^T, both on the 32x32x16 bf16 MFMA and both free of atomics so the
// result is bit-reproducible:
//   1. row pass:    log-sum-exp of every scoring query over all keys (keys split over
//                   work-groups, partial (reference, sum) pairs merged in a fixed order; the
//                   reference is refreshed only when a partial sum runs away);
//   2. column pass: p = exp2(c*s - lse2) with the FINAL normaliser, un-rounded, in fp32,
//                   summed down the query axis (queries split over work-groups, partial
//                   sums added in a fixed order).
// A caller that already has the log-sum-exp skips pass 1.  With scale = ln 2 (the caller folded
// scale * log2(e) into the queries, c == 1) the products of pass 2 start from minus the
// normaliser instead of zero, so an element arrives as s - lse2 and costs a bare exp2.
//
// Both passes have the same shape.  One operand is stationary: every wave keeps 64 of its
// rows as MFMA fragments in registers for the whole kernel (queries in pass 1, keys in
// pass 2).  The other operand streams through a four-slot LDS ring in tiles of 64 rows,
// fetched by direct global->LDS loads three tiles ahead, one work-group barrier per tile.
// Each element of the product costs one exponential, so both passes are bound by the vector
// pipe, not the matrix pipe; matrix and vector instructions overlap only inside one wave's
// instruction stream, so every wave interleaves the 16 products of the next half tile with
// the exponentials of the one before.
#include <math.h>

#include <algorithm>
#include <type_traits>

#include "lds_dma.h"

namespace pc {
namespace {

constexpr int kD = 128;
constexpr int kThreads = 512;        // 8 waves, two per SIMD
constexpr int kWaveRows = 64;        // stationary rows per wave (two 32-row MFMA blocks)
constexpr int kBlockRows = 8 * kWaveRows;
constexpr int kTileRows = 64;        // streamed rows per LDS slot
constexpr int kRowBytes = kD * 2;
constexpr int kTileBytes = kTileRows * kRowBytes;
constexpr int kStages = 4;
constexpr int kLseSlotBytes = kTileRows * 4;
constexpr size_t kRowSmem = kStages * kTileBytes;
constexpr size_t kColSmem = kStages * (kTileBytes + kLseSlotBytes);
constexpr int kMaxSplits = 32;       // key splits of pass 1
constexpr int kMaxQSplits = 8;       // query splits of pass 2
constexpr float kNoMax = -1e30f;     // finite stand-in for "no key seen yet"

// Every staging point issues at most three direct loads per wave; waiting until at most two
// are in flight leaves only (part of) the newest point outstanding.
__device__ __forceinline__ void dma_wait_all_but_newest() { asm volatile("s_waitcnt vmcnt(2)" ::: "memory"); }

// Fetch the two 1-KB pieces of a 64-row tile this wave is responsible for; src(row) is the
// global address of streamed row `row` of the tile.
template <class Src>
__device__ __forceinline__ void stage_rows(Src&& src, uint32_t lds_tile, int wave, int lane) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = (wave * 2 + i) * 4 + (lane >> 4);
    const int chunk = k_chunk_pos(row, lane & 15);
    dma_16B(src(row, i) + chunk * 8, lds_tile + (wave * 2 + i) * 1024);
  }
}

// acc[b] = init(b) + (32 streamed rows at `half`) x (stationary block b)^T, 16 products; after
// each product epi(i) runs one sixteenth of the vector work of the previous half tile.
// kInit = false: the products start from zero and init is not called.
// ring holds the first four fragments of `half` on entry (fetched while the phase before ran) and
// the first four of `next_half` on exit, so that no phase starts by waiting for LDS.
template <bool kInit, class Init, class Epi>
__device__ __forceinline__ void stream_phase(const lds_u8* half, const lds_u8* next_half, const int (&a_off)[8],
                                             const bf16x8 (&st)[2][8], f32x16 (&acc)[2], Init&& init, Epi&& epi,
                                             bf16x8 (&ring)[4]) {
  f32x16 zero;
#pragma unroll
  for (int i = 0; i < 16; ++i) zero[i] = 0.f;
  // issue priority over the SIMD neighbour while inside the interleaved block (measured: +2-3 %)
  __builtin_amdgcn_s_setprio(1);
#pragma unroll
  for (int s = 0; s < 8; ++s) {
    const bf16x8 a = ring[s & 3];
    ring[s & 3] = s + 4 < 8 ? lds_frag(half + a_off[s + 4]) : lds_frag(next_half + a_off[s - 4]);
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      if constexpr (kInit)
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st[b][s], s == 0 ? init(b) : acc[b], 0, 0, 0);
      else
        acc[b] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, st[b][s], s == 0 ? zero : acc[b], 0, 0, 0);
      epi(s * 2 + b);
      __builtin_amdgcn_sched_barrier(0);
    }
  }
  __builtin_amdgcn_s_setprio(0);
}

// ---- pass 1: per-query (max, sum) over a slice of the keys ---------------------------------
// S^T = K Q^T: a lane owns one query column of each stationary block and 16 of the 32 keys
// of the half tile, and keeps its own running (max, sum) over the keys it sees; the two
// halves of the wave are merged once at the end.
struct RowState {
  float m[2], l[2];
};
struct NoInit {
  __device__ const f32x16& operator()(int) const { __builtin_unreachable(); }
};
constexpr float kRowTrigger = 1024.f;  // phase sum that forces a new reference maximum

// Element pair i of the previous half tile: p = exp2(c s - m) against the reference as it
// stands, summed into the phase's partial sums.  No maximum is taken here.
__device__ __forceinline__ void row_epilogue(int i, const f32x16 (&s)[2], const RowState& st, float (&psum)[2],
                                             float c) {
  const int b = i >> 3, e = (i & 7) * 2;
  psum[b] += __builtin_amdgcn_exp2f(fmaf(s[b][e], c, -st.m[b]));
  psum[b] += __builtin_amdgcn_exp2f(fmaf(s[b][e + 1], c, -st.m[b]));
}
// After the phase: add the partial sums; if one ran away (a score outgrew the reference, or
// the reference is still the initial sentinel) redo that half tile against its exact maximum.
__device__ __forceinline__ void row_commit(const f32x16 (&s)[2], RowState& st, float (&psum)[2], float c) {
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    asm volatile("" : "+v"(psum[b]));
    if (__any(!(psum[b] <= kRowTrigger))) {
      float mx = fmaxf(s[b][0], s[b][1]);
#pragma unroll
      for (int k = 2; k < 16; k += 2) mx = fmaxf(mx, fmaxf(s[b][k], s[b][k + 1]));
      const float m_new = fmaxf(st.m[b], mx * c);
      float sum = 0.f;
#pragma unroll
      for (int k = 0; k < 16; ++k) sum += __builtin_amdgcn_exp2f(fmaf(s[b][k], c, -m_new));
      st.l[b] = st.l[b] * __builtin_amdgcn_exp2f(st.m[b] - m_new) + sum;
      st.m[b] = m_new;
    } else {
      st.l[b] += psum[b];
    }
    psum[b] = 0.f;
  }
}

__device__ __forceinline__ void mask_keys(f32x16 (&s)[2], int k0, int Nk, int g) {
#pragma unroll
  for (int i = 0; i < 16; ++i)
    if (k0 + (i >> 2) * 8 + g * 4 + (i & 3) >= Nk) {
      s[0][i] = -INFINITY;
      s[1][i] = -INFINITY;
    }
}

__global__ __launch_bounds__(kThreads, 1) void score_rowpass_bf16(
    const uint16_t* __restrict__ Qs, const int32_t* __restrict__ q_rows, const uint16_t* __restrict__ K,
    float2* __restrict__ part, int Hq, int rep, int n_qs, int Nk, int64_t q_stride_h, int64_t k_stride_h, float c,
    int n_row_tiles, int n_splits) {
  extern __shared__ __align__(16) uint8_t smem_raw[];
  lds_u8* smem = (lds_u8*)smem_raw;
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, g = lane >> 5;
  // logical order: split slowest, so the work-groups of one XCD stream the same keys
  const int L = xcd_contiguous_index(blockIdx.x, gridDim.x);
  const int split = L / (Hq * n_row_tiles);
  const int h = (L / n_row_tiles) % Hq, tile = L % n_row_tiles;
  const int kvh = h / rep;
  const int row0 = tile * kBlockRows + wave * kWaveRows;
  const uint16_t* Qh = Qs + h * q_stride_h;
  const uint16_t* Kh = K + kvh * k_stride_h;

  bf16x8 qf[2][8];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    int row = min(row0 + b * 32 + l32, n_qs - 1);
    if (q_rows) row = q_rows[row];
#pragma unroll
    for (int s = 0; s < 8; ++s)
      qf[b][s] = *reinterpret_cast<const bf16x8*>(Qh + static_cast<int64_t>(row) * kD + s * 16 + g * 8);
  }
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(qf[b][s]));

  const int n_tiles = (Nk + kTileRows - 1) / kTileRows;
  const int per = (n_tiles + n_splits - 1) / n_splits;
  const int t_begin = min(split * per, n_tiles), t_end = min(t_begin + per, n_tiles);
  const int n = t_end - t_begin;
  if (n <= 0) {  // the host never launches an empty split; keep the partials defined anyway
#pragma unroll
    for (int b = 0; b < 2; ++b) {
      const int row = row0 + b * 32 + l32;
      if (g == 0 && row < n_qs) part[(static_cast<int64_t>(split) * Hq + h) * n_qs + row] = make_float2(kNoMax, 0.f);
    }
    return;
  }

  int a_off[8];
#pragma unroll
  for (int s = 0; s < 8; ++s) a_off[s] = l32 * kRowBytes + k_chunk_pos(l32, 2 * s + g) * 16;
  auto stage = [&](int j) {  // tile j of this split (clamped: a repeat of the last tile is never read)
    const int k0 = (t_begin + min(j, n - 1)) * kTileRows;
    stage_rows([&](int row, int) { return Kh + static_cast<int64_t>(min(k0 + row, Nk - 1)) * kD; },
               lds0 + (j & (kStages - 1)) * kTileBytes, wave, lane);
  };
  auto slot = [&](int j) { return smem + (j & (kStages - 1)) * kTileBytes; };

  RowState st;
  st.m[0] = st.m[1] = kNoMax;
  st.l[0] = st.l[1] = 0.f;
  f32x16 sA[2], sB[2];

  float psum[2] = {0.f, 0.f};
  stage(0);
  stage(1);
  stage(2);
  asm volatile("s_waitcnt vmcnt(4)" ::: "memory");
  __syncthreads();
  bf16x8 ring[4];
#pragma unroll
  for (int r = 0; r < 4; ++r) ring[r] = lds_frag(slot(0) + a_off[r]);
  stream_phase<false>(slot(0), slot(0) + 32 * kRowBytes, a_off, qf, sA, NoInit{}, [](int) {}, ring);
  // Tile j lives in LDS slot j % 4; the loop is unrolled over the slots so that their bases are
  // immediates of the LDS reads.
  auto tile_body = [&](int j, auto slot_tag) {
    constexpr int u = decltype(slot_tag)::value;
    const bool tail = (t_begin + j + 1) * kTileRows > Nk;  // only ever the last tile
    dma_wait_all_but_newest();
    __syncthreads();  // tile j+1 has landed everywhere; slot of tile j-1 is free
    stage(j + 3);
    if (tail) mask_keys(sA, (t_begin + j) * kTileRows, Nk, g);
    stream_phase<false>(smem + u * kTileBytes + 32 * kRowBytes, smem + ((u + 1) & 3) * kTileBytes, a_off, qf, sB, NoInit{},
                        [&](int i) { row_epilogue(i, sA, st, psum, c); }, ring);
    row_commit(sA, st, psum, c);
    if (tail) mask_keys(sB, (t_begin + j) * kTileRows + 32, Nk, g);
    if (j + 1 < n) {
      stream_phase<false>(smem + ((u + 1) & 3) * kTileBytes, smem + ((u + 1) & 3) * kTileBytes + 32 * kRowBytes, a_off, qf,
                          sA, NoInit{}, [&](int i) { row_epilogue(i, sB, st, psum, c); }, ring);
    } else {
#pragma unroll
      for (int i = 0; i < 16; ++i) row_epilogue(i, sB, st, psum, c);
    }
    row_commit(sB, st, psum, c);
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
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no direct load may outlive the work-group

#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const float m_o = wave_half_swap(st.m[b]), l_o = wave_half_swap(st.l[b]);
    const float m = fmaxf(st.m[b], m_o);
    const float l = st.l[b] * __builtin_amdgcn_exp2f(st.m[b] - m) + l_o * __builtin_amdgcn_exp2f(m_o - m);
    const int row = row0 + b * 32 + l32;
    if (g == 0 && row < n_qs) part[(static_cast<int64_t>(split) * Hq + h) * n_qs + row] = make_float2(m, l);
  }
}

// Merge the per-split (max, sum) pairs in split order: lse2 = log2 sum_j 2^(c * s_j), stored
// NEGATED (pass 2 adds it).  The result is laid out [head][n_pad] with n_pad a multiple of the
// streamed tile; the padding rows hold -inf so that they add nothing in pass 2.
__global__ void score_merge_rows(const float2* __restrict__ part, float* __restrict__ lse2, int Hq, int n_qs,
                                 int n_pad, int n_splits) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= Hq * n_pad) return;
  const int h = r / n_pad, row = r % n_pad;
  if (row >= n_qs) {
    lse2[r] = -INFINITY;
    return;
  }
  const int64_t n_rows = static_cast<int64_t>(Hq) * n_qs, at = static_cast<int64_t>(h) * n_qs + row;
  float2 p[kMaxSplits];  // all partials first: the loads are independent and overlap
#pragma unroll
  for (int s = 0; s < kMaxSplits; ++s) p[s] = s < n_splits ? part[s * n_rows + at] : make_float2(kNoMax, 0.f);
  float m = -INFINITY;
#pragma unroll
  for (int s = 0; s < kMaxSplits; ++s) m = fmaxf(m, p[s].x);
  float l = 0.f;
#pragma unroll
  for (int s = 0; s < kMaxSplits; ++s)
    if (p[s].y > 0.f) l += p[s].y * exp2f(p[s].x - m);
  lse2[r] = -(m + log2f(l));
}

// A caller's natural-log LSE, indexed like the rows of Qs, -> the dense [head][n_pad] layout
// of pass 2 (times `mul`: -log2(e) for the base-2 kernels, which add the negated normaliser);
// padding rows get `pad`.
__global__ void score_import_lse(const float* __restrict__ lse, int64_t lse_stride_h,
                                 const int32_t* __restrict__ q_rows, float* __restrict__ out, int Hq, int n_qs,
                                 int n_pad, float mul, float pad) {
  const int r = blockIdx.x * blockDim.x + threadIdx.x;
  if (r >= Hq * n_pad) return;
  const int h = r / n_pad, row = r % n_pad;
  out[r] = row < n_qs ? lse[h * lse_stride_h + (q_rows ? q_rows[row] : row)] * mul : pad;
}

// ---- pass 2: column mass --------------------------------------------------------------------
// S = Q K^T: a lane owns one key column of each stationary block and 16 of the 32 query rows
// of the half tile.  The streamed operand is the list of (query head of the group, 64-row
// tile) pairs; the normalisers of a tile travel through LDS beside it.
// nlq: the negated normalisers of the 16 query rows the lane holds.  kUnitC (c == 1): the
// products were started from nlq, so s already holds s - lse2.
template <bool kUnitC>
__device__ __forceinline__ void col_epilogue(int i, const f32x16 (&s)[2], const f32x16& nlq, float (&colsum)[2],
                                             float c) {
  const int b = i >> 3, e = (i & 7) * 2;
  if constexpr (kUnitC) {
    colsum[b] += __builtin_amdgcn_exp2f(s[b][e]);
    colsum[b] += __builtin_amdgcn_exp2f(s[b][e + 1]);
  } else {
    colsum[b] += __builtin_amdgcn_exp2f(fmaf(s[b][e], c, nlq[e]));
    colsum[b] += __builtin_amdgcn_exp2f(fmaf(s[b][e + 1], c, nlq[e + 1]));
  }
}

template <bool kUnitC>
__global__ __launch_bounds__(kThreads, 1) void score_colpass_bf16(
    const uint16_t* __restrict__ Qs, const int32_t* __restrict__ q_rows, const uint16_t* __restrict__ K,
    const float* __restrict__ lse2, float* __restrict__ out, int64_t out_stride_h, int64_t out_stride_split,
    int /*Hkv*/, int rep, int n_qs, int Nk, int64_t q_stride_h, int64_t k_stride_h, float c, int n_key_blocks,
    int n_qsplits) {
  extern __shared__ __align__(16) uint8_t smem_raw[];
  lds_u8* smem = (lds_u8*)smem_raw;
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(smem));
  constexpr int kLse0 = kStages * kTileBytes;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int l32 = lane & 31, g = lane >> 5;
  // logical order: (kv head, query split) slowest, so the work-groups of one XCD stream the same queries
  const int L = xcd_contiguous_index(blockIdx.x, gridDim.x);
  const int kb = L % n_key_blocks, qsplit = (L / n_key_blocks) % n_qsplits, kvh = L / (n_key_blocks * n_qsplits);
  const int key0 = kb * kBlockRows + wave * kWaveRows;
  const uint16_t* Kh = K + kvh * k_stride_h;

  bf16x8 kf[2][8];
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const int key = min(key0 + b * 32 + l32, Nk - 1);
#pragma unroll
    for (int s = 0; s < 8; ++s)
      kf[b][s] = *reinterpret_cast<const bf16x8*>(Kh + static_cast<int64_t>(key) * kD + s * 16 + g * 8);
  }
#pragma unroll
  for (int b = 0; b < 2; ++b)
#pragma unroll
    for (int s = 0; s < 8; ++s) asm volatile("" : "+v"(kf[b][s]));

  const int tiles_per_head = (n_qs + kTileRows - 1) / kTileRows;
  const int n_pad = tiles_per_head * kTileRows;
  const int n_vt = rep * tiles_per_head;
  const int per = (n_vt + n_qsplits - 1) / n_qsplits;
  const int t_begin = min(qsplit * per, n_vt), t_end = min(t_begin + per, n_vt);
  const int n = t_end - t_begin;

  float colsum[2] = {0.f, 0.f};
  if (n > 0) {
    int a_off[8];
#pragma unroll
    for (int s = 0; s < 8; ++s) a_off[s] = l32 * kRowBytes + k_chunk_pos(l32, 2 * s + g) * 16;
    // source row (within its head) of the two pieces this lane fetches for tile j
    auto src_rows = [&](int j, int (&rows)[2]) {
      const int vt = t_begin + min(j, n - 1);
      const int r0 = (vt % tiles_per_head) * kTileRows;
#pragma unroll
      for (int i = 0; i < 2; ++i) {
        const int row = min(r0 + (wave * 2 + i) * 4 + (lane >> 4), n_qs - 1);
        rows[i] = q_rows ? q_rows[row] : row;
      }
    };
    auto stage = [&](int j, const int (&rows)[2]) {
      const int vt = t_begin + min(j, n - 1);
      const int h = kvh * rep + vt / tiles_per_head;
      const uint16_t* Qh = Qs + h * q_stride_h;
      stage_rows([&](int, int i) { return Qh + static_cast<int64_t>(rows[i]) * kD; },
                 lds0 + (j & (kStages - 1)) * kTileBytes, wave, lane);
      if (wave == 0)
        dma_4B(lse2 + static_cast<int64_t>(h) * n_pad + (vt % tiles_per_head) * kTileRows + lane,
               lds0 + kLse0 + (j & (kStages - 1)) * kLseSlotBytes);
    };
    auto slot = [&](int j) { return smem + (j & (kStages - 1)) * kTileBytes; };
    // normalisers of the 16 rows this lane holds in half `half` of tile j
    auto load_lq = [&](int j, int half, f32x16& lq) {
      const lds_u8* base = smem + kLse0 + (j & (kStages - 1)) * kLseSlotBytes + (half * 32 + g * 4) * 4;
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const f32x4 v = *reinterpret_cast<const __attribute__((address_space(3))) f32x4*>(base + q * 32);
#pragma unroll
        for (int e = 0; e < 4; ++e) lq[q * 4 + e] = v[e];
      }
    };

    f32x16 sA[2], sB[2];
    f32x16 lq;            // general path: normalisers of the half tile whose elements the epilogue takes
    f32x16 initA, initB;  // kUnitC: start values of the next sA / sB products, fetched one phase ahead
    auto startA = [&](int) -> const f32x16& { return initA; };
    auto startB = [&](int) -> const f32x16& { return initB; };
    int rows[2];
    src_rows(0, rows);
    stage(0, rows);
    src_rows(1, rows);
    stage(1, rows);
    src_rows(2, rows);
    stage(2, rows);
    src_rows(3, rows);
    asm volatile("s_waitcnt vmcnt(4)" ::: "memory");  // at least the first tile's pieces
    __syncthreads();
    if constexpr (kUnitC) {
      load_lq(0, 0, initA);
      load_lq(0, 1, initB);
    }
    bf16x8 ring[4];
#pragma unroll
    for (int r = 0; r < 4; ++r) ring[r] = lds_frag(slot(0) + a_off[r]);
    stream_phase<kUnitC>(slot(0), slot(0) + 32 * kRowBytes, a_off, kf, sA, startA, [](int) {}, ring);
    auto tile_body = [&](int j, auto slot_tag) {  // slot j % 4 as a compile-time constant, as in pass 1
      constexpr int u = decltype(slot_tag)::value;
      dma_wait_all_but_newest();
      __syncthreads();  // tile j+1 has landed everywhere; slot of tile j-1 is free
      stage(j + 3, rows);
      src_rows(j + 4, rows);
      if constexpr (kUnitC) load_lq((u + 1) & 3, 0, initA); else load_lq(u, 0, lq);
      stream_phase<kUnitC>(smem + u * kTileBytes + 32 * kRowBytes, smem + ((u + 1) & 3) * kTileBytes, a_off, kf, sB, startB,
                           [&](int i) { col_epilogue<kUnitC>(i, sA, lq, colsum, c); }, ring);
      if constexpr (kUnitC) load_lq((u + 1) & 3, 1, initB); else load_lq(u, 1, lq);
      if (j + 1 < n) {
        stream_phase<kUnitC>(smem + ((u + 1) & 3) * kTileBytes, smem + ((u + 1) & 3) * kTileBytes + 32 * kRowBytes, a_off, kf,
                             sA, startA, [&](int i) { col_epilogue<kUnitC>(i, sB, lq, colsum, c); }, ring);
      } else {
#pragma unroll
        for (int i = 0; i < 16; ++i) col_epilogue<kUnitC>(i, sB, lq, colsum, c);
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
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");  // no direct load may outlive the work-group
  }
#pragma unroll
  for (int b = 0; b < 2; ++b) {
    const float v = wave_half_sum(colsum[b]);
    const int key = key0 + b * 32 + l32;
    if (g == 0 && key < Nk) out[qsplit * out_stride_split + kvh * out_stride_h + key] = v;
  }
}

// out[h][j] = sum over parts p of part[p][h][j] (p ascending); with share_heads the heads are
// summed too, head 0 first, into out[j].
__global__ void score_reduce(const float* __restrict__ part, float* __restrict__ out, int64_t out_stride_h,
                             int n_parts, int Hkv, int Nk, int share_heads) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= Nk) return;
  const int64_t split_stride = static_cast<int64_t>(Hkv) * Nk;
  if (share_heads) {
    float s = 0.f;
    for (int h = 0; h < Hkv; ++h) {
      float sh = 0.f;
      for (int p = 0; p < n_parts; ++p) sh += part[p * split_stride + static_cast<int64_t>(h) * Nk + j];
      s += sh;
    }
    out[j] = s;
  } else {
    const int h = blockIdx.y;
    float sh = 0.f;
    for (int p = 0; p < n_parts; ++p) sh += part[p * split_stride + static_cast<int64_t>(h) * Nk + j];
    out[h * out_stride_h + j] = sh;
  }
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
      if (static_cast<int>(threadIdx.x) < nt) ls[threadIdx.x] = lse[static_cast<int64_t>(h) * n_qs + r0 + threadIdx.x];
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
  size_t lse_off, part_off, col_off, total;
};

int padded_rows(int n_qs) { return ceil_div(n_qs, kTileRows) * kTileRows; }

WsLayout ws_layout(int Hq, int Hkv, int n_qs, int Nk, int /*share_heads*/) {
  WsLayout w;
  size_t at = 0;
  w.lse_off = at;
  at += align_up(sizeof(float) * static_cast<size_t>(Hq) * padded_rows(n_qs), 256);
  w.part_off = at;
  at += align_up(sizeof(float2) * static_cast<size_t>(kMaxSplits) * Hq * n_qs, 256);
  w.col_off = at;
  at += align_up(sizeof(float) * static_cast<size_t>(kMaxQSplits) * Hkv * Nk, 256);
  w.total = at;
  return w;
}

// Number of ways to split the streamed axis (n_tiles tiles) so that `base` x splits
// work-groups fill the 256 compute units in whole rounds without making a work-group's
// share so short that its three-tile prologue shows.
int choose_splits(int base, int n_tiles, int max_splits) {
  int best = 1;
  double best_score = -1.0;
  for (int s = 1; s <= std::min(max_splits, n_tiles); ++s) {
    const int blocks = base * s, rounds = ceil_div(blocks, 256), per = ceil_div(n_tiles, s);
    const double score = static_cast<double>(blocks) / (rounds * 256.0) * per / (per + 2.0);
    if (score > best_score * 1.001) {
      best_score = score;
      best = s;
    }
  }
  return best;
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
                        const int32_t* q_rows, float scale, const float* lse, int64_t lse_stride_h, float* score,
                        int64_t score_stride_h, int share_heads, int key_begin, int key_end,
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
  if (key_end <= 0) key_end = Nk;  // 0: up to the last key
  PC_REQUIRE(key_begin >= 0 && key_begin < key_end && key_end <= Nk, PC_ERR_SHAPE,
             "pc_score: key range [%d, %d) outside [0, %d)", key_begin, key_end, Nk);
  // Keys outside the range take part in every normaliser (pass 1 runs over all Nk keys) but get no
  // score: pass 2 simply runs on the sub-range (pointers and counts offset here).
  const int nkr = key_end - key_begin;
  PC_REQUIRE(lse == nullptr || Hq == 1 || lse_stride_h >= n_qs, PC_ERR_SHAPE,
             "pc_score: lse head stride %lld < n_qs", static_cast<long long>(lse_stride_h));
  const WsLayout lay = ws_layout(Hq, Hkv, n_qs, Nk, share_heads);
  PC_REQUIRE(ws != nullptr && ws_bytes >= lay.total, PC_ERR_WORKSPACE,
             "pc_score: workspace %zu bytes, need %zu", ws_bytes, lay.total);
  PC_REQUIRE(reinterpret_cast<uintptr_t>(ws) % 16 == 0, PC_ERR_WORKSPACE, "pc_score: workspace not 16-byte aligned");
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint8_t* wsb = static_cast<uint8_t*>(ws);
  float* ws_lse = reinterpret_cast<float*>(wsb + lay.lse_off);
  float2* ws_part = reinterpret_cast<float2*>(wsb + lay.part_off);
  float* ws_col = reinterpret_cast<float*>(wsb + lay.col_off);
  const int rep = Hq / Hkv;

  if (dtype == PC_BF16) {
    PC_REQUIRE(D == kD, PC_ERR_UNSUPPORTED, "pc_score: bf16 tier needs D=128, got %d", D);
    const uintptr_t al = reinterpret_cast<uintptr_t>(Qs) | reinterpret_cast<uintptr_t>(K);
    PC_REQUIRE(al % 16 == 0 && q_stride_h % 8 == 0 && k_stride_h % 8 == 0, PC_ERR_SHAPE,
               "pc_score: bf16 tensors and head strides must be 16-byte aligned");
    const float c = scale * 1.4426950408889634f;
    // c == 1 (scale = ln 2): the caller folded the softmax scale and log2(e) into the queries, and
    // the column pass takes the affine step out of its loop (the row pass has no registers left
    // for the start values of its products and would gain nothing from rebuilding them per phase)
    const bool unit_c = c == 1.0f;
    const auto col_kernel = unit_c ? score_colpass_bf16<true> : score_colpass_bf16<false>;
    static std::atomic<uint64_t> row_ok{0}, col_ok[2];
    if (int rc = allow_dynamic_lds(reinterpret_cast<const void*>(score_rowpass_bf16), kRowSmem, row_ok, "pc_score"))
      return rc;
    if (int rc = allow_dynamic_lds(reinterpret_cast<const void*>(col_kernel), kColSmem, col_ok[unit_c], "pc_score"))
      return rc;
    const int n_pad = padded_rows(n_qs);
    if (lse == nullptr) {
      const int n_row_tiles = ceil_div(n_qs, kBlockRows);
      const int n_splits = choose_splits(n_row_tiles * Hq, ceil_div(Nk, kTileRows), kMaxSplits);
      score_rowpass_bf16<<<n_row_tiles * Hq * n_splits, kThreads, kRowSmem, s>>>(
          static_cast<const uint16_t*>(Qs), q_rows, static_cast<const uint16_t*>(K), ws_part, Hq, rep, n_qs, Nk,
          q_stride_h, k_stride_h, c, n_row_tiles, n_splits);
      PC_CHECK_LAUNCH("pc_score row pass");
      score_merge_rows<<<ceil_div(Hq * n_pad, 256), 256, 0, s>>>(ws_part, ws_lse, Hq, n_qs, n_pad, n_splits);
      PC_CHECK_LAUNCH("pc_score merge");
    } else {
      score_import_lse<<<ceil_div(Hq * n_pad, 256), 256, 0, s>>>(lse, lse_stride_h, q_rows, ws_lse, Hq, n_qs, n_pad,
                                                                 -1.4426950408889634f, -INFINITY);
      PC_CHECK_LAUNCH("pc_score lse import");
    }
    const int n_key_blocks = ceil_div(nkr, kBlockRows);
    const int n_qsplits = choose_splits(n_key_blocks * Hkv, rep * (n_pad / kTileRows), kMaxQSplits);
    const bool direct = n_qsplits == 1 && !share_heads;
    float* score_r = score + key_begin;
    col_kernel<<<n_key_blocks * Hkv * n_qsplits, kThreads, kColSmem, s>>>(
        static_cast<const uint16_t*>(Qs), q_rows, static_cast<const uint16_t*>(K) + static_cast<int64_t>(key_begin) * kD,
        ws_lse, direct ? score_r : ws_col, direct ? score_stride_h : nkr, static_cast<int64_t>(Hkv) * nkr, Hkv, rep,
        n_qs, nkr, q_stride_h, k_stride_h, c, n_key_blocks, n_qsplits);
    PC_CHECK_LAUNCH("pc_score column pass");
    if (!direct) {
      score_reduce<<<dim3(ceil_div(nkr, 256), share_heads ? 1 : Hkv), 256, 0, s>>>(ws_col, score_r, score_stride_h,
                                                                                   n_qsplits, Hkv, nkr, share_heads);
      PC_CHECK_LAUNCH("pc_score reduce");
    }
    return PC_OK;
  } else {
    PC_REQUIRE(D == 64 || D == 128, PC_ERR_UNSUPPORTED, "pc_score: fp32 tier needs D=64 or 128, got %d", D);
    float* per_head = share_heads ? ws_col : score + key_begin;
    const int64_t per_head_stride = share_heads ? nkr : score_stride_h;
    const float* q = static_cast<const float*>(Qs);
    const float* k = static_cast<const float*>(K);
    const float* k_r = k + static_cast<int64_t>(key_begin) * D;
    const float* lse_in = ws_lse;
    if (lse != nullptr) {
      score_import_lse<<<ceil_div(Hq * n_qs, 256), 256, 0, s>>>(lse, lse_stride_h, q_rows, ws_lse, Hq, n_qs, n_qs, 1.f,
                                                                INFINITY);
      PC_CHECK_LAUNCH("pc_score lse import");
    } else {
      const dim3 grid(ceil_div(n_qs, 64), Hq);
      if (D == 64)
        score_rowpass_f32<64><<<grid, 64, 0, s>>>(q, q_rows, k, ws_lse, rep, n_qs, Nk, q_stride_h, k_stride_h, scale);
      else
        score_rowpass_f32<128><<<grid, 64, 0, s>>>(q, q_rows, k, ws_lse, rep, n_qs, Nk, q_stride_h, k_stride_h, scale);
      PC_CHECK_LAUNCH("pc_score row pass");
    }
    const dim3 grid(ceil_div(nkr, 64), Hkv);
    if (D == 64)
      score_colpass_f32<64><<<grid, 64, 0, s>>>(q, q_rows, k_r, lse_in, per_head, per_head_stride, rep, n_qs, nkr,
                                                  q_stride_h, k_stride_h, scale);
    else
      score_colpass_f32<128><<<grid, 64, 0, s>>>(q, q_rows, k_r, lse_in, per_head, per_head_stride, rep, n_qs, nkr,
                                                   q_stride_h, k_stride_h, scale);
    PC_CHECK_LAUNCH("pc_score column pass");
    if (share_heads) {
      score_reduce<<<ceil_div(nkr, 256), 256, 0, s>>>(ws_col, score + key_begin, score_stride_h, 1, Hkv, nkr, 1);
      PC_CHECK_LAUNCH("pc_score head sum");
    }
  }
  return PC_OK;
}
