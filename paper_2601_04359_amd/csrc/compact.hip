// pc_compact: per-frame top-k selection and physical compaction (Sec. 3.4, Fig. 5(b)).
//
//   select   one work-group per (layer, selection head, segment).  The scores of a past-frame
//            segment sit in registers as order-preserving integers; the k-th largest is found
//            eight bits at a time with an LDS histogram (the bits all keys share are skipped,
//            and the search stops as soon as the k-th key is alone in its bin); equal scores
//            are taken lowest index first; the kept indices come out ascending.  Segments
//            longer than PC_MAX_SELECT_LEN take a one-wave, bit-by-bit variant that re-reads
//            the scores.  A call with many segments (a stack of layers) uses one WAVE per
//            segment instead: fewer instructions per key and no work-group barriers
//            (5,488 segments: 56 us -> 34 us; one layer's 196 segments: 10 us -> 15 us, hence
//            the switch-over at 1,536 segments).
//   gather   HBM-bound.  A work-group owns 128 consecutive packed rows of one
//            KV head: it loads its K, V and position rows (16 bytes per lane), then stores
//            them.  In place, a work-group may only store once every work-group whose SOURCE
//            rows lie in its destination range has finished loading.  Work-groups take their
//            chunk from an atomic ticket per (layer, head), so a chunk only ever waits on
//            chunks with a lower ticket, which are already running and whose loads wait on
//            nothing.
//   A stack of layers is handled by the same two launches (layer strides).
#include <limits.h>
#include <stddef.h>

#include <algorithm>

#include "common.h"

namespace pc {
namespace {

// Packed rows per gather work-group and its size: a thread moves two 16-byte pieces of K and two
// of V.  Measured on 28 layer caches at frame 48 (gamma 0.85): 4 pieces per thread (64 rows, 256
// threads) 931 us, 2 pieces (32 rows, 256 threads) 838 us, (64 rows, 512 threads) 812 us,
// (128 rows, 1,024 threads) 807 us, 1 piece (32 rows, 512 threads) 931 us.  One layer per call
// gains most from the largest shape (40.8 against 42.4 us per layer at gamma 0.7).
constexpr int kGatherRows = 128;
constexpr int kGatherThreads = 1024;
constexpr int kSpinLimit = 1 << 22;

struct SegTable {
  int32_t n;
  int32_t start[PC_MAX_SEGMENTS];  // first source row
  int32_t len[PC_MAX_SEGMENTS];    // source rows
  int32_t keep[PC_MAX_SEGMENTS];   // rows kept
  int32_t dst[PC_MAX_SEGMENTS];    // first packed row
  uint8_t prune[PC_MAX_SEGMENTS];  // 1: past frame with keep < len (needs the select)
};

// fp32 -> uint32 such that integer order = float order; -0 is folded onto +0 first.
__device__ __forceinline__ uint32_t order_key(float f) {
  const uint32_t u = __float_as_uint(f + 0.0f);
  return u ^ (static_cast<uint32_t>(static_cast<int32_t>(u) >> 31) | 0x80000000u);
}

__device__ __forceinline__ int popc64(uint64_t v) { return __popcll(v); }

// Inclusive scan over the 64 lanes (lane l gets op over lanes 0..l) with data-parallel-primitive
// moves: shifts by 1, 2, 4, 8 inside each row of 16 lanes, then lane 15 of a row into the row
// after it and lane 31 into the upper half.  Each step is one vector instruction; a shuffle
// through the LDS crossbar costs a round trip of a hundred cycles per step.
template <class Op>
__device__ __forceinline__ int wave_scan(int x, int identity, Op op) {
  x = op(x, __builtin_amdgcn_update_dpp(identity, x, 0x111, 0xf, 0xf, false));  // row_shr:1
  x = op(x, __builtin_amdgcn_update_dpp(identity, x, 0x112, 0xf, 0xf, false));  // row_shr:2
  x = op(x, __builtin_amdgcn_update_dpp(identity, x, 0x114, 0xf, 0xf, false));  // row_shr:4
  x = op(x, __builtin_amdgcn_update_dpp(identity, x, 0x118, 0xf, 0xf, false));  // row_shr:8
  x = op(x, __builtin_amdgcn_update_dpp(identity, x, 0x142, 0xa, 0xf, false));  // row_bcast:15 -> rows 1, 3
  x = op(x, __builtin_amdgcn_update_dpp(identity, x, 0x143, 0xc, 0xf, false));  // row_bcast:31 -> rows 2, 3
  return x;
}
__device__ __forceinline__ int wave_prefix_sum(int x) {  // sum over lanes 0..l
  return wave_scan(x, 0, [](int a, int b) { return a + b; });
}
__device__ __forceinline__ uint32_t wave_or(uint32_t x) {  // OR over the wave, in every lane
  const int r = wave_scan(static_cast<int>(x), 0, [](int a, int b) { return a | b; });
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(r, 63));
}
__device__ __forceinline__ uint32_t wave_and(uint32_t x) {
  const int r = wave_scan(static_cast<int>(x), -1, [](int a, int b) { return a & b; });
  return static_cast<uint32_t>(__builtin_amdgcn_readlane(r, 63));
}

// One wave selects the top `k` of `len` scores.  Keys are register resident when
// kItems > 0 (len <= 64 * kItems); kItems == 0 re-reads the scores on every pass.
template <int kItems>
__device__ void select_wave(const float* __restrict__ sc, int len, int k, int32_t* __restrict__ out,
                            int start) {
  const int lane = threadIdx.x;
  const uint64_t lt_mask = (1ull << lane) - 1ull;
  constexpr int kRegs = kItems > 0 ? kItems : 1;
  uint32_t key[kRegs];
  const int n_iter = kItems > 0 ? kItems : (len + 63) / 64;
  if constexpr (kItems > 0) {
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
      const int e = i * 64 + lane;
      key[i] = e < len ? order_key(sc[e]) : 0u;  // 0 is below every real key
    }
  }
  auto key_at = [&](int i) -> uint32_t {
    if constexpr (kItems > 0) {
      return key[i];
    } else {
      const int e = i * 64 + lane;
      return e < len ? order_key(sc[e]) : 0u;
    }
  };
  // k-th largest key, most significant bit first
  uint32_t prefix = 0;
  int remaining = k;
  for (int bit = 31; bit >= 0; --bit) {
    const uint32_t cand = prefix | (1u << bit);
    int cnt = 0;
    if constexpr (kItems > 0) {
#pragma unroll
      for (int i = 0; i < kItems; ++i) cnt += popc64(__ballot(((key[i] ^ cand) >> bit) == 0u));
    } else {
      for (int i = 0; i < n_iter; ++i) cnt += popc64(__ballot(((key_at(i) ^ cand) >> bit) == 0u));
    }
    if (cnt >= remaining)
      prefix = cand;
    else
      remaining -= cnt;
  }
  // everything above the threshold, then the first `remaining` keys equal to it
  int out_run = 0, eq_run = 0;
  auto emit = [&](int i, uint32_t kv) {
    const int e = i * 64 + lane;
    const bool valid = e < len;
    const bool eq = valid && kv == prefix;
    const uint64_t beq = __ballot(eq);
    const bool keep = valid && (kv > prefix || (eq && eq_run + popc64(beq & lt_mask) < remaining));
    const uint64_t bk = __ballot(keep);
    const int at = out_run + popc64(bk & lt_mask);
    if (keep && at < k) out[at] = start + e;
    out_run += popc64(bk);
    eq_run += popc64(beq);
  };
  if constexpr (kItems > 0) {
#pragma unroll
    for (int i = 0; i < kItems; ++i)
      if (i * 64 < len) emit(i, key[i]);
  } else {
    for (int i = 0; i < n_iter; ++i) emit(i, key_at(i));
  }
}

template <int kItems>
__global__ __launch_bounds__(64) void select_kernel(const float* __restrict__ score,
                                                    int64_t score_stride_h, int32_t* __restrict__ idx,
                                                    int64_t idx_stride_h, SegTable tab, int hsel,
                                                    int64_t score_stride_l, int64_t idx_stride_l) {
  const int s = blockIdx.x, h = blockIdx.y;  // h runs over layers x selection heads
  const int64_t sc_off = (h / hsel) * score_stride_l + (h % hsel) * score_stride_h;
  const int start = tab.start[s], len = tab.len[s], keep = tab.keep[s];
  int32_t* out = idx + (h / hsel) * idx_stride_l + (h % hsel) * idx_stride_h + tab.dst[s];
  if (keep <= 0) return;
  if (!tab.prune[s]) {  // anchors, current frame, or a frame within budget: keep every row
    for (int e = threadIdx.x; e < len; e += 64) out[e] = start + e;
    return;
  }
  select_wave<kItems>(score + sc_off + start, len, keep, out, start);
}

// One work-group of 256 threads per segment; thread t keeps the kItems CONSECUTIVE keys
// [t kItems, (t+1) kItems) of the segment in registers as order-preserving integers.
//   * The bits all keys share (sign, most of the exponent) are found with one AND / OR reduction
//     and skipped.
//   * The k-th largest key is then found eleven bits at a time: keys that still match the prefix
//     vote into a 2,048-bin LDS histogram; a thread owns eight neighbouring bins, the 256 threads
//     take a suffix sum over their totals (wave scan + one exchange) and the thread whose bins
//     contain the k-th key walks its eight.  With 4,032 keys over 2,048 bins the chosen bin
//     nearly always holds a handful of keys: up to 64 are put into LDS and ranked against each
//     other by every wave (no second pass over the histogram); more than 64 take another pass.
//   * Output in ascending index order: with consecutive keys per thread a kept key's position is
//     (kept keys of lower threads) + (kept keys earlier in this thread), so one more scan over
//     the threads (keys above the threshold and keys equal to it, packed in one word) places
//     everything; equal keys are taken lowest index first.
// The kernel is bound by its instruction count once a stack of layers fills the chip with these
// work-groups, hence few, wide passes and no per-key cross-lane work.
// Blocks also clear the in-place gather's ticket counters and flags (n_clear words).
template <int kItems>
__global__ __launch_bounds__(256) void select_block_kernel(const float* __restrict__ score,
                                                           int64_t score_stride_h,
                                                           int32_t* __restrict__ idx, int64_t idx_stride_h,
                                                           SegTable tab, int32_t* __restrict__ clear,
                                                           int n_clear, int hsel, int64_t score_stride_l,
                                                           int64_t idx_stride_l) {
  constexpr int kBits = 11, kBins = 1 << kBits, kOwn = kBins / 256;  // bins per thread
  static_assert(kOwn == 8, "a thread reads its bins with two 16-byte loads");
  __shared__ __align__(16) int s_hist[kBins];
  __shared__ int s_wave_sum[4];
  __shared__ int s_pick[3];  // chosen digit, keys above it, keys in it
  __shared__ uint32_t s_and[4], s_or[4];
  __shared__ uint32_t s_cand[64];  // the keys of the chosen bin when they are few
  __shared__ int s_n_cand;
  const int s = blockIdx.x, h = blockIdx.y;
  {
    const int nb = gridDim.x * gridDim.y, b = h * gridDim.x + s;
    for (int i = b * 256 + threadIdx.x; i < n_clear; i += nb * 256) clear[i] = 0;
  }
  const int start = tab.start[s], len = tab.len[s], k = tab.keep[s];
  int32_t* out = idx + (h / hsel) * idx_stride_l + (h % hsel) * idx_stride_h + tab.dst[s];
  if (k <= 0) return;  // block-uniform
  if (!tab.prune[s]) {
    for (int e = threadIdx.x; e < len; e += 256) out[e] = start + e;
    return;
  }
  const float* sc = score + (h / hsel) * score_stride_l + (h % hsel) * score_stride_h + start;
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  const int e0 = t * kItems;
  uint32_t key[kItems];
  if constexpr (kItems % 4 == 0) {
    const bool aligned = (reinterpret_cast<uintptr_t>(sc) & 15) == 0;  // block-uniform
#pragma unroll
    for (int q = 0; q < kItems / 4; ++q) {
      const int e = e0 + q * 4;
      float v[4] = {0.f, 0.f, 0.f, 0.f};
      if (aligned && e + 3 < len) {
        const f32x4 x = *reinterpret_cast<const f32x4*>(sc + e);
#pragma unroll
        for (int j = 0; j < 4; ++j) v[j] = x[j];
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j)
          if (e + j < len) v[j] = sc[e + j];
      }
#pragma unroll
      for (int j = 0; j < 4; ++j) key[q * 4 + j] = e + j < len ? order_key(v[j]) : 0u;  // 0 is below every real key
    }
  } else {
#pragma unroll
    for (int i = 0; i < kItems; ++i) key[i] = e0 + i < len ? order_key(sc[e0 + i]) : 0u;
  }
  // Bits shared by every key of the segment are settled at once: only the bits from the highest
  // differing one down go through the histogram.
  uint32_t k_and = 0xFFFFFFFFu, k_or = 0u;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    if (e0 + i < len) {
      k_and &= key[i];
      k_or |= key[i];
    }
  }
  k_and = wave_and(k_and);
  k_or = wave_or(k_or);
  if (lane == 0) {
    s_and[wave] = k_and;
    s_or[wave] = k_or;
  }
  int4* h4 = reinterpret_cast<int4*>(s_hist);
  h4[2 * t] = make_int4(0, 0, 0, 0);  // this thread's own eight bins, cleared for the first pass
  h4[2 * t + 1] = make_int4(0, 0, 0, 0);
  if (t == 0) s_n_cand = 0;
  __syncthreads();
  k_and = s_and[0] & s_and[1] & s_and[2] & s_and[3];
  k_or = s_or[0] | s_or[1] | s_or[2] | s_or[3];
  const uint32_t differ = k_and ^ k_or;
  int hi = differ ? 32 - __clz(differ) : 0;  // number of undecided low bits
  uint32_t prefix = hi >= 32 ? 0u : (k_or >> hi) << hi;
  int remaining = k;
  bool cleared = true;
  while (hi > 0) {
    const int width = min(kBits, hi), shift = hi - width;
    if (!cleared) {  // a further pass (rare): the bins are cleared behind the reads of the pass before
      h4[2 * t] = make_int4(0, 0, 0, 0);
      h4[2 * t + 1] = make_int4(0, 0, 0, 0);
      __syncthreads();
    }
    cleared = false;
    const uint32_t hi_mask = hi >= 32 ? 0u : 0xFFFFFFFFu << hi;
    const uint32_t digit_mask = (1u << width) - 1u;
#pragma unroll
    for (int i = 0; i < kItems; ++i)
      if (e0 + i < len && (key[i] & hi_mask) == (prefix & hi_mask))
        atomicAdd(&s_hist[(key[i] >> shift) & digit_mask], 1);
    __syncthreads();
    const int4 lo4 = h4[2 * t], hi4 = h4[2 * t + 1];
    const int c[kOwn] = {lo4.x, lo4.y, lo4.z, lo4.w, hi4.x, hi4.y, hi4.z, hi4.w};
    int mine = 0;  // votes for bins 8 t .. 8 t + 7
#pragma unroll
    for (int j = 0; j < kOwn; ++j) mine += c[j];
    // suffix sums over the threads: above = matching keys with a digit beyond this thread's bins
    const int upto = wave_prefix_sum(mine);
    const int incl = __builtin_amdgcn_readlane(upto, 63) - upto + mine;  // this lane and the lanes above it
    if (lane == 0) s_wave_sum[wave] = incl;
    __syncthreads();
    int above = incl - mine;
    for (int w = wave + 1; w < 4; ++w) above += s_wave_sum[w];
    if (above < remaining && remaining <= above + mine) {  // exactly one thread: walk its bins downwards
      int ab = above, digit = 0, cnt = 0;
      bool found = false;
#pragma unroll
      for (int j = kOwn - 1; j >= 0; --j) {
        if (!found && remaining <= ab + c[j]) {
          found = true;
          digit = t * kOwn + j;
          cnt = c[j];
          s_pick[1] = ab;
        }
        if (!found) ab += c[j];
      }
      s_pick[0] = digit;
      s_pick[2] = cnt;
    }
    __syncthreads();
    prefix |= static_cast<uint32_t>(s_pick[0]) << shift;
    remaining -= s_pick[1];
    hi = shift;
    if (hi > 0 && s_pick[2] <= 64) {
      // block-uniform: the chosen bin holds few keys (with 4,032 keys over 2,048 bins nearly always).
      // They go to LDS, and every wave ranks them for itself: lane j counts the candidates above and
      // not below its own; the lane whose counts bracket the remaining rank holds the threshold.
      const uint32_t lo_mask = 0xFFFFFFFFu << hi;
#pragma unroll
      for (int i = 0; i < kItems; ++i)
        if (e0 + i < len && (key[i] & lo_mask) == prefix) {
          const int at = atomicAdd(&s_n_cand, 1);
          if (at < 64) s_cand[at] = key[i];
        }
      __syncthreads();
      const int n_cand = min(s_n_cand, 64);
      const bool has = lane < n_cand;
      const uint32_t my = has ? s_cand[lane] : 0u;
      int gt = 0, ge = 0;
      for (int j = 0; j < n_cand; ++j) {
        const uint32_t x = __builtin_amdgcn_readlane(my, j);
        gt += x > my ? 1 : 0;
        ge += x >= my ? 1 : 0;
      }
      const uint64_t thr_mask = __ballot(has && gt < remaining && remaining <= ge);
      const int thr_lane = thr_mask ? __builtin_ctzll(thr_mask) : 0;
      prefix = __builtin_amdgcn_readlane(my, thr_lane);
      remaining -= __builtin_amdgcn_readlane(gt, thr_lane);  // of the keys equal to the threshold, this many are taken
      hi = 0;
    }
  }
  // keys above the threshold (low half-word) and equal to it (high half-word) in this thread
  int mine = 0;
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const bool valid = e0 + i < len;
    mine += (valid && key[i] > prefix ? 1 : 0) + (valid && key[i] == prefix ? 1 << 16 : 0);
  }
  const int incl = wave_prefix_sum(mine);  // this lane and the lanes below it
  __syncthreads();  // s_wave_sum is free again
  if (lane == 63) s_wave_sum[wave] = incl;
  __syncthreads();
  int before = incl - mine;
  for (int w = 0; w < wave; ++w) before += s_wave_sum[w];
  const int gt_before = before & 0xFFFF;
  int eq_run = before >> 16;                       // threshold keys at lower indices
  int at = gt_before + min(eq_run, remaining);     // kept keys at lower indices
#pragma unroll
  for (int i = 0; i < kItems; ++i) {
    const bool valid = e0 + i < len;
    const bool is_eq = valid && key[i] == prefix;
    const bool kept = valid && (key[i] > prefix || (is_eq && eq_run < remaining));
    if (kept && at < k) out[at] = start + e0 + i;
    at += kept ? 1 : 0;
    eq_run += is_eq ? 1 : 0;
  }
}

// One WAVE per segment (a work-group is one wave), no work-group barrier anywhere: the form for
// a stack of layers, where thousands of segments fill the chip and the cost is instructions per
// key, not the latency of one segment.  Lane l keeps keys l, l + 64, l + 128, ... in registers: the
// n_full = len / 64 rows of 64 keys in key[], the ragged last row (len % 64 keys) in a register of
// its own.  A sweep over the keys runs from row n_full - 1 down to row 0 behind one scalar
// compare per row, so a full row costs no per-lane validity test.
//   * Shared leading bits are skipped as in the block form; then ONE 2,048-bin histogram pass
//     over the next eleven bits (the wave's own 8 KB of LDS; every key votes, no test).  A lane
//     sums the 32 bins it owns, a suffix scan over the lanes finds the owner of the k-th key and
//     32 lanes scan its bins.
//   * The chosen bin nearly always holds a handful of keys: up to 64 candidates are written to
//     LDS (ballot + lane count, no atomics), one per lane, and each lane counts the candidates
//     above / not below its own by reading the others lane by lane; the lane whose counts bracket
//     the remaining rank holds the threshold.  More than 64 candidates: another histogram pass.
//   * Output: exactly k keys are kept, so with the rows taken last to first a kept key's position
//     is k - (kept in later rows) - (kept in this row at its lane or above), a ballot and a lane
//     count; stores of a row land next to each other.  Equal keys are taken lowest index first.
#ifndef PC_ROWS_SELECT_MIN_UNITS
#define PC_ROWS_SELECT_MIN_UNITS 1536
#endif
#ifndef PC_ROWS_SELECT_MIN_LEN
#define PC_ROWS_SELECT_MIN_LEN 1024
#endif
// the wave form is used from this many segments per call on (measured cross-over: 7-8 layers of 196
// segments), when the longest pruned segment is longer than kRowsSelectMinLen
constexpr int kRowsSelectMinUnits = PC_ROWS_SELECT_MIN_UNITS, kRowsSelectMinLen = PC_ROWS_SELECT_MIN_LEN;
// f(n - 1), ..., f(0) with compile-time row numbers; n in [0, 64] is wave-uniform
template <class F>
__device__ __forceinline__ void rows_down_from(int n, F&& f) {
#pragma unroll
  for (int i = 63; i >= 0; --i) {
    asm volatile("" : "+s"(n));  // one scalar compare here, not 64 lane masks kept from sweep to sweep
    if (i < n) f(i);
  }
}

__device__ __forceinline__ int lanes_below(uint64_t mask, int base) {  // base + set bits of mask below this lane
  return __builtin_amdgcn_mbcnt_hi(static_cast<uint32_t>(mask >> 32),
                                   __builtin_amdgcn_mbcnt_lo(static_cast<uint32_t>(mask), base));
}

__global__ __launch_bounds__(64) void select_rows_kernel(
    const float* __restrict__ score, int64_t score_stride_h, int32_t* __restrict__ idx, int64_t idx_stride_h,
    SegTable tab, int32_t* __restrict__ clear, int n_clear, int hsel, int64_t score_stride_l, int64_t idx_stride_l) {
  constexpr int kRows = PC_MAX_SELECT_LEN / 64;                     // 64 full rows at most
  constexpr int kBits = 11, kBins = 1 << kBits, kOwn = kBins / 64;  // 32 bins per lane
  static_assert(kRows == 64, "rows_down_from covers 64 rows");
  __shared__ __align__(16) int hist[kBins];
  const int lane = threadIdx.x;
  const int s = blockIdx.x, h = blockIdx.y;  // wave-uniform, like everything read from the table
  for (int i = (h * gridDim.x + s) * 64 + lane; i < n_clear; i += gridDim.x * gridDim.y * 64) clear[i] = 0;
  const int layer = __builtin_amdgcn_readfirstlane(h / hsel), head = __builtin_amdgcn_readfirstlane(h % hsel);
  const int start = tab.start[s], len = tab.len[s], k = tab.keep[s];
  int32_t* out = idx + layer * idx_stride_l + head * idx_stride_h + tab.dst[s];
  if (k <= 0) return;
  if (!tab.prune[s]) {
    for (int e = lane; e < len; e += 64) out[e] = start + e;
    return;
  }
  const float* sc = score + layer * score_stride_l + head * score_stride_h + start;
  uint32_t* cand = reinterpret_cast<uint32_t*>(hist);  // the candidates reuse the histogram's first words
  auto wave_sync = [] {  // LDS written by other lanes of this wave becomes visible; nothing moves across
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
  };
  const int n_full = len >> 6, tail = len & 63;
  const bool in_tail = lane < tail;  // this lane has a key in the ragged row
  uint32_t key[kRows], key_r;
  {  // every load in flight before the first use; rows past n_full are neither loaded nor looked at
    float v[kRows];
    const float v_r = sc[min(n_full * 64 + lane, len - 1)];
    // a buffer descriptor that spans exactly the segment's scores (raw 32-bit data): the row offset
    // is a scalar operand of the load and the lane's byte offset one register for all rows, so a
    // load costs no vector address arithmetic; only rows that lie inside the segment are loaded
    const __amdgpu_buffer_rsrc_t rsrc =
        __builtin_amdgcn_make_buffer_rsrc(const_cast<float*>(sc), 0, len * 4, 0x00020000);
    const int lane_bytes = lane * 4;
    rows_down_from(n_full, [&](int i) {
      v[i] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rsrc, lane_bytes, i * 256, 0));
    });
    rows_down_from(n_full, [&](int i) {
      asm volatile("" : "+v"(v[i]));  // the conversion stays in this sweep, behind all the loads
      key[i] = order_key(v[i]);
    });
    key_r = order_key(v_r);
  }
  // bits in which any two keys differ: every key against the segment's first one (one three-input
  // bit operation per key), then an OR over the lanes
  const uint32_t key0 = __builtin_amdgcn_readfirstlane(n_full > 0 ? key[0] : key_r);
  uint32_t differ = in_tail ? key_r ^ key0 : 0u;
  rows_down_from(n_full, [&](int i) { differ |= key[i] ^ key0; });
  differ = wave_or(differ);  // the same in every lane: scalar from here on
  int hi = differ ? 32 - __clz(differ) : 0;  // number of undecided low bits
  uint32_t prefix = hi >= 32 ? 0u : (key0 >> hi) << hi;
  int remaining = k;   // rank of the threshold among the keys that match the prefix
  int eq_total = len;  // keys equal to the threshold once hi == 0
  bool first = true;
  while (hi > 0) {
    const int width = min(kBits, hi), shift = hi - width;
    int4* h4 = reinterpret_cast<int4*>(hist);
#pragma unroll
    for (int j = 0; j < kOwn / 4; ++j) h4[j * 64 + lane] = make_int4(0, 0, 0, 0);
    wave_sync();
    // byte offset of a key's bin: the digit times four, as one shift and one mask
    const uint32_t byte_mask = ((1u << width) - 1u) << 2;
    const uint32_t rot = static_cast<uint32_t>(shift - 2) & 31u;  // rotate right: bit `shift` lands on bit 2
    auto vote = [&](uint32_t kv) {
      const uint32_t off = __builtin_amdgcn_alignbit(kv, kv, rot) & byte_mask;
      atomicAdd(reinterpret_cast<int*>(reinterpret_cast<char*>(hist) + off), 1);
    };
    if (first) {  // every key matches the shared prefix
      if (in_tail) vote(key_r);
      rows_down_from(n_full, [&](int i) { vote(key[i]); });
    } else {
      const uint32_t hi_mask = 0xFFFFFFFFu << hi;  // hi < 32 after the first pass
      if (in_tail && (key_r & hi_mask) == prefix) vote(key_r);
      rows_down_from(n_full, [&](int i) {
        if ((key[i] & hi_mask) == prefix) vote(key[i]);
      });
    }
    first = false;
    wave_sync();
    // lane l owns bins 32 l .. 32 l + 31; the eight 16-byte reads are rotated by the lane so that
    // neighbouring lanes use different LDS banks
    int mine = 0;
#pragma unroll
    for (int j = 0; j < kOwn / 4; ++j) {
      const int4 c = h4[lane * (kOwn / 4) + ((j + lane) & (kOwn / 4 - 1))];
      mine += (c.x + c.y) + (c.z + c.w);
    }
    const int upto = wave_prefix_sum(mine);
    const int above = __builtin_amdgcn_readlane(upto, 63) - upto;  // votes in the bins of the lanes above
    const uint64_t owner_mask = __ballot(above < remaining && remaining <= above + mine);  // exactly one lane
    const int owner = owner_mask ? __builtin_ctzll(owner_mask) : 0;
    const int above_owner = __builtin_amdgcn_readlane(above, owner);
    // the owner's 32 bins, one per lane of the lower half wave; suffix sums again
    const int c_bin = lane < kOwn ? hist[owner * kOwn + lane] : 0;
    const int upto_b = wave_prefix_sum(c_bin);
    const int above_b = above_owner + __builtin_amdgcn_readlane(upto_b, kOwn - 1) - upto_b;  // matching keys with a larger digit
    const uint64_t bin_mask = __ballot(lane < kOwn && above_b < remaining && remaining <= above_b + c_bin);
    const int bin_lane = bin_mask ? __builtin_ctzll(bin_mask) : 0;
    const int cnt = __builtin_amdgcn_readlane(c_bin, bin_lane);
    remaining -= __builtin_amdgcn_readlane(above_b, bin_lane);
    prefix |= static_cast<uint32_t>(owner * kOwn + bin_lane) << shift;
    hi = shift;
    eq_total = cnt;
    if (hi > 0 && cnt <= 64) {
      // the candidates (keys that match the prefix so far), one per lane
      const uint32_t lo_mask = 0xFFFFFFFFu << hi;
      int n_cand = 0;
      wave_sync();  // the histogram has been read
      auto collect = [&](uint32_t kv, bool m) {
        const uint64_t bm = __ballot(m);
        if (bm != 0) {  // wave-uniform
          const int at = lanes_below(bm, n_cand);
          if (m && at < 64) cand[at] = kv;
          n_cand += popc64(bm);
        }
      };
      collect(key_r, in_tail && (key_r & lo_mask) == prefix);
      rows_down_from(n_full, [&](int i) { collect(key[i], (key[i] & lo_mask) == prefix); });
      wave_sync();
      n_cand = min(n_cand, 64);
      const bool has = lane < n_cand;
      const uint32_t my = has ? cand[lane] : 0u;
      int gt = 0, ge = 0;
      for (int c = 0; c < n_cand; ++c) {
        const uint32_t x = __builtin_amdgcn_readlane(my, c);
        gt += x > my ? 1 : 0;
        ge += x >= my ? 1 : 0;
      }
      const uint64_t thr_mask = __ballot(has && gt < remaining && remaining <= ge);  // the lanes holding the threshold
      const int thr_lane = thr_mask ? __builtin_ctzll(thr_mask) : 0;
      prefix = __builtin_amdgcn_readlane(my, thr_lane);
      const int gt_t = __builtin_amdgcn_readlane(gt, thr_lane), ge_t = __builtin_amdgcn_readlane(ge, thr_lane);
      remaining -= gt_t;
      eq_total = ge_t - gt_t;
      hi = 0;
    }
  }
  // `remaining` of the eq_total keys equal to the threshold are taken, lowest index first; rows
  // are written last to first, `after` counting the kept keys of the rows already written
  const int lane_start = start + lane;
  int after = 0;
  if (eq_total == remaining) {  // all of them: one compare per key
    auto put = [&](bool keep, int row) {
      const uint64_t bk = __ballot(keep);
      after += popc64(bk);
      const int at = lanes_below(bk, k - after);
      if (keep && static_cast<uint32_t>(at) < static_cast<uint32_t>(k))
        *reinterpret_cast<int32_t*>(reinterpret_cast<char*>(out) + static_cast<uint32_t>(at) * 4u) = lane_start + row * 64;
    };
    put(in_tail && key_r >= prefix, n_full);
    rows_down_from(n_full, [&](int i) { put(key[i] >= prefix, i); });
  } else {
    int eq_after = 0;
    auto put = [&](uint32_t kv, bool valid, int row) {
      const bool eq = valid && kv == prefix;
      const uint64_t beq = __ballot(eq);
      eq_after += popc64(beq);
      const int eq_at = lanes_below(beq, eq_total - eq_after);  // equal keys at lower indices
      const bool keep = valid && (kv > prefix || (eq && eq_at < remaining));
      const uint64_t bk = __ballot(keep);
      after += popc64(bk);
      const int at = lanes_below(bk, k - after);
      if (keep && static_cast<uint32_t>(at) < static_cast<uint32_t>(k))
        *reinterpret_cast<int32_t*>(reinterpret_cast<char*>(out) + static_cast<uint32_t>(at) * 4u) = lane_start + row * 64;
    };
    put(key_r, in_tail, n_full);
    rows_down_from(n_full, [&](int i) { put(key[i], true, i); });
  }
}

// ---- gather ----------------------------------------------------------------------------------
constexpr int kMaxTicketHeads = 256;  // layers x KV heads of one call
struct GatherSync {  // one ticket counter per (layer, KV head), each on its own 128-byte line
  int32_t abort;
  int32_t pad[31];
  int32_t ticket[kMaxTicketHeads][32];
};

__global__ void clear_words(int32_t* p, int n) {
  const int i = blockIdx.x * blockDim.x + threadIdx.x;
  if (i < n) p[i] = 0;
}

template <int cpr /* 16-byte chunks per row */, int kRows /* packed rows per work-group */, bool kInPlace>
__global__ __launch_bounds__(kGatherThreads) void gather_kernel(
    const u32x4* __restrict__ K, const u32x4* __restrict__ V, const int32_t* __restrict__ pos,
    u32x4* __restrict__ Ko, u32x4* __restrict__ Vo, int32_t* __restrict__ pos_o,
    const int32_t* __restrict__ idx, int64_t idx_stride_h, int share_heads, int Hkv, int Nk_in, int Nk_out,
    int64_t in_stride_c, int64_t out_stride_c,
    int64_t pos_stride_h, int64_t pos_out_stride_h, GatherSync* sync, int32_t* flags,
    int chunks_per_head, SegTable tab, int n_layers, int64_t in_stride_lc, int64_t out_stride_lc,
    int64_t pos_stride_l, int64_t pos_out_stride_l, int64_t idx_stride_l) {
  __shared__ int s_ticket;
  // launch order: layer by layer, the KV heads of a layer side by side (a few long sequential
  // streams at a time suit the memory better than one stream per (layer, head) all at once)
  const int per_layer = gridDim.x / n_layers;
  const int l = blockIdx.x / per_layer, in_layer = blockIdx.x % per_layer;
  const int h = in_layer % Hkv;
  const int vh = l * Hkv + h;            // (layer, KV head) pair
  int cc = in_layer / Hkv;
  if constexpr (kInPlace) {  // chunks of a head are taken in ticket order, not in launch order
    if (threadIdx.x == 0) s_ticket = atomicAdd(&sync->ticket[vh][0], 1);
    __syncthreads();
    cc = s_ticket;
    // A ticket outside the launch's chunks means the counters were not cleared by the SELECT half
    // of this call (GATHER alone, or on another workspace): flag it and move nothing rather than
    // index the flags with it.  Block-uniform, and before any other barrier.
    if (cc < 0 || cc >= per_layer / Hkv) {
      if (threadIdx.x == 0) __hip_atomic_store(&sync->abort, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      return;
    }
  }
  const int hs = share_heads ? 0 : h;
  const int r0 = cc * kRows;
  const int r1 = min(r0 + kRows, Nk_out);
  const int32_t* idx_h = idx + l * idx_stride_l + hs * idx_stride_h;
  const int64_t in_base = l * in_stride_lc + h * in_stride_c, out_base = l * out_stride_lc + h * out_stride_c;
  const int64_t pos_in_base = l * pos_stride_l + hs * pos_stride_h;
  const int64_t pos_out_base = l * pos_out_stride_l + hs * pos_out_stride_h;

  // ---- load: a thread moves one 16-byte chunk of a K row and the same chunk of its V row ----
  constexpr int kRowsPerPass = kGatherThreads / cpr;
  constexpr int kPasses = kRows / kRowsPerPass;
  const int ch = threadIdx.x % cpr, rp = threadIdx.x / cpr;
  u32x4 kval[kPasses], vval[kPasses];
  int64_t dst_off[kPasses];
#pragma unroll
  for (int it = 0; it < kPasses; ++it) {
    const int row = r0 + it * kRowsPerPass + rp;
    dst_off[it] = -1;
    if (row < r1) {
      const int src = min(max(idx_h[row], 0), Nk_in - 1);  // a valid table never needs the clamp
      if (!kInPlace || src != row) {
        const int64_t so = in_base + static_cast<int64_t>(src) * cpr + ch;
        kval[it] = __builtin_nontemporal_load(&K[so]);
        vval[it] = __builtin_nontemporal_load(&V[so]);
        dst_off[it] = out_base + static_cast<int64_t>(row) * cpr + ch;
      }
    }
  }
  int32_t pval = 0;
  int64_t pdst = -1;
  static_assert(kRows * 3 <= kGatherThreads, "one thread per position component");
  if ((share_heads ? h == 0 : true) && static_cast<int>(threadIdx.x) < (r1 - r0) * 3) {
    const int row = r0 + threadIdx.x / 3, comp = threadIdx.x % 3;
    const int src = min(max(idx_h[row], 0), Nk_in - 1);
    if (!kInPlace || src != row) {
      pval = pos[pos_in_base + static_cast<int64_t>(src) * 3 + comp];
      pdst = pos_out_base + static_cast<int64_t>(row) * 3 + comp;
    }
  }

  if constexpr (kInPlace) {
    // Publish "my sources are in registers", then wait for every lower chunk of this head
    // whose sources may lie in [r0, r1).  Only the ORDER of my stores after their loads
    // matters (nobody reads what another work-group wrote), so no cache maintenance is
    // needed: each thread pins its loaded registers (which makes the compiler wait for the
    // loads), the work-group barrier collects all threads, and relaxed device-scope
    // accesses carry the flag.
#pragma unroll
    for (int it = 0; it < kPasses; ++it) asm volatile("" : "+v"(kval[it]), "+v"(vval[it]));
    asm volatile("" : "+v"(pval));
    __syncthreads();
    int32_t* flags_h = flags + static_cast<int64_t>(vh) * chunks_per_head;
    if (threadIdx.x == 0)
      __hip_atomic_store(&flags_h[cc], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    // Source row of the i-th kept row of a segment: start + i <= src <= start + (len - keep) + i.
    int row_lo = INT_MAX, row_hi = -1;
    int first = 0;  // first segment that ends behind r0 (segments are in row order): binary search
    for (int lo = 0, hi = tab.n; lo < hi;) {
      const int mid = (lo + hi) >> 1;
      if (tab.start[mid] + tab.len[mid] <= r0) {
        lo = mid + 1;
        first = lo;
      } else {
        hi = mid;
        first = lo;
      }
    }
    for (int s = first; s < tab.n && tab.start[s] < r1; ++s) {
      if (tab.keep[s] <= 0) continue;
      const int a = tab.start[s];
      const int slack = tab.len[s] - tab.keep[s];
      const int i_lo = max(0, r0 - a - slack), i_hi = min(tab.keep[s] - 1, r1 - 1 - a);
      if (i_lo <= i_hi) {
        row_lo = min(row_lo, tab.dst[s] + i_lo);
        row_hi = max(row_hi, tab.dst[s] + i_hi);
      }
    }
    if (row_hi >= 0) {
      const int c_lo = row_lo / kRows, c_hi = min(row_hi / kRows, cc - 1);
      for (int c = c_lo + threadIdx.x; c <= c_hi; c += kGatherThreads) {
        int spins = 0;
        while (__hip_atomic_load(&flags_h[c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) == 0) {
          if (__hip_atomic_load(&sync->abort, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0) break;
          if (++spins > kSpinLimit) {  // cannot happen (lower tickets never wait to load); never hang
            __hip_atomic_store(&sync->abort, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
          }
          __builtin_amdgcn_s_sleep(2);
        }
      }
    }
    __syncthreads();
  }

  // ---- store ----
#pragma unroll
  for (int it = 0; it < kPasses; ++it) {
    if (dst_off[it] >= 0) {
      __builtin_nontemporal_store(kval[it], &Ko[dst_off[it]]);
      __builtin_nontemporal_store(vval[it], &Vo[dst_off[it]]);
    }
  }
  if (pdst >= 0) pos_o[pdst] = pval;
}

// score of a masked token -> -1: below every real score (sums of probabilities are >= 0), so
// the select never prefers it to an unmasked token
__global__ void mask_scores_kernel(float* __restrict__ score, int64_t score_stride_h, int Nk,
                                   const uint8_t* __restrict__ valid) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j < Nk && valid[j] == 0) score[blockIdx.y * score_stride_h + j] = -1.f;
}

struct WsLayout {
  size_t idx_off, sync_off, flags_off, clear_bytes, total;
  int chunks_per_head;
};

WsLayout ws_layout(int n_layers, int Hkv, int Nk_in, int share_heads) {
  WsLayout w;
  const int hsel = share_heads ? 1 : Hkv;
  // the bookkeeping leads (pc_compact_status reads the abort word at offset 0); the flags follow
  // it directly, so one contiguous range is cleared per call
  size_t at = 0;
  w.sync_off = at;
  at += align_up(sizeof(GatherSync), 256);
  w.flags_off = at;
  w.chunks_per_head = ceil_div(Nk_in, kGatherRows);
  at += align_up(sizeof(int32_t) * static_cast<size_t>(n_layers) * Hkv * w.chunks_per_head, 256);
  w.clear_bytes = at;
  w.idx_off = at;
  at += align_up(sizeof(int32_t) * static_cast<size_t>(n_layers) * hsel * Nk_in, 256);
  w.total = at;
  return w;
}

// ---- pc_compact_static: the workspace as a file-scope device array ---------------------------
// For callers that cannot allocate.  Every GPU the library runs on holds its own copy of the
// array at its own address; in host code the array's NAME is only a handle for
// hipGetSymbolAddress, never a device address: kernels and every other use get the pointer
// looked up once per device.
static __device__ __align__(256) unsigned char scratch[PC_COMPACT_STATIC_BYTES];

constexpr int kMaxDevices = 64;
std::atomic<void*> g_scratch_ptr[kMaxDevices];   // per device: where its copy of `scratch` lives

// Device address of the current device's copy of the array (looked up on the first call on that
// device, with that device current).  Safe from several host threads: they all get the same answer.
int static_scratch(void** out) {
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  PC_REQUIRE(e == hipSuccess, PC_ERR_HIP, "pc_compact_static: hipGetDevice: %s", hipGetErrorString(e));
  PC_REQUIRE(dev >= 0 && dev < kMaxDevices, PC_ERR_UNSUPPORTED, "pc_compact_static: device %d outside [0, %d)", dev,
             kMaxDevices);
  void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
  if (p == nullptr) {
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    PC_REQUIRE(e == hipSuccess && p != nullptr, PC_ERR_HIP, "pc_compact_static: hipGetSymbolAddress: %s",
               hipGetErrorString(e));
    g_scratch_ptr[dev].store(p, std::memory_order_release);
  }
  *out = p;
  return PC_OK;
}

}  // namespace
}  // namespace pc

using namespace pc;

extern "C" size_t pc_compact_workspace_bytes(int Hkv, int Nk_in, int share_heads) {
  if (Hkv <= 0 || Nk_in <= 0) return 0;
  return ws_layout(1, Hkv, Nk_in, share_heads).total;
}

extern "C" size_t pc_compact_batch_workspace_bytes(int n_layers, int Hkv, int Nk_in, int share_heads) {
  if (n_layers <= 0 || Hkv <= 0 || Nk_in <= 0) return 0;
  return ws_layout(n_layers, Hkv, Nk_in, share_heads).total;
}

extern "C" int pc_compact(void* K, void* V, int32_t* pos, int dtype, int Hkv, int D,
                          int64_t kv_stride_h, int64_t pos_stride_h, const float* score,
                          int64_t score_stride_h, const pc_segment* seg_in, int n_seg,
                          const int32_t* budget, int share_heads, void* K_out, void* V_out,
                          int32_t* pos_out, int64_t kv_out_stride_h, int64_t pos_out_stride_h,
                          int32_t* idx_out, int64_t idx_stride_h, pc_segment* seg_out,
                          int32_t* Nk_out, void* ws, size_t ws_bytes, void* stream) {
  return pc_compact_batch(1, K, V, pos, dtype, Hkv, D, kv_stride_h, 0, pos_stride_h, 0, score, score_stride_h, 0,
                          seg_in, n_seg, budget, share_heads, K_out, V_out, pos_out, kv_out_stride_h, 0,
                          pos_out_stride_h, 0, idx_out, idx_stride_h, 0, seg_out, Nk_out, ws, ws_bytes, stream);
}

extern "C" size_t pc_compact_static_capacity(void) { return PC_COMPACT_STATIC_BYTES; }

extern "C" int pc_compact_static(void* K, void* V, int32_t* pos, int dtype, int Hkv, int D,
                                 int64_t kv_stride_h, int64_t pos_stride_h, const float* score,
                                 int64_t score_stride_h, const pc_segment* seg_in, int n_seg,
                                 const int32_t* budget, int share_heads, void* K_out, void* V_out,
                                 int32_t* pos_out, int64_t kv_out_stride_h, int64_t pos_out_stride_h,
                                 int32_t* idx_out, int64_t idx_stride_h, pc_segment* seg_out,
                                 int32_t* Nk_out, void* stream) {
  PC_REQUIRE(Hkv > 0 && n_seg >= 0 && n_seg <= PC_MAX_SEGMENTS && (n_seg == 0 || seg_in != nullptr), PC_ERR_SHAPE,
             "pc_compact_static: Hkv=%d n_seg=%d", Hkv, n_seg);
  const int64_t nk_in = n_seg ? static_cast<int64_t>(seg_in[n_seg - 1].start) + seg_in[n_seg - 1].len : 0;
  PC_REQUIRE(nk_in >= 0 && nk_in <= INT_MAX, PC_ERR_SHAPE, "pc_compact_static: segment table ends at row %lld",
             static_cast<long long>(nk_in));
  const size_t need = nk_in ? ws_layout(1, Hkv, static_cast<int>(nk_in), share_heads).total : 0;
  PC_REQUIRE(need <= PC_COMPACT_STATIC_BYTES, PC_ERR_WORKSPACE,
             "pc_compact_static: Hkv=%d x %lld rows needs %zu bytes of scratch, the built-in array holds %zu; "
             "use pc_compact with a workspace of the caller's",
             Hkv, static_cast<long long>(nk_in), need, static_cast<size_t>(PC_COMPACT_STATIC_BYTES));
  void* ptr = nullptr;
  if (int rc = static_scratch(&ptr)) return rc;
  // the select kernel of every call clears the tickets, flags and abort word it is about to use
  // (a fill kernel, not a memset), so what the last call left in the array does not matter
  return pc_compact(K, V, pos, dtype, Hkv, D, kv_stride_h, pos_stride_h, score, score_stride_h, seg_in, n_seg,
                    budget, share_heads, K_out, V_out, pos_out, kv_out_stride_h, pos_out_stride_h, idx_out,
                    idx_stride_h, seg_out, Nk_out, ptr, PC_COMPACT_STATIC_BYTES, stream);
}

extern "C" int pc_compact_batch(int n_layers, void* K, void* V, int32_t* pos, int dtype, int Hkv, int D,
                                int64_t kv_stride_h, int64_t kv_stride_l, int64_t pos_stride_h,
                                int64_t pos_stride_l, const float* score, int64_t score_stride_h,
                                int64_t score_stride_l, const pc_segment* seg_in, int n_seg,
                                const int32_t* budget, int share_heads, void* K_out, void* V_out,
                                int32_t* pos_out, int64_t kv_out_stride_h, int64_t kv_out_stride_l,
                                int64_t pos_out_stride_h, int64_t pos_out_stride_l, int32_t* idx_out,
                                int64_t idx_stride_h, int64_t idx_stride_l, pc_segment* seg_out,
                                int32_t* Nk_out, void* ws, size_t ws_bytes, void* stream) {
  return pc_compact_batch_phase(PC_COMPACT_SELECT | PC_COMPACT_GATHER, n_layers, K, V, pos, dtype, Hkv, D,
                                kv_stride_h, kv_stride_l, pos_stride_h, pos_stride_l, score, score_stride_h,
                                score_stride_l, seg_in, n_seg, budget, share_heads, K_out, V_out, pos_out,
                                kv_out_stride_h, kv_out_stride_l, pos_out_stride_h, pos_out_stride_l, idx_out,
                                idx_stride_h, idx_stride_l, seg_out, Nk_out, ws, ws_bytes, stream);
}

extern "C" int pc_compact_batch_phase(int phases, int n_layers, void* K, void* V, int32_t* pos, int dtype, int Hkv,
                                      int D, int64_t kv_stride_h, int64_t kv_stride_l, int64_t pos_stride_h,
                                      int64_t pos_stride_l, const float* score, int64_t score_stride_h,
                                      int64_t score_stride_l, const pc_segment* seg_in, int n_seg,
                                      const int32_t* budget, int share_heads, void* K_out, void* V_out,
                                      int32_t* pos_out, int64_t kv_out_stride_h, int64_t kv_out_stride_l,
                                      int64_t pos_out_stride_h, int64_t pos_out_stride_l, int32_t* idx_out,
                                      int64_t idx_stride_h, int64_t idx_stride_l, pc_segment* seg_out,
                                      int32_t* Nk_out, void* ws, size_t ws_bytes, void* stream) {
  PC_REQUIRE(phases >= 1 && phases <= (PC_COMPACT_SELECT | PC_COMPACT_GATHER), PC_ERR_SHAPE,
             "pc_compact: phases=%d", phases);
  PC_REQUIRE(dtype == PC_F32 || dtype == PC_BF16, PC_ERR_DTYPE, "pc_compact: dtype %d", dtype);
  PC_REQUIRE(Hkv > 0 && D > 0 && n_layers >= 1, PC_ERR_SHAPE, "pc_compact: layers=%d Hkv=%d D=%d", n_layers, Hkv, D);
  PC_REQUIRE(n_seg >= 0 && n_seg <= PC_MAX_SEGMENTS, PC_ERR_SHAPE,
             "pc_compact: n_seg=%d outside [0, %d]", n_seg, PC_MAX_SEGMENTS);
  pc_segment plan[PC_MAX_SEGMENTS];
  int32_t nk_out = 0;
  const int rc = pc_compact_plan(seg_in, n_seg, budget, plan, &nk_out);
  if (rc != PC_OK) return rc;
  if (seg_out)
    for (int s = 0; s < n_seg; ++s) seg_out[s] = plan[s];
  if (Nk_out) *Nk_out = nk_out;
  const int nk_in = n_seg ? seg_in[n_seg - 1].start + seg_in[n_seg - 1].len : 0;
  if (nk_in == 0 || nk_out == 0) return PC_OK;

  const int elt = dtype == PC_BF16 ? 2 : 4;
  const int row_bytes = D * elt;
  PC_REQUIRE(row_bytes == 256 || row_bytes == 512, PC_ERR_UNSUPPORTED,
             "pc_compact: rows of %d bytes (supported: 256 and 512)", row_bytes);
  PC_REQUIRE(K && V && pos && score && K_out && V_out && pos_out, PC_ERR_NULL,
             "pc_compact: K, V, pos, score or an output is NULL");
  const bool in_place = K_out == K;
  PC_REQUIRE((V_out == V) == in_place && (pos_out == pos) == in_place, PC_ERR_SHAPE,
             "pc_compact: outputs must alias the inputs all together or not at all");
  PC_REQUIRE(!in_place || (kv_out_stride_h == kv_stride_h && pos_out_stride_h == pos_stride_h &&
                           kv_out_stride_l == kv_stride_l && pos_out_stride_l == pos_stride_l),
             PC_ERR_SHAPE, "pc_compact: in-place compaction needs equal input and output strides");
  const int hsel = share_heads ? 1 : Hkv;
  PC_REQUIRE(kv_stride_h >= static_cast<int64_t>(nk_in) * D && kv_out_stride_h >= static_cast<int64_t>(nk_out) * D,
             PC_ERR_SHAPE, "pc_compact: a K/V head stride is smaller than rows*D");
  PC_REQUIRE(hsel == 1 || (pos_stride_h >= static_cast<int64_t>(nk_in) * 3 &&
                           pos_out_stride_h >= static_cast<int64_t>(nk_out) * 3 && score_stride_h >= nk_in),
             PC_ERR_SHAPE, "pc_compact: a pos/score head stride is too small");
  PC_REQUIRE(idx_out == nullptr || hsel == 1 || idx_stride_h >= nk_out, PC_ERR_SHAPE,
             "pc_compact: idx head stride %lld < Nk_out", static_cast<long long>(idx_stride_h));
  const uintptr_t al = reinterpret_cast<uintptr_t>(K) | reinterpret_cast<uintptr_t>(V) |
                       reinterpret_cast<uintptr_t>(K_out) | reinterpret_cast<uintptr_t>(V_out);
  PC_REQUIRE(al % 16 == 0 && (kv_stride_h * elt) % 16 == 0 && (kv_out_stride_h * elt) % 16 == 0 &&
                 (kv_stride_l * elt) % 16 == 0 && (kv_out_stride_l * elt) % 16 == 0,
             PC_ERR_SHAPE, "pc_compact: K/V buffers and head / layer strides must be 16-byte aligned");
  if (n_layers > 1) {
    PC_REQUIRE(kv_stride_l >= kv_stride_h * (Hkv - 1) + static_cast<int64_t>(nk_in) * D &&
                   kv_out_stride_l >= kv_out_stride_h * (Hkv - 1) + static_cast<int64_t>(nk_out) * D &&
                   pos_stride_l >= pos_stride_h * (hsel - 1) + static_cast<int64_t>(nk_in) * 3 &&
                   pos_out_stride_l >= pos_out_stride_h * (hsel - 1) + static_cast<int64_t>(nk_out) * 3 &&
                   score_stride_l >= score_stride_h * (hsel - 1) + nk_in &&
                   (idx_out == nullptr || idx_stride_l >= idx_stride_h * (hsel - 1) + nk_out),
               PC_ERR_SHAPE, "pc_compact_batch: a layer stride is smaller than one layer");
    PC_REQUIRE(!in_place || n_layers * Hkv <= kMaxTicketHeads, PC_ERR_UNSUPPORTED,
               "pc_compact_batch: in place supports at most %d (layer, KV head) pairs per call", kMaxTicketHeads);
  }
  const WsLayout lay = ws_layout(n_layers, Hkv, nk_in, share_heads);
  PC_REQUIRE(ws != nullptr && ws_bytes >= lay.total, PC_ERR_WORKSPACE,
             "pc_compact: workspace %zu bytes, need %zu", ws_bytes, lay.total);
  PC_REQUIRE(reinterpret_cast<uintptr_t>(ws) % 16 == 0, PC_ERR_WORKSPACE, "pc_compact: workspace not 16-byte aligned");

  SegTable tab;
  tab.n = n_seg;
  int max_prune_len = 0;
  for (int s = 0; s < n_seg; ++s) {
    tab.start[s] = seg_in[s].start;
    tab.len[s] = seg_in[s].len;
    tab.keep[s] = plan[s].len;
    tab.dst[s] = plan[s].start;
    tab.prune[s] = seg_in[s].kind == PC_SEG_FRAME && plan[s].len < seg_in[s].len;
    if (tab.prune[s]) max_prune_len = std::max(max_prune_len, seg_in[s].len);
  }
  for (int s = n_seg; s < PC_MAX_SEGMENTS; ++s) {
    tab.start[s] = tab.len[s] = tab.keep[s] = tab.dst[s] = 0;
    tab.prune[s] = 0;
  }

  hipStream_t st = static_cast<hipStream_t>(stream);
  uint8_t* wsb = static_cast<uint8_t*>(ws);
  int32_t* idx = idx_out ? idx_out : reinterpret_cast<int32_t*>(wsb + lay.idx_off);
  const int64_t idx_stride = idx_out ? idx_stride_h : nk_in;
  const int64_t idx_stride_layer = idx_out ? idx_stride_l : static_cast<int64_t>(hsel) * nk_in;
  GatherSync* sync = reinterpret_cast<GatherSync*>(wsb + lay.sync_off);
  int32_t* flags = reinterpret_cast<int32_t*>(wsb + lay.flags_off);

  const dim3 sgrid(n_seg, hsel * n_layers);
  // the select kernel also clears the in-place gather's counters and flags (contiguous in ws)
  int32_t* clear = in_place ? reinterpret_cast<int32_t*>(sync) : nullptr;
  const int n_clear = in_place ? static_cast<int>(lay.clear_bytes / sizeof(int32_t)) : 0;
  if (!(phases & PC_COMPACT_SELECT)) {
    // indices and cleared counters come from an earlier SELECT call with the same arguments
  } else if (max_prune_len > kRowsSelectMinLen && max_prune_len <= PC_MAX_SELECT_LEN &&
             n_seg * hsel * n_layers >= kRowsSelectMinUnits)
    select_rows_kernel<<<sgrid, 64, 0, st>>>(score, score_stride_h, idx, idx_stride, tab, clear, n_clear, hsel,
                                             score_stride_l, idx_stride_layer);
  else if (max_prune_len <= 256)
    select_block_kernel<1><<<sgrid, 256, 0, st>>>(score, score_stride_h, idx, idx_stride, tab, clear, n_clear, hsel,
                                                   score_stride_l, idx_stride_layer);
  else if (max_prune_len <= 1024)
    select_block_kernel<4><<<sgrid, 256, 0, st>>>(score, score_stride_h, idx, idx_stride, tab, clear, n_clear, hsel,
                                                   score_stride_l, idx_stride_layer);
  else if (max_prune_len <= PC_MAX_SELECT_LEN)
    select_block_kernel<16><<<sgrid, 256, 0, st>>>(score, score_stride_h, idx, idx_stride, tab, clear, n_clear, hsel,
                                                   score_stride_l, idx_stride_layer);
  else
  {
    select_kernel<0><<<sgrid, 64, 0, st>>>(score, score_stride_h, idx, idx_stride, tab, hsel, score_stride_l,
                                           idx_stride_layer);
    if (in_place) {
      PC_CHECK_LAUNCH("pc_compact select");
      clear_words<<<ceil_div(n_clear, 256), 256, 0, st>>>(clear, n_clear);
    }
  }
  PC_CHECK_LAUNCH("pc_compact select");
  if (!(phases & PC_COMPACT_GATHER)) return PC_OK;

  const int cpr = row_bytes / 16;
  const int chunks_per_head = ceil_div(nk_out, kGatherRows);
  const int64_t in_stride_c = kv_stride_h * elt / 16, out_stride_c = kv_out_stride_h * elt / 16;
  const dim3 ggrid(chunks_per_head * Hkv * n_layers);
  PC_REQUIRE(!in_place || Hkv * n_layers <= kMaxTicketHeads, PC_ERR_UNSUPPORTED,
             "pc_compact: in place supports at most %d (layer, KV head) pairs", kMaxTicketHeads);
  const int64_t in_stride_lc = kv_stride_l * elt / 16, out_stride_lc = kv_out_stride_l * elt / 16;
#define PC_LAUNCH_GATHER(CPR, ROWS, INPLACE)                                                             \
  gather_kernel<CPR, ROWS, INPLACE><<<ggrid, kGatherThreads, 0, st>>>(                                   \
      static_cast<const u32x4*>(K), static_cast<const u32x4*>(V), pos, static_cast<u32x4*>(K_out),       \
      static_cast<u32x4*>(V_out), pos_out, idx, idx_stride, share_heads, Hkv, nk_in, nk_out, in_stride_c, \
      out_stride_c, pos_stride_h, pos_out_stride_h, sync, flags, lay.chunks_per_head, tab, n_layers,      \
      in_stride_lc, out_stride_lc, pos_stride_l, pos_out_stride_l, idx_stride_layer)
  if (cpr == 16) {
    if (in_place) PC_LAUNCH_GATHER(16, kGatherRows, true); else PC_LAUNCH_GATHER(16, kGatherRows, false);
  } else if (cpr == 32) {
    if (in_place) PC_LAUNCH_GATHER(32, kGatherRows, true); else PC_LAUNCH_GATHER(32, kGatherRows, false);
  } else {
    PC_FAIL(PC_ERR_UNSUPPORTED, "pc_compact: rows of %d bytes (supported: 256 and 512)", row_bytes);
  }
#undef PC_LAUNCH_GATHER
  PC_CHECK_LAUNCH("pc_compact gather");
  return PC_OK;
}

extern "C" int pc_compact_status(const void* ws, void* stream) {
  PC_REQUIRE(ws != nullptr, PC_ERR_NULL, "pc_compact_status: ws is NULL");
  static_assert(offsetof(GatherSync, abort) == 0, "the abort word leads the workspace");
  int32_t word = 0;
  hipStream_t st = static_cast<hipStream_t>(stream);
  hipError_t e = hipMemcpyAsync(&word, ws, sizeof(word), hipMemcpyDeviceToHost, st);
  if (e == hipSuccess) e = hipStreamSynchronize(st);
  PC_REQUIRE(e == hipSuccess, PC_ERR_HIP, "pc_compact_status: %s", hipGetErrorString(e));
  PC_REQUIRE(word == 0, PC_ERR_ABORTED,
             "pc_compact_status: an in-place gather gave up waiting (workspace shared by overlapping calls?)");
  return PC_OK;
}

extern "C" int pc_mask_scores(float* score, int Hsel, int Nk, int64_t score_stride_h, const uint8_t* valid,
                              void* stream) {
  PC_REQUIRE(Hsel >= 0 && Nk >= 0, PC_ERR_SHAPE, "pc_mask_scores: Hsel=%d Nk=%d", Hsel, Nk);
  if (Hsel == 0 || Nk == 0) return PC_OK;
  PC_REQUIRE(score && valid, PC_ERR_NULL, "pc_mask_scores: score or valid is NULL");
  PC_REQUIRE(Hsel == 1 || score_stride_h >= Nk, PC_ERR_SHAPE, "pc_mask_scores: score head stride %lld < Nk",
             static_cast<long long>(score_stride_h));
  mask_scores_kernel<<<dim3(ceil_div(Nk, 256), Hsel), 256, 0, static_cast<hipStream_t>(stream)>>>(
      score, score_stride_h, Nk, valid);
  PC_CHECK_LAUNCH("pc_mask_scores");
  return PC_OK;
}
