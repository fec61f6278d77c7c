// Host-only half of libpackcache: status strings, budgets (Sec. 3.4, Eq. 4-8) and the
// segment bookkeeping of compaction.  No device work happens in this file.
#include <math.h>
#include <string.h>

#include <algorithm>
#include <vector>

#include "common.h"

namespace pc {

static thread_local char g_detail[512] = "";

void set_detail(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_detail, sizeof(g_detail), fmt, ap);
  va_end(ap);
}

namespace {

// Minimal unsigned big integer: enough to floor products and quotients of powers of a
// double exactly, so that budgets are integers fixed by the mathematics and not by the
// rounding of pow().
struct BigU {
  std::vector<uint32_t> w;  // little endian limbs, no leading zeros

  BigU() {}
  explicit BigU(uint64_t v) {
    while (v) {
      w.push_back(static_cast<uint32_t>(v));
      v >>= 32;
    }
  }
  void trim() {
    while (!w.empty() && w.back() == 0) w.pop_back();
  }
  size_t bits() const {
    if (w.empty()) return 0;
    return 32 * (w.size() - 1) + (32 - __builtin_clz(w.back()));
  }
  void mul_small(uint64_t m) {
    unsigned __int128 carry = 0;
    for (size_t i = 0; i < w.size(); ++i) {
      unsigned __int128 t = static_cast<unsigned __int128>(w[i]) * m + carry;
      w[i] = static_cast<uint32_t>(t);
      carry = t >> 32;
    }
    while (carry) {
      w.push_back(static_cast<uint32_t>(carry));
      carry >>= 32;
    }
    trim();
  }
  void shl(size_t s) {
    if (w.empty() || s == 0) return;
    const size_t limbs = s / 32, b = s % 32;
    std::vector<uint32_t> r(w.size() + limbs + 1, 0);
    for (size_t i = 0; i < w.size(); ++i) {
      const uint64_t v = static_cast<uint64_t>(w[i]) << b;
      r[i + limbs] |= static_cast<uint32_t>(v);
      r[i + limbs + 1] |= static_cast<uint32_t>(v >> 32);
    }
    w.swap(r);
    trim();
  }
  void add(const BigU& o) {
    if (o.w.size() > w.size()) w.resize(o.w.size(), 0);
    uint64_t carry = 0;
    for (size_t i = 0; i < w.size(); ++i) {
      const uint64_t t = static_cast<uint64_t>(w[i]) + (i < o.w.size() ? o.w[i] : 0) + carry;
      w[i] = static_cast<uint32_t>(t);
      carry = t >> 32;
    }
    if (carry) w.push_back(static_cast<uint32_t>(carry));
  }
  // floor(*this / 2^s), which the caller knows fits in 64 bits
  uint64_t shr_to_u64(size_t s) const {
    const size_t li = s / 32, b = s % 32;
    auto limb = [&](size_t i) -> unsigned __int128 { return i < w.size() ? w[i] : 0u; };
    const unsigned __int128 v = limb(li) | (limb(li + 1) << 32) | (limb(li + 2) << 64);
    return static_cast<uint64_t>(v >> b);
  }
  static int cmp(const BigU& a, const BigU& b) {
    if (a.w.size() != b.w.size()) return a.w.size() < b.w.size() ? -1 : 1;
    for (size_t i = a.w.size(); i-- > 0;)
      if (a.w[i] != b.w[i]) return a.w[i] < b.w[i] ? -1 : 1;
    return 0;
  }
  long double approx(int* exp2) const {  // value ~= ret * 2^exp2, ret from the top 96 bits
    long double v = 0;
    const size_t n = w.size(), take = std::min<size_t>(n, 3);
    for (size_t i = 0; i < take; ++i) v = v * 4294967296.0L + w[n - 1 - i];
    *exp2 = static_cast<int>(32 * (n - take));
    return v;
  }
};

// floor(a / b) for a quotient known to be below 2^40: estimate from the leading bits,
// then settle the last unit with exact comparisons.
uint64_t floor_div_small_quotient(const BigU& a, const BigU& b) {
  if (b.w.empty() || BigU::cmp(a, b) < 0) return 0;
  int ea, eb;
  const long double fa = a.approx(&ea), fb = b.approx(&eb);
  long double est = ldexpl(fa / fb, ea - eb);
  uint64_t q = est > 1 ? static_cast<uint64_t>(est) : 0;
  if (q > 0) --q;  // start at or below the true quotient (estimate is good to < 1 unit)
  for (int guard = 0; guard < 8; ++guard) {
    BigU t = b;
    t.mul_small(q + 1);
    if (BigU::cmp(t, a) <= 0)
      ++q;
    else
      break;
  }
  for (int guard = 0; guard < 8; ++guard) {
    BigU t = b;
    t.mul_small(q);
    if (BigU::cmp(t, a) > 0)
      --q;
    else
      break;
  }
  return q;
}

// gamma = mant * 2^(-shift) exactly, mant odd or zero, shift >= 0 for gamma in (0, 1].
void dyadic(double gamma, uint64_t* mant, int* shift) {
  int x;
  const double f = frexp(gamma, &x);  // gamma = f * 2^x, f in [0.5, 1)
  uint64_t m = static_cast<uint64_t>(ldexp(f, 53));
  int s = 53 - x;
  while (m && !(m & 1) && s > 0) {
    m >>= 1;
    --s;
  }
  *mant = m;
  *shift = s;
}

int active_window(int b_one, int w, int q_min) {
  if (q_min <= 0) return w;
  return static_cast<int>(std::min<int64_t>(w, b_one / q_min));
}

// t_d = q_min + floor(free * num_d / den) with exact integers; leftovers to d = 1.
void waterfill(int b_one, int q_min, const std::vector<BigU>& num, const BigU& den, int n_total,
               int32_t* out) {
  const int w = static_cast<int>(num.size());
  const int64_t free_tokens = static_cast<int64_t>(b_one) - static_cast<int64_t>(w) * q_min;
  int64_t sum = 0;
  for (int d = 0; d < w; ++d) {
    BigU a = num[d];
    a.mul_small(static_cast<uint64_t>(free_tokens));
    out[d] = static_cast<int32_t>(q_min + static_cast<int64_t>(floor_div_small_quotient(a, den)));
    sum += out[d];
  }
  if (w > 0) out[0] += static_cast<int32_t>(b_one - sum);
  for (int d = w; d < n_total; ++d) out[d] = 0;
}

}  // namespace
}  // namespace pc

using namespace pc;

extern "C" const char* pc_strerror(int status) {
  switch (status) {
    case PC_OK: return "ok";
    case PC_ERR_NULL: return "required pointer is NULL";
    case PC_ERR_SHAPE: return "inconsistent shape, stride or segment table";
    case PC_ERR_DTYPE: return "unknown dtype";
    case PC_ERR_UNSUPPORTED: return "configuration not covered by the kernels";
    case PC_ERR_BUDGET: return "invalid budget, decay factor or budget mode";
    case PC_ERR_WORKSPACE: return "workspace missing or too small";
    case PC_ERR_HIP: return "HIP runtime error";
    case PC_ERR_ABORTED: return "in-place compaction gave up a wait";
    default: return "unknown status";
  }
}

extern "C" const char* pc_last_error_detail(void) { return g_detail; }

extern "C" int pc_version(void) { return 104; }

extern "C" int pc_budget(int mode, int n_frame_tokens, int n_past, double gamma, int b_min,
                         int32_t* budget_out) {
  PC_REQUIRE(n_frame_tokens >= 0 && n_past >= 0 && b_min >= 0, PC_ERR_BUDGET,
             "pc_budget: N=%d n_past=%d b_min=%d must be non-negative", n_frame_tokens, n_past, b_min);
  PC_REQUIRE(mode >= PC_BUDGET_POW && mode <= PC_BUDGET_SLIDE, PC_ERR_BUDGET,
             "pc_budget: unknown mode %d", mode);
  if (n_past == 0) return PC_OK;
  PC_REQUIRE(budget_out != nullptr, PC_ERR_NULL, "pc_budget: budget_out is NULL");
  const int N = n_frame_tokens;
  const bool needs_gamma = mode == PC_BUDGET_POW || mode == PC_BUDGET_NORM;
  PC_REQUIRE(!needs_gamma || (gamma > 0.0 && gamma <= 1.0), PC_ERR_BUDGET,
             "pc_budget: decay factor %g outside (0, 1]", gamma);

  if (mode == PC_BUDGET_SLIDE) {
    for (int d = 0; d < n_past; ++d) budget_out[d] = d == 0 ? N : 0;
    return PC_OK;
  }

  if (mode == PC_BUDGET_POW) {
    uint64_t mant;
    int shift;
    dyadic(gamma, &mant, &shift);
    BigU p(static_cast<uint64_t>(N));  // N * mant^d
    for (int d = 1; d <= n_past; ++d) {
      p.mul_small(mant);
      const size_t s = static_cast<size_t>(shift) * d;
      int64_t b = s >= p.bits() ? 0 : static_cast<int64_t>(p.shr_to_u64(s));
      b = std::max<int64_t>(b, b_min);
      budget_out[d - 1] = static_cast<int32_t>(std::min<int64_t>(b, N));
    }
    return PC_OK;
  }

  const int we = active_window(N, n_past, b_min);
  std::vector<BigU> num(we);
  BigU den;
  if (mode == PC_BUDGET_NORM) {
    // rho^d / sum_j rho^j with rho = mant / 2^shift: scale both by 2^(shift * we).
    uint64_t mant;
    int shift;
    dyadic(gamma, &mant, &shift);
    BigU pw(1);
    for (int d = 1; d <= we; ++d) {
      pw.mul_small(mant);
      num[d - 1] = pw;
      num[d - 1].shl(static_cast<size_t>(shift) * (we - d));
      den.add(num[d - 1]);
    }
  } else {  // PC_BUDGET_HALF: 2^-min(d, we-1), scaled by 2^(we-1); the shares sum to one
    for (int d = 1; d <= we; ++d) {
      num[d - 1] = BigU(1);
      num[d - 1].shl(static_cast<size_t>(we - 1 - std::min(d, we - 1)));
    }
    den = BigU(1);
    den.shl(static_cast<size_t>(std::max(we - 1, 0)));
  }
  waterfill(N, b_min, num, den, n_past, budget_out);
  return PC_OK;
}

extern "C" int pc_compact_plan(const pc_segment* seg_in, int n_seg, const int32_t* budget,
                               pc_segment* seg_out, int32_t* Nk_out) {
  PC_REQUIRE(n_seg >= 0, PC_ERR_SHAPE, "pc_compact_plan: n_seg=%d", n_seg);
  PC_REQUIRE(n_seg == 0 || (seg_in && budget), PC_ERR_NULL, "pc_compact_plan: seg_in/budget is NULL");
  int64_t at_in = 0, at_out = 0;
  for (int s = 0; s < n_seg; ++s) {
    const pc_segment& g = seg_in[s];
    PC_REQUIRE(g.len >= 0 && g.start == at_in, PC_ERR_SHAPE,
               "pc_compact_plan: segment %d (start %d, len %d) does not continue at row %lld", s,
               g.start, g.len, static_cast<long long>(at_in));
    PC_REQUIRE(g.kind >= PC_SEG_TEXT && g.kind <= PC_SEG_SELF, PC_ERR_SHAPE,
               "pc_compact_plan: segment %d has unknown kind %d", s, g.kind);
    int keep = g.len;
    if (g.kind == PC_SEG_FRAME) {
      PC_REQUIRE(budget[s] >= 0, PC_ERR_BUDGET, "pc_compact_plan: budget[%d]=%d is negative", s,
                 budget[s]);
      keep = std::min(g.len, budget[s]);
    }
    if (seg_out) seg_out[s] = pc_segment{static_cast<int32_t>(at_out), keep, g.kind, g.frame};
    at_in += g.len;
    at_out += keep;
    PC_REQUIRE(at_in <= INT32_MAX, PC_ERR_SHAPE, "pc_compact_plan: more than 2^31-1 rows");
  }
  if (Nk_out) *Nk_out = static_cast<int32_t>(at_out);
  return PC_OK;
}

extern "C" int pc_masked_budgets(const pc_segment* seg, int n_seg, const int32_t* budget, const uint8_t* valid,
                                 int32_t* budget_out) {
  PC_REQUIRE(n_seg >= 0, PC_ERR_SHAPE, "pc_masked_budgets: n_seg=%d", n_seg);
  PC_REQUIRE(n_seg == 0 || (seg && budget && valid && budget_out), PC_ERR_NULL,
             "pc_masked_budgets: a pointer is NULL");
  for (int s = 0; s < n_seg; ++s) {
    const pc_segment& g = seg[s];
    PC_REQUIRE(g.len >= 0 && g.start >= 0, PC_ERR_SHAPE, "pc_masked_budgets: segment %d (start %d, len %d)", s,
               g.start, g.len);
    int32_t b = budget[s];
    if (g.kind == PC_SEG_FRAME) {
      PC_REQUIRE(b >= 0, PC_ERR_BUDGET, "pc_masked_budgets: budget[%d]=%d is negative", s, b);
      int32_t n_valid = 0;
      for (int32_t i = 0; i < g.len; ++i) n_valid += valid[g.start + i] != 0;
      b = std::min(b, n_valid);
    }
    budget_out[s] = b;
  }
  return PC_OK;
}
