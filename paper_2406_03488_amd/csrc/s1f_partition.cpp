// Computation-wise partition (Section 3.4, Eq. 7-8) and its variants: host-only, exact integer arithmetic.
//
// Additive cost model: token t (1-based) costs w(t) = 6*hidden + t, a prefix of x tokens costs
// W(x) = 6*hidden*x + x(x+1)/2 (Eq. 8 with P/L = 12*hidden^2, made additive over tokens, common factor
// 4*L*hidden removed).  Boundary i is the aligned x whose prefix cost is nearest to i/k of the total.  W is
// increasing, so a binary search over the aligned positions finds the first one reaching the target, and one
// comparison with its left neighbour decides which is nearer.
//
// Literal cost model: Eq. 8's per-segment line as printed, cost(a, b] = (b - a) * (12*hidden + b) in units of
// 2*L*hidden.  It is not additive, so the partition is the composition with the smallest largest cost: binary
// search on that bound T; for one T the latest segments are laid out from the right, each boundary as far left
// as T allows (the cost of (a, b] falls as a rises and rises with b, so the leftmost feasible boundaries are
// also the lexicographically smallest optimum).
//
// Re-balancing: measured segment costs define a piecewise-linear prefix cost; the same nearest rule places the
// new boundaries.  Prefix costs are compared as fractions with 128-bit cross products.
#include <cstdint>

#include "s1f.h"

namespace {
typedef unsigned __int128 u128;

inline u128 prefix_cost(uint64_t x, uint64_t hidden) { return (u128)6 * hidden * x + (u128)x * (x + 1) / 2; }

inline u128 absdiff(u128 a, u128 b) { return a >= b ? a - b : b - a; }

// Interior boundaries live on multiples of `align`; the last one must leave the final segment a token.
struct Grid {
  uint64_t n, k, align, last;   // last = largest aligned position below n
  bool ok() const { return last / align >= k - 1; }
  uint64_t clamp(uint64_t x, uint64_t prev, uint64_t i) const {
    const uint64_t lo = prev + align, hi = last - (k - 1 - i) * align;
    return x < lo ? lo : (x > hi ? hi : x);
  }
};

inline Grid make_grid(int64_t n, int32_t k, int64_t align) {
  Grid g;
  g.n = (uint64_t)n; g.k = (uint64_t)k; g.align = (uint64_t)align;
  g.last = (g.n - 1) / g.align * g.align;
  return g;
}

// Aligned position whose prefix cost is nearest to a target, for a non-decreasing prefix cost: `reach(x)` tells
// whether position x has reached the target, `nearer_left(x)` whether x - align is at least as near as x.
template <class Reach, class NearerLeft>
uint64_t nearest_aligned(const Grid &g, Reach reach, NearerLeft nearer_left) {
  uint64_t lo = 0, hi = g.n / g.align;                 // positions m * align, m in [lo, hi]
  if (!reach(hi * g.align)) return hi * g.align;       // target beyond the last aligned position
  while (lo < hi) {
    const uint64_t mid = (lo + hi) / 2;
    if (reach(mid * g.align)) hi = mid; else lo = mid + 1;
  }
  uint64_t x = lo * g.align;
  if (x > 0 && nearer_left(x)) x -= g.align;           // nearer on the left, or a tie: the smaller x
  return x;
}

int additive(const Grid &g, uint64_t h, int64_t *b) {
  const u128 total = prefix_cost(g.n, h);
  b[0] = 0;
  for (uint64_t i = 1; i < g.k; ++i) {
    const u128 target = (u128)i * total;               // compare k*W(x) with i*W(n)
    const uint64_t x = nearest_aligned(
        g, [&](uint64_t p) { return (u128)g.k * prefix_cost(p, h) >= target; },
        [&](uint64_t p) {
          return absdiff((u128)g.k * prefix_cost(p - g.align, h), target) <=
                 absdiff((u128)g.k * prefix_cost(p, h), target);
        });
    b[i] = (int64_t)g.clamp(x, (uint64_t)b[i - 1], i);
  }
  b[g.k] = (int64_t)g.n;
  return S1F_OK;
}

// Leftmost boundaries with every segment's literal cost <= T, laid out from the right; false if T is too small.
bool literal_layout(const Grid &g, uint64_t h, u128 T, int64_t *b) {
  uint64_t right = g.n;
  b[g.k] = (int64_t)g.n;
  for (uint64_t i = g.k; i >= 1; --i) {
    const u128 per_token = (u128)12 * h + right;
    const u128 span = T / per_token;                   // most tokens segment i may hold
    if (span == 0) return false;
    uint64_t a = span >= right ? 0 : right - (uint64_t)span;
    a = (a + g.align - 1) / g.align * g.align;         // boundaries sit on aligned positions
    if (a < (i - 1) * g.align) a = (i - 1) * g.align;  // i - 1 non-empty segments must fit on the left
    if (a >= right) return false;
    if (i == 1 && a != 0) return false;
    b[i - 1] = (int64_t)a;
    right = a;
  }
  return true;
}

int literal(const Grid &g, uint64_t h, int64_t *b) {
  u128 lo = 1, hi = (u128)g.n * ((u128)12 * h + g.n);  // one segment holding everything costs hi
  while (lo < hi) {
    const u128 mid = lo + (hi - lo) / 2;
    if (literal_layout(g, h, mid, b)) hi = mid; else lo = mid + 1;
  }
  return literal_layout(g, h, lo, b) ? S1F_OK : S1F_EINVAL;
}
}  // namespace

extern "C" int s1f_partition_ex(int64_t seq_len, int32_t n_seg, int32_t hidden, int32_t heads, int32_t cost_model,
                                int64_t align, int64_t *boundaries) {
  if (boundaries == nullptr || n_seg < 1 || seq_len < n_seg || hidden < 1 || heads < 1 || hidden % heads != 0 ||
      align < 1)
    return S1F_EINVAL;
  if (seq_len > (int64_t(1) << 30) || hidden > (1 << 24)) return S1F_EINVAL;   // keeps W(n) below 2^62
  const Grid g = make_grid(seq_len, n_seg, align);
  if (!g.ok()) return S1F_EINVAL;
  if (cost_model == S1F_COST_ADDITIVE) return additive(g, (uint64_t)hidden, boundaries);
  if (cost_model == S1F_COST_LITERAL) return literal(g, (uint64_t)hidden, boundaries);
  return S1F_EINVAL;
}

extern "C" int s1f_partition(int64_t seq_len, int32_t n_seg, int32_t hidden, int32_t heads, int64_t *boundaries) {
  return s1f_partition_ex(seq_len, n_seg, hidden, heads, S1F_COST_ADDITIVE, 1, boundaries);
}

extern "C" int s1f_partition_rebalance(int32_t n_seg, const int64_t *boundaries_in, const int64_t *seg_cost,
                                       int64_t align, int64_t *boundaries_out) {
  if (n_seg < 1 || n_seg > 65536 || boundaries_in == nullptr || seg_cost == nullptr || boundaries_out == nullptr || align < 1 ||
      boundaries_in[0] != 0)
    return S1F_EINVAL;
  u128 total = 0;
  for (int32_t i = 0; i < n_seg; ++i) {
    if (boundaries_in[i + 1] <= boundaries_in[i] || seg_cost[i] < 0) return S1F_EINVAL;
    total += (u128)seg_cost[i];
  }
  const int64_t n = boundaries_in[n_seg];
  // 2^16 segments * 2^48 cost * (2^30 tokens)^2 keeps every cross product below 2^128
  if (total == 0 || total > ((u128)1 << 48) || n > (int64_t(1) << 30)) return S1F_EINVAL;
  const Grid g = make_grid(n, n_seg, align);
  if (!g.ok()) return S1F_EINVAL;

  // prefix cost at position x as the fraction num/den: cost of whole segments before x + a linear share
  struct Frac { u128 num, den; };
  auto prefix = [&](uint64_t x) {
    u128 before = 0;
    int32_t s = 0;
    while (s < n_seg - 1 && (uint64_t)boundaries_in[s + 1] <= x) before += (u128)seg_cost[s++];
    const u128 len = (u128)(boundaries_in[s + 1] - boundaries_in[s]);
    return Frac{before * len + (u128)seg_cost[s] * (x - (uint64_t)boundaries_in[s]), len};
  };
  boundaries_out[0] = 0;
  for (uint64_t j = 1; j < g.k; ++j) {
    const u128 target = (u128)j * total;               // compare k*C(x) with j*total
    auto err_times_den = [&](const Frac &f) { return absdiff((u128)g.k * f.num, target * f.den); };
    const uint64_t x = nearest_aligned(
        g, [&](uint64_t p) { const Frac f = prefix(p); return (u128)g.k * f.num >= target * f.den; },
        [&](uint64_t p) {
          const Frac l = prefix(p - g.align), r = prefix(p);
          return err_times_den(l) * r.den <= err_times_den(r) * l.den;
        });
    // segments that cost nothing make the prefix cost flat: the smallest position of equal cost wins the tie
    const Frac fx = prefix(x);
    uint64_t lo = 0, hi = x / g.align;
    while (lo < hi) {
      const uint64_t mid = (lo + hi) / 2;
      const Frac fm = prefix(mid * g.align);
      if (fm.num * fx.den >= fx.num * fm.den) hi = mid; else lo = mid + 1;
    }
    boundaries_out[j] = (int64_t)g.clamp(lo * g.align, (uint64_t)boundaries_out[j - 1], j);
  }
  boundaries_out[n_seg] = n;
  return S1F_OK;
}
