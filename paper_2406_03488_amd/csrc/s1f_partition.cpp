// Computation-wise partition (Section 3.4, Eq. 7-8): host-only, exact integer arithmetic.
//
// Token t (1-based) costs w(t) = 6*hidden + t, a prefix of x tokens costs W(x) = 6*hidden*x + x(x+1)/2
// (Eq. 8 with P/L = 12*hidden^2, made additive over tokens, common factor 4*L*hidden removed).
// Boundary i is the x whose prefix cost is nearest to i/k of the total.  W is strictly increasing, so
// the nearest x is found from the real root of W(x) = i*W(n)/k (closed form, used only as a starting
// guess) followed by an exact integer walk to the first x with k*W(x) >= i*W(n) and a comparison with
// its left neighbour.
#include <cmath>
#include <cstdint>

#include "s1f.h"

namespace {
typedef unsigned __int128 u128;

inline u128 prefix_cost(uint64_t x, uint64_t hidden) { return (u128)6 * hidden * x + (u128)x * (x + 1) / 2; }
}  // namespace

extern "C" int s1f_partition(int64_t seq_len, int32_t n_seg, int32_t hidden, int32_t heads, int64_t *boundaries) {
  if (boundaries == nullptr || n_seg < 1 || seq_len < n_seg || hidden < 1 || heads < 1 || hidden % heads != 0)
    return S1F_EINVAL;
  if (seq_len > (int64_t(1) << 30) || hidden > (1 << 24)) return S1F_EINVAL;   // keeps W(n) below 2^62
  const uint64_t n = (uint64_t)seq_len, k = (uint64_t)n_seg, h = (uint64_t)hidden;
  const u128 total = prefix_cost(n, h);
  boundaries[0] = 0;
  for (uint64_t i = 1; i < k; ++i) {
    const u128 target = (u128)i * total;   // compare k*W(x) with i*W(n)
    // real root of x^2/2 + (6h + 1/2) x - i W(n)/k = 0
    const long double bq = 6.0L * (long double)h + 0.5L;
    const long double rhs = (long double)i * (long double)total / (long double)k;
    long double guess = -bq + sqrtl(bq * bq + 2.0L * rhs);
    if (!(guess >= 0.0L)) guess = 0.0L;
    if (guess > (long double)n) guess = (long double)n;
    uint64_t x = (uint64_t)guess;
    while (x < n && (u128)k * prefix_cost(x, h) < target) ++x;          // first x reaching the target ...
    while (x > 0 && (u128)k * prefix_cost(x - 1, h) >= target) --x;     // ... and no earlier one does
    if (x > 0) {
      const u128 above = (u128)k * prefix_cost(x, h) >= target ? (u128)k * prefix_cost(x, h) - target
                                                                  : target - (u128)k * prefix_cost(x, h);
      const u128 below = target - (u128)k * prefix_cost(x - 1, h);
      if (below <= above) --x;   // nearer on the left, or a tie: the smaller x
    }
    // every segment keeps at least one token
    const uint64_t lo = (uint64_t)boundaries[i - 1] + 1, hi = n - (k - i);
    if (x < lo) x = lo;
    if (x > hi) x = hi;
    boundaries[i] = (int64_t)x;
  }
  boundaries[n_seg] = seq_len;
  return S1F_OK;
}
