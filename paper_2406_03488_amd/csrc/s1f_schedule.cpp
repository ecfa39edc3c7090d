// Order of passes of one pipeline device under the sequence-level 1F1B schedule (Section 3.2, Eq. 4).
// Host code, no device work.  The order is enumerated in closed form: the forward passes run in
// (micro-batch, segment) order; the backward passes run micro-batch by micro-batch with the segments of a
// micro-batch in descending order (what the partially ordered queue of Section 3.2 returns when every
// micro-batch it holds at its head is complete, which the warm-up count guarantees); the first backward pass
// follows forward pass number warm-up + 1.
#include <stdint.h>

#include "s1f.h"

namespace {
bool valid(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg) {
  return pp_size >= 1 && device >= 1 && device <= pp_size && n_micro >= 1 && n_seg >= 1 &&
         (int64_t)n_micro * n_seg <= (int64_t(1) << 40);
}
int64_t warmup_of(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg) {
  const int64_t total = (int64_t)n_micro * n_seg;
  if (n_micro <= pp_size) return total;   // no steady phase: every forward pass comes first
  const int64_t w = (int64_t)pp_size - device - 1 + n_seg;
  return w < total ? w : total;
}
}  // namespace

extern "C" int s1f_seq1f1b_warmup(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg, int64_t *warmup) {
  if (!valid(pp_size, device, n_micro, n_seg) || !warmup) return S1F_EINVAL;
  *warmup = warmup_of(pp_size, device, n_micro, n_seg);
  return S1F_OK;
}

extern "C" int s1f_seq1f1b_order(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg, s1f_pass *order,
                                 int64_t capacity, int64_t *n_passes) {
  if (!valid(pp_size, device, n_micro, n_seg) || !n_passes) return S1F_EINVAL;
  const int64_t total = (int64_t)n_micro * n_seg;
  *n_passes = 2 * total;
  if (!order || capacity < 2 * total) return S1F_EINVAL;
  const int64_t w = warmup_of(pp_size, device, n_micro, n_seg);
  int64_t at = 0;
  auto forward = [&](int64_t u) { order[at++] = s1f_pass{(int32_t)(u / n_seg), (int32_t)(u % n_seg), 0}; };
  auto backward = [&](int64_t t) { order[at++] = s1f_pass{(int32_t)(t / n_seg), (int32_t)(n_seg - 1 - t % n_seg), 1}; };
  for (int64_t u = 0; u < w; ++u) forward(u);                      // warm-up phase
  for (int64_t t = 0; t < total - w; ++t) {                        // steady phase
    forward(w + t);
    backward(t);
  }
  for (int64_t t = total - w; t < total; ++t) backward(t);         // cooling-down phase
  return S1F_OK;
}

// Share of a batch's intermediate states that device i holds at its peak (Section 3.1: A * w_i / sum_j w_j for
// total activation memory A), as the exact fraction w_i / sum_j w_j of the warm-up counts of Eq. 4 (Eq. 1 for
// n_seg = 1).  For M > P the cap of the warm-up count at M * k never binds (M * k >= (P + 1) k > P + k - 2), so
// the sum has the closed form P (P - 1) / 2 + P (k - 1); for M <= P every device holds everything: 1 / P.
extern "C" int s1f_seq1f1b_peak_memory_share(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg,
                                             int64_t *numerator, int64_t *denominator) {
  if (!valid(pp_size, device, n_micro, n_seg) || !numerator || !denominator) return S1F_EINVAL;
  const int64_t P = pp_size, k = n_seg;
  const int64_t den = n_micro <= pp_size ? P * (int64_t)n_micro * k : P * (P - 1) / 2 + P * (k - 1);
  if (den == 0) return S1F_EINVAL;   // one device, whole sequences: no warm-up phase anywhere, the share is undefined
  *numerator = warmup_of(pp_size, device, n_micro, n_seg);
  *denominator = den;
  return S1F_OK;
}
