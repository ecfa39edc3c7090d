// Pipeline calculators (host code, no device work): warm-up counts and pass order of the interleaved
// sequence-level schedule (Section 3.3, Eq. 5-6), and a timeline of all devices of a pipeline that yields the
// makespan, each device's busy time (hence the bubble ratio) and the intermediate states it holds at its peak
// (Sections 3.1-3.3), optionally with the backward pass split into an input-gradient pass and a deferrable
// weight-gradient pass (Appendix A.1).
//
// Interleaved order, enumerated in closed form.  The M*k sub-sequences in forward order are cut into groups of
// P.  Forward pass number v: group v / (P n), inside it stage-chunk (v mod P n) / P and member v mod P.
// Backward pass number t: same group, chunks from last to first, members in the order of the partially ordered
// queue of Section 3.2 — a group holds P / k whole micro-batches, so member q is micro-batch q / k of the group,
// segment k - 1 - q mod k.
//
// Timeline.  Every device walks its fixed order; a pass starts when the device is free and its input has arrived
// (the same sub-sequence from the previous stage for a forward pass, from the next stage for a backward pass,
// its own forward pass on the last stage; plus the transfer time when that stage is on another device).  The
// loop sweeps the devices, advancing each as far as its inputs are known, until all passes are placed; a sweep
// that places nothing is a dead-lock.
#include <stdint.h>

#include <vector>

#include "s1f.h"

namespace {
struct Shape {
  int64_t P, M, k, n;
  int64_t units() const { return M * k; }          // sub-sequences of a batch
  int64_t per_device() const { return M * k * n; } // forward passes of one device
};

bool valid(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg, int32_t n_chunks) {
  return pp_size >= 1 && device >= 1 && device <= pp_size && n_micro >= 1 && n_seg >= 1 && n_chunks >= 1 &&
         (int64_t)n_micro * n_seg * n_chunks <= (int64_t(1) << 40);
}

bool groups_hold_whole_micro_batches(const Shape &s) { return s.units() % s.P == 0 && s.P % s.k == 0; }

int64_t interleaved_warmup(const Shape &s, int64_t device) {
  const int64_t w = (s.P - device) * 2 + (s.n - 1) * s.P + s.k - 1;   // Eq. 6; Eq. 5 when k = 1
  return w < s.per_device() ? w : s.per_device();
}

s1f_stage_pass interleaved_forward(const Shape &s, int64_t v) {
  const int64_t g = v / (s.P * s.n), r = v % (s.P * s.n), u = g * s.P + r % s.P;
  return s1f_stage_pass{0, (int32_t)(u / s.k), (int32_t)(u % s.k), (int32_t)(r / s.P)};
}

s1f_stage_pass interleaved_backward(const Shape &s, int64_t t) {
  const int64_t g = t / (s.P * s.n), r = t % (s.P * s.n), q = r % s.P;
  return s1f_stage_pass{1, (int32_t)(g * (s.P / s.k) + q / s.k), (int32_t)(s.k - 1 - q % s.k),
                        (int32_t)(s.n - 1 - r / s.P)};
}

// warm-up forward passes, then one forward and one backward per step, then the remaining backward passes
template <class Fwd, class Bwd, class Emit>
void one_f_one_b(int64_t total, int64_t warmup, Fwd fwd, Bwd bwd, Emit emit) {
  for (int64_t v = 0; v < warmup; ++v) emit(fwd(v));
  for (int64_t t = 0; t < total - warmup; ++t) {
    emit(fwd(warmup + t));
    emit(bwd(t));
  }
  for (int64_t t = total - warmup; t < total; ++t) emit(bwd(t));
}

void device_order(const Shape &s, int64_t device, std::vector<s1f_stage_pass> &out) {
  out.clear();
  out.reserve(2 * s.per_device());
  auto emit = [&](const s1f_stage_pass &p) { out.push_back(p); };
  if (s.n == 1) {   // the sequence-level 1F1B order of Section 3.2 (Eq. 4)
    int64_t w = 0;
    s1f_seq1f1b_warmup((int32_t)s.P, (int32_t)device, (int32_t)s.M, (int32_t)s.k, &w);
    one_f_one_b(
        s.units(), w,
        [&](int64_t u) { return s1f_stage_pass{0, (int32_t)(u / s.k), (int32_t)(u % s.k), 0}; },
        [&](int64_t t) { return s1f_stage_pass{1, (int32_t)(t / s.k), (int32_t)(s.k - 1 - t % s.k), 0}; }, emit);
  } else {
    one_f_one_b(
        s.per_device(), interleaved_warmup(s, device), [&](int64_t v) { return interleaved_forward(s, v); },
        [&](int64_t t) { return interleaved_backward(s, t); }, emit);
  }
}
}  // namespace

extern "C" int s1f_seq1f1b_interleaved_warmup(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg,
                                              int32_t n_chunks, int64_t *warmup) {
  if (!valid(pp_size, device, n_micro, n_seg, n_chunks) || !warmup) return S1F_EINVAL;
  *warmup = interleaved_warmup(Shape{pp_size, n_micro, n_seg, n_chunks}, device);
  return S1F_OK;
}

extern "C" int s1f_seq1f1b_interleaved_order(int32_t pp_size, int32_t device, int32_t n_micro, int32_t n_seg,
                                             int32_t n_chunks, s1f_stage_pass *order, int64_t capacity,
                                             int64_t *n_passes) {
  if (!valid(pp_size, device, n_micro, n_seg, n_chunks) || !n_passes) return S1F_EINVAL;
  const Shape s{pp_size, n_micro, n_seg, n_chunks};
  if (!groups_hold_whole_micro_batches(s)) return S1F_EUNSUPPORTED;
  *n_passes = 2 * s.per_device();
  if (!order || capacity < *n_passes) return S1F_EINVAL;
  int64_t at = 0;
  one_f_one_b(
      s.per_device(), interleaved_warmup(s, device), [&](int64_t v) { return interleaved_forward(s, v); },
      [&](int64_t t) { return interleaved_backward(s, t); }, [&](const s1f_stage_pass &p) { order[at++] = p; });
  return S1F_OK;
}

extern "C" int s1f_pipeline_simulate(const s1f_pipeline_desc *desc, int64_t *makespan, int64_t *busy,
                                     int64_t *peak_live, int64_t *peak_pending_wgrad, double *bubble_ratio) {
  if (!desc || !makespan || !busy || !peak_live || !desc->t_fwd || !desc->t_bwd || desc->reserved != 0)
    return S1F_EINVAL;
  if (!valid(desc->pp_size, 1, desc->n_micro, desc->n_seg, desc->n_chunks)) return S1F_EINVAL;
  const bool split = desc->split_weight_grad != 0;
  if ((desc->split_weight_grad & ~1) != 0 || (split && !desc->t_wgrad) || desc->t_comm < 0 ||
      desc->max_pending_wgrad < 0)
    return S1F_EINVAL;
  const Shape s{desc->pp_size, desc->n_micro, desc->n_seg, desc->n_chunks};
  if (s.per_device() * s.P > (int64_t(1) << 24)) return S1F_EINVAL;      // keeps the tables below 1 GiB
  if (s.n > 1 && !groups_hold_whole_micro_batches(s)) return S1F_EUNSUPPORTED;
  for (int64_t j = 0; j < s.k; ++j) {
    const int64_t limit = int64_t(1) << 36;                               // sums stay far below 2^63
    if (desc->t_fwd[j] < 0 || desc->t_bwd[j] < 0 || desc->t_fwd[j] > limit || desc->t_bwd[j] > limit) return S1F_EINVAL;
    if (split && (desc->t_wgrad[j] < 0 || desc->t_wgrad[j] > limit)) return S1F_EINVAL;
    if (desc->seg_tokens && desc->seg_tokens[j] < 0) return S1F_EINVAL;
  }
  if (desc->t_comm > (int64_t(1) << 36)) return S1F_EINVAL;

  const int64_t V = s.n * s.P;
  // end time of pass (backward?, micro-batch, segment, stage); -1 = not placed yet
  std::vector<int64_t> finish((size_t)(2 * s.units() * V), -1);
  auto slot = [&](int backward, int64_t m, int64_t j, int64_t stage) {
    return (size_t)(((backward * s.M + m) * s.k + j) * V + stage);
  };
  std::vector<std::vector<s1f_stage_pass>> order((size_t)s.P);
  for (int64_t d = 0; d < s.P; ++d) device_order(s, d + 1, order[(size_t)d]);

  struct Device {
    size_t next = 0;
    int64_t free_at = 0, busy = 0, live = 0, peak_live = 0, peak_pending = 0;
    std::vector<int32_t> pending;   // segments of the weight-gradient passes waiting, oldest first
    size_t pending_head = 0;
  };
  std::vector<Device> dev((size_t)s.P);
  auto tokens = [&](int64_t j) { return desc->seg_tokens ? desc->seg_tokens[j] : int64_t(1); };
  auto run_wgrad = [&](Device &dv) {
    const int32_t j = dv.pending[dv.pending_head++];
    dv.free_at += desc->t_wgrad[j];
    dv.busy += desc->t_wgrad[j];
    dv.live -= tokens(j);
  };

  int64_t remaining = 2 * s.per_device() * s.P;
  while (remaining > 0) {
    bool moved = false;
    for (int64_t d = 0; d < s.P; ++d) {
      Device &dv = dev[(size_t)d];
      const std::vector<s1f_stage_pass> &ord = order[(size_t)d];
      while (dv.next < ord.size()) {
        const s1f_stage_pass &p = ord[dv.next];
        const int64_t stage = (int64_t)p.chunk * s.P + d;
        int64_t ready = 0;
        if (p.kind == 0 ? stage > 0 : true) {
          int64_t src_stage, src_end;
          if (p.kind == 0) {
            src_stage = stage - 1;
            src_end = finish[slot(0, p.micro_batch, p.segment, src_stage)];
          } else if (stage == V - 1) {
            src_stage = stage;
            src_end = finish[slot(0, p.micro_batch, p.segment, stage)];
          } else {
            src_stage = stage + 1;
            src_end = finish[slot(1, p.micro_batch, p.segment, src_stage)];
          }
          if (src_end < 0) break;   // input not produced yet
          ready = src_end + (src_stage % s.P != d ? desc->t_comm : 0);
        }
        if (split)
          while (dv.pending_head < dv.pending.size() &&
                 (ready > dv.free_at || (int64_t)(dv.pending.size() - dv.pending_head) > desc->max_pending_wgrad))
            run_wgrad(dv);
        const int64_t start = dv.free_at > ready ? dv.free_at : ready;
        const int64_t dur = p.kind == 0 ? desc->t_fwd[p.segment] : desc->t_bwd[p.segment];
        dv.free_at = start + dur;
        dv.busy += dur;
        finish[slot(p.kind, p.micro_batch, p.segment, stage)] = dv.free_at;
        if (p.kind == 0) {
          dv.live += tokens(p.segment);
          if (dv.live > dv.peak_live) dv.peak_live = dv.live;
        } else if (!split) {
          dv.live -= tokens(p.segment);
        } else {
          dv.pending.push_back(p.segment);
          const int64_t waiting = (int64_t)(dv.pending.size() - dv.pending_head);
          if (waiting > dv.peak_pending) dv.peak_pending = waiting;
        }
        ++dv.next;
        --remaining;
        moved = true;
      }
    }
    if (!moved) return S1F_EUNSUPPORTED;   // dead-lock: cannot happen with the orders generated above
  }
  *makespan = 0;
  int64_t busy_sum = 0;
  for (int64_t d = 0; d < s.P; ++d) {
    Device &dv = dev[(size_t)d];
    while (dv.pending_head < dv.pending.size()) run_wgrad(dv);
    if (dv.free_at > *makespan) *makespan = dv.free_at;
    busy[d] = dv.busy;
    busy_sum += dv.busy;
    peak_live[d] = dv.peak_live;
    if (peak_pending_wgrad) peak_pending_wgrad[d] = dv.peak_pending;
  }
  // share of the devices' time spent idle: 1 - sum(busy) / (P * makespan)
  if (bubble_ratio) *bubble_ratio = *makespan > 0 ? 1.0 - (double)busy_sum / ((double)s.P * (double)*makespan) : 0.0;
  return S1F_OK;
}
