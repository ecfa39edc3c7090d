// Command-line driver around the library's HOST entry points (partition variants, pass orders, pipeline timeline),
// built by tests/test_host_sanitizers.py together with their sources under AddressSanitizer and
// UndefinedBehaviorSanitizer.  Every caller-sized array is a heap vector of exactly the documented size, so a write
// past the end or an overflowing index aborts the run.  Reads commands from stdin, prints "rc value value ..." per
// command; the test compares the values with the oracle.
#include <cinttypes>
#include <cstdio>
#include <iostream>
#include <string>
#include <vector>

#include "s1f.h"

namespace {
template <typename T> T next() {
  T x;
  if (!(std::cin >> x)) std::exit(3);
  return x;
}
std::vector<int64_t> next_array(size_t n) {
  std::vector<int64_t> v(n);
  for (auto &x : v) x = next<int64_t>();
  return v;
}
void print(int rc, const std::vector<int64_t> &vals) {
  std::printf("%d", rc);
  if (rc == 0)
    for (int64_t v : vals) std::printf(" %" PRId64, v);
  std::printf("\n");
}
}  // namespace

int main() {
  std::string cmd;
  while (std::cin >> cmd) {
    if (cmd == "part" || cmd == "partex") {
      const int64_t n = next<int64_t>();
      const int32_t k = next<int32_t>(), hidden = next<int32_t>(), heads = next<int32_t>();
      std::vector<int64_t> b((size_t)(k > 0 ? k : 0) + 1);
      int rc;
      if (cmd == "part") {
        rc = s1f_partition(n, k, hidden, heads, b.data());
      } else {
        const int32_t model = next<int32_t>();
        const int64_t align = next<int64_t>();
        rc = s1f_partition_ex(n, k, hidden, heads, model, align, b.data());
      }
      print(rc, b);
    } else if (cmd == "rebal") {
      const int32_t k = next<int32_t>();
      const int64_t align = next<int64_t>();
      const std::vector<int64_t> b = next_array((size_t)k + 1), c = next_array((size_t)k);
      std::vector<int64_t> out((size_t)k + 1);
      const int rc = s1f_partition_rebalance(k, b.data(), c.data(), align, out.data());
      print(rc, out);
    } else if (cmd == "warm" || cmd == "share" || cmd == "order") {
      const int32_t P = next<int32_t>(), i = next<int32_t>(), M = next<int32_t>(), k = next<int32_t>();
      if (cmd == "warm") {
        int64_t w = -1;
        const int rc = s1f_seq1f1b_warmup(P, i, M, k, &w);
        print(rc, {w});
      } else if (cmd == "share") {
        int64_t num = -1, den = -1;
        const int rc = s1f_seq1f1b_peak_memory_share(P, i, M, k, &num, &den);
        print(rc, {num, den});
      } else {
        int64_t n_passes = -1;
        s1f_seq1f1b_order(P, i, M, k, nullptr, 0, &n_passes);   // sizing call
        std::vector<s1f_pass> order((size_t)(n_passes > 0 ? n_passes : 0));
        const int rc = s1f_seq1f1b_order(P, i, M, k, order.data(), (int64_t)order.size(), &n_passes);
        std::vector<int64_t> flat;
        for (const s1f_pass &p : order) { flat.push_back(p.backward); flat.push_back(p.micro_batch); flat.push_back(p.segment); }
        print(rc, flat);
      }
    } else if (cmd == "iwarm" || cmd == "iorder") {
      const int32_t P = next<int32_t>(), i = next<int32_t>(), M = next<int32_t>(), k = next<int32_t>(), n = next<int32_t>();
      if (cmd == "iwarm") {
        int64_t w = -1;
        const int rc = s1f_seq1f1b_interleaved_warmup(P, i, M, k, n, &w);
        print(rc, {w});
      } else {
        int64_t n_passes = -1;
        s1f_seq1f1b_interleaved_order(P, i, M, k, n, nullptr, 0, &n_passes);
        std::vector<s1f_stage_pass> order((size_t)(n_passes > 0 ? n_passes : 0));
        const int rc = s1f_seq1f1b_interleaved_order(P, i, M, k, n, order.data(), (int64_t)order.size(), &n_passes);
        std::vector<int64_t> flat;
        for (const s1f_stage_pass &p : order) {
          flat.push_back(p.kind); flat.push_back(p.micro_batch); flat.push_back(p.segment); flat.push_back(p.chunk);
        }
        print(rc, flat);
      }
    } else if (cmd == "sim") {
      s1f_pipeline_desc d = {};
      d.pp_size = next<int32_t>(); d.n_micro = next<int32_t>(); d.n_seg = next<int32_t>(); d.n_chunks = next<int32_t>();
      d.split_weight_grad = next<int32_t>(); d.max_pending_wgrad = next<int64_t>(); d.t_comm = next<int64_t>();
      const int32_t has_tokens = next<int32_t>();
      const size_t k = (size_t)(d.n_seg > 0 ? d.n_seg : 0), P = (size_t)(d.pp_size > 0 ? d.pp_size : 0);
      const std::vector<int64_t> tf = next_array(k), tb = next_array(k);
      std::vector<int64_t> tw, tok;
      if (d.split_weight_grad) tw = next_array(k);
      if (has_tokens) tok = next_array(k);
      d.t_fwd = tf.data(); d.t_bwd = tb.data();
      d.t_wgrad = d.split_weight_grad ? tw.data() : nullptr;
      d.seg_tokens = has_tokens ? tok.data() : nullptr;
      int64_t span = -1;
      double bubble = -1.0;
      std::vector<int64_t> busy(P), live(P), pend(P);
      const int rc = s1f_pipeline_simulate(&d, &span, busy.data(), live.data(), pend.data(), &bubble);
      std::vector<int64_t> flat = {span};
      flat.insert(flat.end(), busy.begin(), busy.end());
      flat.insert(flat.end(), live.begin(), live.end());
      flat.insert(flat.end(), pend.begin(), pend.end());
      std::printf("%d", rc);
      if (rc == 0) {
        for (int64_t v : flat) std::printf(" %" PRId64, v);
        std::printf(" %.17g", bubble);
      }
      std::printf("\n");
    } else {
      return 2;
    }
  }
  return 0;
}
