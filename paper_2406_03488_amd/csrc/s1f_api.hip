// C ABI of the library: argument validation and kernel dispatch.  See include/s1f.h for the contract.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdint>
#include <mutex>

#include "attn_bwd.hpp"
#include "attn_fwd.hpp"
#include "s1f.h"

namespace {
using namespace s1f;

// Tile shapes per element type: query blocks per wave (NQ), key blocks per wave (NK), keys per staged
// K/V tile (BN), rows per staged Q/dO tile (BQ).
template <typename T> struct Shape;
//   forward: FNQ query blocks per wave, FKB 32-key blocks per LDS tile, FNW waves, FOCC waves per SIMD
//   dq:      QNQ, QBN keys per LDS tile, QOCC;   dk/dv: KNW waves (32 keys each), copy distance KDIST, phase lag KLAG,
//            KWGS workgroups per compute unit
// bf16 dK/dV: two workgroups of 128 keys per compute unit, each with a two-stage tile ring.  Their barriers are
// independent, so one's vector phases, prologue and accumulator epilogue overlap the other's matrix phases; in a
// whole step this kernel measured 4 % (131072 tokens, grouped heads) to 9 % (32768 and 65536 tokens) faster than
// one workgroup of 256 keys whose upper waves run one phase late (KNW = 8, KDIST = 2, KLAG = 1, KWGS = 1).
// bf16 dQ: 32-key tiles; 64-key tiles measure the same within noise and hold twice the LDS.
template <> struct Shape<bf16_t> {
  static constexpr int FNQ = 1, FKB = 1, FNW = 4, FOCC = 3, QNQ = 1, QBN = 32, QOCC = 2, KNW = 4, KDIST = 1, KLAG = 0,
                       KWGS = 2;
};
template <> struct Shape<float> {
  static constexpr int FNQ = 1, FKB = 1, FNW = 4, FOCC = 1, QNQ = 1, QBN = 32, QOCC = 1, KNW = 4, KDIST = 1, KLAG = 0,
                       KWGS = 1;
};

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_desc(const s1f_desc *d) {
  if (d == nullptr) return S1F_EINVAL;
  if (d->batch < 1 || d->n_q_heads < 1 || d->n_kv_heads < 1 || d->n_q_heads % d->n_kv_heads != 0) return S1F_EINVAL;
  if (d->reserved != 0 || d->kv_capacity < 1) return S1F_EINVAL;
  if (d->dtype != S1F_F32 && d->dtype != S1F_BF16) return S1F_EUNSUPPORTED;
  if (d->head_dim != 64 && d->head_dim != 80 && d->head_dim != 128) return S1F_EUNSUPPORTED;
  if (d->batch > 65535 || d->n_q_heads > 65535) return S1F_EUNSUPPORTED;
  if ((int64_t)d->batch * d->n_q_heads > 0x7fffffff) return S1F_EUNSUPPORTED;   // (batch, head) pairs are counted in 32 bits
  // 16-byte vector accesses: every row must start on a 16-byte boundary
  const int64_t ce = d->dtype == S1F_BF16 ? 8 : 4;
  const int64_t s[6] = {d->q_stride_b, d->q_stride_h, d->q_stride_s, d->kv_stride_b, d->kv_stride_h, d->kv_stride_s};
  for (int i = 0; i < 6; ++i)
    if (s[i] < 0 || s[i] % ce != 0) return S1F_EINVAL;
  if (d->q_stride_s < d->head_dim || d->kv_stride_s < d->head_dim) return S1F_EINVAL;
  // the asynchronous tile copies address the rows of a tile (up to 64 rows) with 32-bit byte offsets
  if (d->q_stride_s >= (int64_t(1) << 23) || d->kv_stride_s >= (int64_t(1) << 23)) return S1F_EUNSUPPORTED;
  return S1F_OK;
}

int check_seg(const s1f_desc *d, int64_t seg_off, int64_t seg_len) {
  if (seg_off < 0 || seg_len < 1 || seg_off + seg_len > d->kv_capacity) return S1F_ERANGE;
  if (seg_off + seg_len > (int64_t(1) << 30)) return S1F_ERANGE;   // kernels index rows with 32-bit integers
  return S1F_OK;
}

AttnArgs make_args(const s1f_desc *d, int64_t seg_off, int64_t seg_len) {
  AttnArgs a = {};
  a.q_sb = d->q_stride_b; a.q_sh = d->q_stride_h; a.q_ss = d->q_stride_s;
  a.kv_sb = d->kv_stride_b; a.kv_sh = d->kv_stride_h; a.kv_ss = d->kv_stride_s;
  a.seg_off = (int32_t)seg_off; a.seg_len = (int32_t)seg_len;
  a.n_q_heads = d->n_q_heads; a.group = d->n_q_heads / d->n_kv_heads;
  a.scale = (float)(1.0 / std::sqrt((double)d->head_dim));
  return a;
}

// Kernels that need more than 64 KiB of LDS have to be told so once per device; `prepare` does that the first time
// a kernel instantiation is used on the current device (a template: one flag set per instantiation).
constexpr int kMaxDevices = 64;
template <typename K> int prepare(K kernel, int lds_bytes) {
  if (lds_bytes <= 64 * 1024) return S1F_OK;
  static std::atomic<bool> done[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess) return S1F_EDEVICE;
  const bool cached = dev >= 0 && dev < kMaxDevices;
  if (cached && done[dev].load(std::memory_order_acquire)) return S1F_OK;
  if (hipFuncSetAttribute(reinterpret_cast<const void *>(kernel), hipFuncAttributeMaxDynamicSharedMemorySize,
                          lds_bytes) != hipSuccess)
    return S1F_EDEVICE;
  if (cached) done[dev].store(true, std::memory_order_release);
  return S1F_OK;
}

// Order of the row tiles of the forward and dQ kernels within an XCD.  Tile by tile over the XCD's heads whenever
// query heads share K/V heads: an XCD then holds the query heads of one K/V group, and running the same row tile of
// all of them side by side makes them stream the same K/V rows through its L2 at the same time.  Otherwise head by
// head (all row tiles of a head side by side share its K/V rows), except for a SHORT launch whose tiles differ a lot
// in length (a first segment of a few rounds of workgroups): tile by tile the light tiles of every head then come
// last and fill the end of the launch.  A long first segment (many rounds: one unsegmented pass over 65536 tokens
// and 56 heads measured 11 % faster in the forward, 9 % in the dQ kernel) stays head by head.
constexpr int64_t kTileMajorMaxUnits = 6144;   // about eight rounds of row tiles
int row_tile_order(const s1f_desc *d, const AttnArgs &a) {
  if (d->n_q_heads > d->n_kv_heads) return 1;
  const int64_t units = (((int64_t)a.seg_len + 127) / 128) * d->n_q_heads * d->batch;
  return 2 * (int64_t)a.seg_off < (int64_t)a.seg_len && units <= kTileMajorMaxUnits;
}

// Key-split of the last units of a launch (see split_unit in attn_device.hpp).  A launch of `units` equal-sized
// units runs in rounds of `slots` (the workgroups the chip holds at once); its last round holds only r = units mod
// slots of them and still lasts as long as a full one.  Cutting each of those r units into n chunks turns that round
// into ceil(r n / slots) rounds of 1/n the length; n (at most kMaxSplit, chunks at least kMinChunkKeys keys long,
// partial results within `cap` bytes) is chosen to minimise that plus what the chunks cost: their own start-up and
// the merge kernel, which reads every partial result once, both measured against the time a whole unit takes
// (its keys times the kernel's time per key).  Deterministic in (shape, device, cap): the workspace-size queries
// and the launches derive the same plan.
constexpr int kMaxSplit = kMaxChunks;
constexpr int64_t kMinChunkKeys = 256;
constexpr int64_t kMaxPartBytes = int64_t(512) << 20;      // partial results of one launch with a caller's workspace
constexpr int64_t kStaticPartBytes = int64_t(32) << 20;    // ... with the library's built-in scratch
constexpr double kChunkStartup = 0.004;                    // a chunk's prologue and epilogue, in whole-unit times
constexpr double kMergeSeconds = 12e-6, kMergeBytesPerSecond = 2.5e12;   // the merge kernel: fixed part, read rate
constexpr double kFwdSecondsPerKey = 0.035e-6, kDqSecondsPerKey = 0.05e-6;   // a 128-row tile against one key
struct SplitPlan {
  int64_t n_whole = 0;        // leading workgroup ids that are whole units
  int64_t n_split_units = 0;  // units cut into chunks
  int n_split = 1;            // chunks per split unit
  int64_t grid() const { return n_whole + n_split_units * n_split; }
};

SplitPlan plan_split(int64_t units, int slots, int64_t seg_off, double unit_seconds, int64_t part_bytes_per_chunk,
                     int64_t cap) {
  SplitPlan p;
  p.n_whole = units;
  if (slots <= 0 || units <= 0 || unit_seconds <= 0) return p;
  const int64_t r = units % slots;
  if (r == 0) return p;
  int best = 1;
  double best_t = 1.0;   // length of the last round in units of a whole unit's time
  for (int n = 2; n <= kMaxSplit; ++n) {
    if (n > seg_off / kMinChunkKeys || r * n * part_bytes_per_chunk > cap) break;
    const double merge = (kMergeSeconds + (double)(r * n * part_bytes_per_chunk) / kMergeBytesPerSecond) / unit_seconds;
    const double t = (double)((r * n + slots - 1) / slots) / n + kChunkStartup * n + merge;
    if (t < best_t - 1e-9) { best = n; best_t = t; }
  }
  if (best_t > 0.95) return p;   // not worth a second kernel
  p.n_whole = units - r;
  p.n_split_units = r;
  p.n_split = best;
  return p;
}

// Workgroups of `kernel` that the current device holds at once (0 if that cannot be found out, e.g. without a
// device: launches are then never split).  Looked up once per kernel instantiation and device.
template <typename K> int resident_workgroups(K kernel, int threads, int lds_bytes) {
  static std::atomic<int> cached[kMaxDevices];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) {
    (void)hipGetLastError();
    return 0;
  }
  int n = cached[dev].load(std::memory_order_acquire);
  if (n > 0) return n;
  int per_cu = 0, cus = 0;
  if (prepare(kernel, lds_bytes) != S1F_OK ||
      hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, reinterpret_cast<const void *>(kernel), threads,
                                                   (size_t)lds_bytes) != hipSuccess ||
      hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) {
    (void)hipGetLastError();
    return 0;
  }
  n = per_cu * cus;
  if (n > 0) cached[dev].store(n, std::memory_order_release);
  return n;
}

// One-dimensional grid; the kernels decode (unit -> tile, batch*head; chunk) themselves.
// `tile_major`: order of the workgroups within an XCD; chosen per kernel from the shape of the segment.
// With `enqueue` false only the one-time preparation runs, so that a caller of several kernels can finish
// everything that may fail before the first of them is enqueued.  The status reflects this launch only (the
// return code of the launch call, not the runtime's sticky last error).
template <typename K>
int launch(K kernel, int64_t n_tiles, int64_t n_bh, int tile_major, int threads, int lds_bytes, AttnArgs a, hipStream_t st,
           bool enqueue, const SplitPlan *plan = nullptr) {
  if (n_tiles * n_bh > 0x7fffffff) return S1F_EUNSUPPORTED;
  const int rc = prepare(kernel, lds_bytes);
  if (rc != S1F_OK || !enqueue) return rc;
  a.n_tiles = (int32_t)n_tiles;
  a.n_bh = (int32_t)n_bh;
  a.tile_major = tile_major;
  a.n_whole = (int32_t)(plan ? plan->n_whole : n_tiles * n_bh);
  a.n_split = plan ? plan->n_split : 1;
  a.n_split_units = (int32_t)(plan ? plan->n_split_units : 0);
  const int64_t grid = plan ? plan->grid() : n_tiles * n_bh;
  void *params[] = {&a};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3((unsigned)grid), dim3(threads), params,
                                       (size_t)lds_bytes, st);
  return e == hipSuccess ? S1F_OK : S1F_EDEVICE;
}

// The merge kernel behind a split launch: `groups` workgroups (of a few rows each) per split unit.
template <typename K> int launch_merge(K kernel, AttnArgs a, const SplitPlan &plan, int groups, hipStream_t st) {
  void *params[] = {&a};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3((unsigned)(plan.n_split_units * groups)),
                                       dim3(256), params, 0, st);
  return e == hipSuccess ? S1F_OK : S1F_EDEVICE;
}

inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

// ---- forward ----
template <typename T, int D> struct FwdLaunch {
  typedef Shape<T> S;
  typedef FwdCfg<T, D, S::FNQ, S::FKB, S::FNW> Cfg;
  static constexpr int64_t kPartBytes = (int64_t)Cfg::BM * D * 4, kMlBytes = (int64_t)Cfg::BM * 2 * 4;
  static auto kernel() { return seg_attn_fwd_kernel<T, D, S::FNQ, S::FKB, S::FNW, S::FOCC>; }
  static int64_t tiles(int64_t seg_len) { return (seg_len + Cfg::BM - 1) / Cfg::BM; }
  // `split`: the caller brought a workspace (only the bf16 kernels split; fp32 is the reference-precision mode)
  static SplitPlan plan(const s1f_desc *d, int64_t seg_off, int64_t seg_len, bool split) {
    const int64_t units = tiles(seg_len) * d->n_q_heads * d->batch;
    if (!split || sizeof(T) != 2) return plan_split(units, 0, 0, 0, 0, 0);
    return plan_split(units, resident_workgroups(kernel(), Cfg::THREADS, Cfg::LDS_BYTES), seg_off,
                      kFwdSecondsPerKey * (double)(seg_off + seg_len / 2), kPartBytes + kMlBytes, kMaxPartBytes);
  }
  static size_t workspace_bytes(const SplitPlan &p) {
    const int64_t chunks = p.n_split_units * p.n_split;
    return chunks == 0 ? 0 : align256((size_t)(chunks * kPartBytes)) + (size_t)(chunks * kMlBytes);
  }
};

template <typename T, int D>
int fwd_impl(const s1f_desc *d, AttnArgs a, hipStream_t st, void *workspace, size_t workspace_bytes, bool split) {
  typedef FwdLaunch<T, D> L;
  const SplitPlan p = L::plan(d, a.seg_off, a.seg_len, split);
  if (L::workspace_bytes(p) > workspace_bytes) return S1F_EINVAL;
  const int64_t chunks = p.n_split_units * p.n_split;
  a.part = reinterpret_cast<float *>(workspace);
  a.part_ml = reinterpret_cast<float *>(reinterpret_cast<char *>(workspace) + align256((size_t)(chunks * L::kPartBytes)));
  const int64_t n_bh = (int64_t)d->n_q_heads * d->batch;
  const int order = row_tile_order(d, a);
  int rc = launch(L::kernel(), L::tiles(a.seg_len), n_bh, order, L::Cfg::THREADS, L::Cfg::LDS_BYTES, a, st, true, &p);
  if (rc != S1F_OK || chunks == 0) return rc;
  a.n_tiles = (int32_t)L::tiles(a.seg_len); a.n_bh = (int32_t)n_bh; a.tile_major = order;
  a.n_whole = (int32_t)p.n_whole; a.n_split = p.n_split; a.n_split_units = (int32_t)p.n_split_units;
  return launch_merge(seg_attn_fwd_merge_kernel<T, D, L::Cfg::BM>, a, p, MergeRows<D>::groups(L::Cfg::BM), st);
}
template <typename T, int D> size_t fwd_ws_impl(const s1f_desc *d, int64_t seg_off, int64_t seg_len) {
  return FwdLaunch<T, D>::workspace_bytes(FwdLaunch<T, D>::plan(d, seg_off, seg_len, true));
}

// ---- backward ----
// Workspace: the two planes of row statistics, then (256-byte aligned) the partial dQ rows of a split dQ launch.
template <typename T, int D> struct DqLaunch {
  typedef Shape<T> S;
  typedef BwdDqCfg<T, D, S::QNQ, S::QBN> QC;
  static constexpr int64_t kPartBytes = (int64_t)QC::BM * D * 4;
  static auto kernel() { return seg_attn_bwd_dq_kernel<T, D, S::QNQ, S::QBN, S::QOCC>; }
  static int64_t tiles(int64_t seg_len) { return (seg_len + QC::BM - 1) / QC::BM; }
  static SplitPlan plan(const s1f_desc *d, int64_t seg_off, int64_t seg_len, int64_t cap) {
    const int64_t units = tiles(seg_len) * d->n_q_heads * d->batch;
    if (sizeof(T) != 2) return plan_split(units, 0, 0, 0, 0, 0);
    return plan_split(units, resident_workgroups(kernel(), 256, QC::LDS_BYTES), seg_off,
                      kDqSecondsPerKey * (double)(seg_off + seg_len / 2), kPartBytes, cap);
  }
};
inline size_t stat_bytes(const s1f_desc *d, int64_t seg_len) {
  return align256(2 * (size_t)d->batch * (size_t)d->n_q_heads * (size_t)seg_len * sizeof(float));
}
template <typename T, int D> size_t bwd_ws_impl(const s1f_desc *d, int64_t seg_off, int64_t seg_len, int64_t cap) {
  const SplitPlan p = DqLaunch<T, D>::plan(d, seg_off, seg_len, cap);
  return stat_bytes(d, seg_len) + (size_t)(p.n_split_units * p.n_split * DqLaunch<T, D>::kPartBytes);
}

template <typename T, int D> int bwd_dq_impl(const s1f_desc *d, AttnArgs a, hipStream_t st, bool enqueue) {
  typedef DqLaunch<T, D> L;
  const SplitPlan p = L::plan(d, a.seg_off, a.seg_len, a.part_cap);
  a.part = reinterpret_cast<float *>(reinterpret_cast<char *>(a.delta) + stat_bytes(d, a.seg_len));
  const int64_t n_bh = (int64_t)d->n_q_heads * d->batch;
  const int order = row_tile_order(d, a);
  int rc = launch(L::kernel(), L::tiles(a.seg_len), n_bh, order, 256, L::QC::LDS_BYTES, a, st, enqueue, &p);
  if (rc != S1F_OK || !enqueue || p.n_split_units == 0) return rc;
  a.n_tiles = (int32_t)L::tiles(a.seg_len); a.n_bh = (int32_t)n_bh; a.tile_major = order;
  a.n_whole = (int32_t)p.n_whole; a.n_split = p.n_split; a.n_split_units = (int32_t)p.n_split_units;
  return launch_merge(seg_attn_bwd_dq_merge_kernel<T, D, L::QC::BM>, a, p, MergeRows<D>::groups(L::QC::BM), st);
}

template <typename T, int D> int bwd_dkdv_impl(const s1f_desc *d, const AttnArgs &a, hipStream_t st, bool enqueue) {
  typedef Shape<T> S;
  typedef BwdDkdvCfg<T, D, S::KNW, S::KDIST, S::KLAG> KC;
  const int64_t kv_len = (int64_t)a.seg_off + a.seg_len;
  return launch(seg_attn_bwd_dkdv_kernel<T, D, S::KNW, S::KDIST, S::KLAG, S::KWGS>, (kv_len + KC::BNW - 1) / KC::BNW,
                (int64_t)d->n_kv_heads * d->batch, 2 * (int64_t)a.seg_off < (int64_t)a.seg_len, KC::THREADS, KC::LDS_BYTES,
                a, st, enqueue);
}


#define S1F_DISPATCH(fn, d, ...)                                                        \
  do {                                                                                  \
    if ((d)->dtype == S1F_BF16) {                                                       \
      switch ((d)->head_dim) {                                                          \
        case 64: return fn<bf16_t, 64>(__VA_ARGS__);                                    \
        case 80: return fn<bf16_t, 80>(__VA_ARGS__);                                    \
        case 128: return fn<bf16_t, 128>(__VA_ARGS__);                                  \
      }                                                                                 \
    } else {                                                                            \
      switch ((d)->head_dim) {                                                          \
        case 64: return fn<float, 64>(__VA_ARGS__);                                     \
        case 80: return fn<float, 80>(__VA_ARGS__);                                     \
        case 128: return fn<float, 128>(__VA_ARGS__);                                   \
      }                                                                                 \
    }                                                                                   \
    return S1F_EUNSUPPORTED;                                                            \
  } while (0)

}  // namespace

namespace {
int fwd_entry(const s1f_desc *desc, const void *q_seg, const void *k_prefix, const void *v_prefix, int64_t seg_off,
              int64_t seg_len, void *out, float *lse, void *workspace, size_t workspace_bytes, bool split,
              void *hip_stream) {
  int rc = check_desc(desc);
  if (rc != S1F_OK) return rc;
  if (!q_seg || !k_prefix || !v_prefix || !out || !lse) return S1F_EINVAL;
  if (!aligned16(q_seg) || !aligned16(k_prefix) || !aligned16(v_prefix) || !aligned16(out)) return S1F_EINVAL;
  if (workspace_bytes > 0 && (!workspace || !aligned16(workspace))) return S1F_EINVAL;
  rc = check_seg(desc, seg_off, seg_len);
  if (rc != S1F_OK) return rc;
  AttnArgs a = make_args(desc, seg_off, seg_len);
  a.q = q_seg; a.k = k_prefix; a.v = v_prefix; a.out_w = out; a.lse = lse;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  S1F_DISPATCH(fwd_impl, desc, desc, a, st, workspace, workspace_bytes, split);
}
// (callers have validated the descriptor: the dispatch below always finds its kernel)
size_t fwd_ws_dispatch(const s1f_desc *d, int64_t seg_off, int64_t seg_len) {
  if (d->dtype != S1F_BF16) return 0;   // fp32 launches are never split
  switch (d->head_dim) {
    case 64: return fwd_ws_impl<bf16_t, 64>(d, seg_off, seg_len);
    case 80: return fwd_ws_impl<bf16_t, 80>(d, seg_off, seg_len);
    case 128: return fwd_ws_impl<bf16_t, 128>(d, seg_off, seg_len);
  }
  return 0;
}
size_t bwd_ws_dispatch(const s1f_desc *d, int64_t seg_off, int64_t seg_len, int64_t cap) {
  if (d->dtype != S1F_BF16) return stat_bytes(d, seg_len);
  switch (d->head_dim) {
    case 64: return bwd_ws_impl<bf16_t, 64>(d, seg_off, seg_len, cap);
    case 80: return bwd_ws_impl<bf16_t, 80>(d, seg_off, seg_len, cap);
    case 128: return bwd_ws_impl<bf16_t, 128>(d, seg_off, seg_len, cap);
  }
  return stat_bytes(d, seg_len);
}
}  // namespace

extern "C" int s1f_seg_attn_fwd(const s1f_desc *desc, const void *q_seg, const void *k_prefix, const void *v_prefix,
                                int64_t seg_off, int64_t seg_len, void *out, float *lse, void *hip_stream) {
  return fwd_entry(desc, q_seg, k_prefix, v_prefix, seg_off, seg_len, out, lse, nullptr, 0, false, hip_stream);
}

extern "C" size_t s1f_fwd_workspace_bytes(const s1f_desc *desc, int64_t seg_off, int64_t seg_len) {
  if (check_desc(desc) != S1F_OK || check_seg(desc, seg_off, seg_len) != S1F_OK) return 0;
  return fwd_ws_dispatch(desc, seg_off, seg_len);
}

extern "C" int s1f_seg_attn_fwd_ws(const s1f_desc *desc, const void *q_seg, const void *k_prefix, const void *v_prefix,
                                   int64_t seg_off, int64_t seg_len, void *out, float *lse, void *workspace,
                                   size_t workspace_bytes, void *hip_stream) {
  return fwd_entry(desc, q_seg, k_prefix, v_prefix, seg_off, seg_len, out, lse, workspace, workspace_bytes, true, hip_stream);
}

extern "C" size_t s1f_bwd_workspace_bytes(const s1f_desc *desc, int64_t seg_off, int64_t seg_len) {
  if (check_desc(desc) != S1F_OK || check_seg(desc, seg_off, seg_len) != S1F_OK) return 0;
  return bwd_ws_dispatch(desc, seg_off, seg_len, kMaxPartBytes);
}

namespace {
int bwd_dq_dispatch(const s1f_desc *d, const AttnArgs &a, hipStream_t st, bool enqueue) {
  S1F_DISPATCH(bwd_dq_impl, d, d, a, st, enqueue);
}
int bwd_dkdv_dispatch(const s1f_desc *d, const AttnArgs &a, hipStream_t st, bool enqueue) {
  S1F_DISPATCH(bwd_dkdv_impl, d, d, a, st, enqueue);
}

// Validation shared by the backward entry points; fills `a` on success.
int bwd_prepare(const s1f_desc *desc, const void *dout, const void *q_seg, const void *k_prefix, const void *v_prefix,
                const float *lse, int64_t seg_off, int64_t seg_len, const void *workspace, size_t workspace_bytes,
                AttnArgs *a, int64_t part_cap = kMaxPartBytes) {
  int rc = check_desc(desc);
  if (rc != S1F_OK) return rc;
  if (!dout || !q_seg || !k_prefix || !v_prefix || !lse || !workspace) return S1F_EINVAL;
  if (!aligned16(dout) || !aligned16(q_seg) || !aligned16(k_prefix) || !aligned16(v_prefix) || !aligned16(workspace))
    return S1F_EINVAL;
  rc = check_seg(desc, seg_off, seg_len);
  if (rc != S1F_OK) return rc;
  if (workspace_bytes < bwd_ws_dispatch(desc, seg_off, seg_len, part_cap)) return S1F_EINVAL;
  // the asynchronous copies address the workspace with 32-bit byte offsets
  const int64_t stat_rows = (int64_t)desc->batch * desc->n_q_heads * seg_len;
  if (stat_rows > (int64_t(1) << 28)) return S1F_EUNSUPPORTED;
  *a = make_args(desc, seg_off, seg_len);
  a->q = q_seg; a->k = k_prefix; a->v = v_prefix; a->dout = dout;
  a->lse = const_cast<float *>(lse);
  a->delta = reinterpret_cast<float *>(const_cast<void *>(workspace));
  a->ws_plane = stat_rows;
  a->part_cap = part_cap;
  return S1F_OK;
}

// s1f_seg_attn_bwd; `part_cap` bounds the partial dQ rows a split dQ launch may leave behind the statistics.
int bwd_entry(const s1f_desc *desc, const void *dout, const void *q_seg, const void *k_prefix, const void *v_prefix,
              const void *out, const float *lse, int64_t seg_off, int64_t seg_len, void *dq, float *dk_prefix_acc,
              float *dv_prefix_acc, void *workspace, size_t workspace_bytes, int64_t part_cap, void *hip_stream) {
  AttnArgs a;
  const int rc = bwd_prepare(desc, dout, q_seg, k_prefix, v_prefix, lse, seg_off, seg_len, workspace, workspace_bytes, &a,
                             part_cap);
  if (rc != S1F_OK) return rc;
  if (!out || !dq || !dk_prefix_acc || !dv_prefix_acc) return S1F_EINVAL;
  if (!aligned16(out) || !aligned16(dq) || !aligned16(dk_prefix_acc) || !aligned16(dv_prefix_acc)) return S1F_EINVAL;
  a.out = out; a.dq = dq; a.dk_acc = dk_prefix_acc; a.dv_acc = dv_prefix_acc;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  // everything that can fail short of the launches themselves happens before the first kernel is enqueued
  int rc2 = bwd_dq_dispatch(desc, a, st, false);
  if (rc2 == S1F_OK) rc2 = bwd_dkdv_dispatch(desc, a, st, false);
  if (rc2 != S1F_OK) return rc2;
  rc2 = bwd_dq_dispatch(desc, a, st, true);
  if (rc2 != S1F_OK) return rc2;
  return bwd_dkdv_dispatch(desc, a, st, true);
}
}  // namespace

extern "C" int s1f_seg_attn_bwd_dq(const s1f_desc *desc, const void *dout, const void *q_seg, const void *k_prefix,
                                   const void *v_prefix, const void *out, const float *lse, int64_t seg_off,
                                   int64_t seg_len, void *dq, void *workspace, size_t workspace_bytes,
                                   void *hip_stream) {
  AttnArgs a;
  const int rc = bwd_prepare(desc, dout, q_seg, k_prefix, v_prefix, lse, seg_off, seg_len, workspace, workspace_bytes, &a);
  if (rc != S1F_OK) return rc;
  if (!out || !dq || !aligned16(out) || !aligned16(dq)) return S1F_EINVAL;
  a.out = out; a.dq = dq;
  return bwd_dq_dispatch(desc, a, reinterpret_cast<hipStream_t>(hip_stream), true);
}

extern "C" int s1f_seg_attn_bwd_dkdv(const s1f_desc *desc, const void *dout, const void *q_seg, const void *k_prefix,
                                     const void *v_prefix, const float *lse, int64_t seg_off, int64_t seg_len,
                                     float *dk_prefix_acc, float *dv_prefix_acc, const void *workspace,
                                     size_t workspace_bytes, void *hip_stream) {
  AttnArgs a;
  const int rc = bwd_prepare(desc, dout, q_seg, k_prefix, v_prefix, lse, seg_off, seg_len, workspace, workspace_bytes, &a);
  if (rc != S1F_OK) return rc;
  if (!dk_prefix_acc || !dv_prefix_acc || !aligned16(dk_prefix_acc) || !aligned16(dv_prefix_acc)) return S1F_EINVAL;
  a.dk_acc = dk_prefix_acc; a.dv_acc = dv_prefix_acc;
  return bwd_dkdv_dispatch(desc, a, reinterpret_cast<hipStream_t>(hip_stream), true);
}

extern "C" int s1f_seg_attn_bwd(const s1f_desc *desc, const void *dout, const void *q_seg, const void *k_prefix,
                                const void *v_prefix, const void *out, const float *lse, int64_t seg_off,
                                int64_t seg_len, void *dq, float *dk_prefix_acc, float *dv_prefix_acc,
                                void *workspace, size_t workspace_bytes, void *hip_stream) {
  return bwd_entry(desc, dout, q_seg, k_prefix, v_prefix, out, lse, seg_off, seg_len, dq, dk_prefix_acc, dv_prefix_acc,
                   workspace, workspace_bytes, kMaxPartBytes, hip_stream);
}

// ---- the backward for callers that cannot allocate --------------------------------------------------------------
// Its row statistics live in a device array that is part of the library's code object instead of a workspace
// argument.  In host code the array's name is only a handle: its device address is looked up once per device
// (each device holds its own copy) and that address is what the kernels receive.
namespace {
constexpr int64_t kStaticStatRows = int64_t(1) << 21;            // batch * n_q_heads * seg_len the array holds
// two planes of row statistics (16 MiB), then the partial dQ rows of a split dQ launch (at most kStaticPartBytes)
constexpr size_t kStaticScratchBytes = 2 * (size_t)kStaticStatRows * sizeof(float) + (size_t)kStaticPartBytes;
static __device__ __align__(256) float scratch[kStaticScratchBytes / sizeof(float)];

std::mutex scratch_mutex;
float *scratch_ptr[kMaxDevices];   // device address of `scratch` on each device, null until looked up

int static_scratch(float **out) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return S1F_EDEVICE;
  std::lock_guard<std::mutex> lock(scratch_mutex);
  if (scratch_ptr[dev] == nullptr) {
    void *p = nullptr;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || p == nullptr) return S1F_EDEVICE;
    scratch_ptr[dev] = static_cast<float *>(p);
  }
  *out = scratch_ptr[dev];
  return S1F_OK;
}
}  // namespace

extern "C" size_t s1f_static_scratch_rows(void) { return (size_t)kStaticStatRows; }

extern "C" int s1f_seg_attn_bwd_noalloc(const s1f_desc *desc, const void *dout, const void *q_seg, const void *k_prefix,
                                        const void *v_prefix, const void *out, const float *lse, int64_t seg_off,
                                        int64_t seg_len, void *dq, float *dk_prefix_acc, float *dv_prefix_acc,
                                        void *hip_stream) {
  int rc = check_desc(desc);
  if (rc != S1F_OK) return rc;
  rc = check_seg(desc, seg_off, seg_len);
  if (rc != S1F_OK) return rc;
  if ((int64_t)desc->batch * desc->n_q_heads * seg_len > kStaticStatRows) return S1F_ESCRATCH;
  float *ws = nullptr;
  rc = static_scratch(&ws);
  if (rc != S1F_OK) return rc;
  // every plane entry the dK/dV kernel reads is written by the dQ kernel of the same call: nothing to clear
  return bwd_entry(desc, dout, q_seg, k_prefix, v_prefix, out, lse, seg_off, seg_len, dq, dk_prefix_acc, dv_prefix_acc, ws,
                   kStaticScratchBytes, kStaticPartBytes, hip_stream);
}

extern "C" const char *s1f_strerror(int status) {
  switch (status) {
    case S1F_OK: return "ok";
    case S1F_EINVAL: return "invalid argument (null or misaligned pointer, bad size or stride, workspace too small)";
    case S1F_EUNSUPPORTED: return "unsupported dtype or head_dim (supported: f32/bf16 with head_dim 64, 80, 128)";
    case S1F_ERANGE: return "segment out of range (seg_off < 0, seg_len < 1 or seg_off + seg_len > kv_capacity)";
    case S1F_EDEVICE: return "HIP runtime error at kernel launch";
    case S1F_ESCRATCH:
      return "batch * n_q_heads * seg_len exceeds the built-in scratch of s1f_seg_attn_bwd_noalloc "
             "(s1f_static_scratch_rows); use s1f_seg_attn_bwd with a workspace";
    default: return "unknown status";
  }
}

extern "C" int s1f_version(void) { return 200; }
