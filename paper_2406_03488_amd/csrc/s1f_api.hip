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
//   dq:      QNQ, QBN keys per LDS tile, QOCC;   dk/dv: KNW waves (32 keys each), copy distance KDIST, phase lag KLAG
template <> struct Shape<bf16_t> {
  static constexpr int FNQ = 1, FKB = 1, FNW = 4, FOCC = 3, QNQ = 1, QBN = 64, QOCC = 2, KNW = 8, KDIST = 2, KLAG = 1;
};
template <> struct Shape<float> {
  static constexpr int FNQ = 1, FKB = 1, FNW = 4, FOCC = 1, QNQ = 1, QBN = 32, QOCC = 1, KNW = 4, KDIST = 1, KLAG = 0;
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

// Order of the row tiles of the forward and dQ kernels within an XCD.  Tile by tile over the XCD's heads when the
// tiles of the launch differ a lot in length (a first segment: the light tiles of every head then come last), and
// whenever query heads share K/V heads: an XCD then holds the query heads of one K/V group, and running the same
// row tile of all of them side by side makes them stream the same K/V rows through its L2 at the same time.
int row_tile_order(const s1f_desc *d, const AttnArgs &a) {
  return 2 * (int64_t)a.seg_off < (int64_t)a.seg_len || d->n_q_heads > d->n_kv_heads;
}

// One-dimensional grid of n_tiles * n_bh workgroups; the kernels decode (tile, batch*head) themselves.
// `tile_major`: order of the workgroups within an XCD; chosen per kernel from the shape of the segment.
// With `enqueue` false only the one-time preparation runs, so that a caller of several kernels can finish
// everything that may fail before the first of them is enqueued.  The status reflects this launch only (the
// return code of the launch call, not the runtime's sticky last error).
template <typename K>
int launch(K kernel, int64_t n_tiles, int64_t n_bh, int tile_major, int threads, int lds_bytes, AttnArgs a, hipStream_t st,
           bool enqueue) {
  if (n_tiles * n_bh > 0x7fffffff) return S1F_EUNSUPPORTED;
  const int rc = prepare(kernel, lds_bytes);
  if (rc != S1F_OK || !enqueue) return rc;
  a.n_tiles = (int32_t)n_tiles;
  a.n_bh = (int32_t)n_bh;
  a.tile_major = tile_major;
  void *params[] = {&a};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(kernel), dim3((unsigned)(n_tiles * n_bh)),
                                       dim3(threads), params, (size_t)lds_bytes, st);
  return e == hipSuccess ? S1F_OK : S1F_EDEVICE;
}

template <typename T, int D> int fwd_impl(const s1f_desc *d, const AttnArgs &a, hipStream_t st, bool enqueue) {
  typedef Shape<T> S;
  typedef FwdCfg<T, D, S::FNQ, S::FKB, S::FNW> Cfg;
  return launch(seg_attn_fwd_kernel<T, D, S::FNQ, S::FKB, S::FNW, S::FOCC>, (a.seg_len + Cfg::BM - 1) / Cfg::BM,
                (int64_t)d->n_q_heads * d->batch, row_tile_order(d, a), Cfg::THREADS, Cfg::LDS_BYTES, a, st, enqueue);
}

template <typename T, int D> int bwd_dq_impl(const s1f_desc *d, const AttnArgs &a, hipStream_t st, bool enqueue) {
  typedef Shape<T> S;
  typedef BwdDqCfg<T, D, S::QNQ, S::QBN> QC;
  return launch(seg_attn_bwd_dq_kernel<T, D, S::QNQ, S::QBN, S::QOCC>, (a.seg_len + QC::BM - 1) / QC::BM,
                (int64_t)d->n_q_heads * d->batch, row_tile_order(d, a), 256, QC::LDS_BYTES, a, st, enqueue);
}

template <typename T, int D> int bwd_dkdv_impl(const s1f_desc *d, const AttnArgs &a, hipStream_t st, bool enqueue) {
  typedef Shape<T> S;
  typedef BwdDkdvCfg<T, D, S::KNW, S::KDIST, S::KLAG> KC;
  const int64_t kv_len = (int64_t)a.seg_off + a.seg_len;
  return launch(seg_attn_bwd_dkdv_kernel<T, D, S::KNW, S::KDIST, S::KLAG>, (kv_len + KC::BNW - 1) / KC::BNW,
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

extern "C" int s1f_seg_attn_fwd(const s1f_desc *desc, const void *q_seg, const void *k_prefix, const void *v_prefix,
                                int64_t seg_off, int64_t seg_len, void *out, float *lse, void *hip_stream) {
  int rc = check_desc(desc);
  if (rc != S1F_OK) return rc;
  if (!q_seg || !k_prefix || !v_prefix || !out || !lse) return S1F_EINVAL;
  if (!aligned16(q_seg) || !aligned16(k_prefix) || !aligned16(v_prefix) || !aligned16(out)) return S1F_EINVAL;
  rc = check_seg(desc, seg_off, seg_len);
  if (rc != S1F_OK) return rc;
  AttnArgs a = make_args(desc, seg_off, seg_len);
  a.q = q_seg; a.k = k_prefix; a.v = v_prefix; a.out_w = out; a.lse = lse;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  S1F_DISPATCH(fwd_impl, desc, desc, a, st, true);
}

extern "C" size_t s1f_bwd_workspace_bytes(const s1f_desc *desc, int64_t seg_off, int64_t seg_len) {
  if (check_desc(desc) != S1F_OK || check_seg(desc, seg_off, seg_len) != S1F_OK) return 0;
  return 2 * (size_t)desc->batch * (size_t)desc->n_q_heads * (size_t)seg_len * sizeof(float);
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
                AttnArgs *a) {
  int rc = check_desc(desc);
  if (rc != S1F_OK) return rc;
  if (!dout || !q_seg || !k_prefix || !v_prefix || !lse || !workspace) return S1F_EINVAL;
  if (!aligned16(dout) || !aligned16(q_seg) || !aligned16(k_prefix) || !aligned16(v_prefix) || !aligned16(workspace))
    return S1F_EINVAL;
  rc = check_seg(desc, seg_off, seg_len);
  if (rc != S1F_OK) return rc;
  if (workspace_bytes < s1f_bwd_workspace_bytes(desc, seg_off, seg_len)) return S1F_EINVAL;
  // the asynchronous copies address the workspace with 32-bit byte offsets
  const int64_t stat_rows = (int64_t)desc->batch * desc->n_q_heads * seg_len;
  if (stat_rows > (int64_t(1) << 28)) return S1F_EUNSUPPORTED;
  *a = make_args(desc, seg_off, seg_len);
  a->q = q_seg; a->k = k_prefix; a->v = v_prefix; a->dout = dout;
  a->lse = const_cast<float *>(lse);
  a->delta = reinterpret_cast<float *>(const_cast<void *>(workspace));
  a->ws_plane = stat_rows;
  return S1F_OK;
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
  AttnArgs a;
  const int rc = bwd_prepare(desc, dout, q_seg, k_prefix, v_prefix, lse, seg_off, seg_len, workspace, workspace_bytes, &a);
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

// ---- the backward for callers that cannot allocate --------------------------------------------------------------
// Its row statistics live in a device array that is part of the library's code object instead of a workspace
// argument.  In host code the array's name is only a handle: its device address is looked up once per device
// (each device holds its own copy) and that address is what the kernels receive.
namespace {
constexpr int64_t kStaticStatRows = int64_t(1) << 21;            // batch * n_q_heads * seg_len the array holds
static __device__ __align__(256) float scratch[2 * kStaticStatRows];   // two planes, 16 MiB per device

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
  return s1f_seg_attn_bwd(desc, dout, q_seg, k_prefix, v_prefix, out, lse, seg_off, seg_len, dq, dk_prefix_acc,
                          dv_prefix_acc, ws, 2 * (size_t)kStaticStatRows * sizeof(float), hip_stream);
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
