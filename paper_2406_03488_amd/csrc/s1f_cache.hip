// The two steps on either side of the attention calls of one segment (Section 3.2): appending the segment's
// new K/V rows to the prefix cache before its forward pass, and, after its backward pass, emitting the rows
// of the fp32 dK/dV accumulators that have become final (rows of segment i receive no further contribution
// once the backward passes of segments k .. i have run) in the tensors' element type for the backward of
// the projection that produced K and V.  Pure data movement: bound by HBM bandwidth.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "attn_device.hpp"
#include "s1f.h"

namespace s1f {
namespace {

struct CopyArgs {
  const void *src0, *src1;
  void *dst0, *dst1;
  int64_t src_sb, src_sh, src_ss, dst_sb, dst_sh, dst_ss;   // elements of the respective tensor (sb: host side only)
  int32_t rows, heads, chunks;                               // chunks of 8 elements per row
};

// One thread moves 8 consecutive head_dim elements of one row of both tensors of one batch entry.
// SRC/DST: element types (float or bf16_t); float -> bf16 rounds to nearest even.
template <typename SRC, typename DST> __global__ void __launch_bounds__(256) rows_kernel(const CopyArgs a) {
  const int64_t id = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int64_t per_head = (int64_t)a.rows * a.chunks;
  if (id >= per_head * a.heads) return;
  const int h = (int)(id / per_head);
  const int64_t rem = id % per_head;
  const int r = (int)(rem / a.chunks), c = (int)(rem % a.chunks);
  const int64_t so = h * a.src_sh + (int64_t)r * a.src_ss + 8 * c;
  const int64_t dof = h * a.dst_sh + (int64_t)r * a.dst_ss + 8 * c;
#pragma unroll
  for (int t = 0; t < 2; ++t) {
    const SRC *s = reinterpret_cast<const SRC *>(t ? a.src1 : a.src0) + so;
    DST *d = reinterpret_cast<DST *>(t ? a.dst1 : a.dst0) + dof;
    if (sizeof(SRC) == sizeof(DST)) {
      if (sizeof(SRC) == 2) {
        *reinterpret_cast<u32x4 *>(d) = *reinterpret_cast<const u32x4 *>(s);
      } else {
        reinterpret_cast<u32x4 *>(d)[0] = reinterpret_cast<const u32x4 *>(s)[0];
        reinterpret_cast<u32x4 *>(d)[1] = reinterpret_cast<const u32x4 *>(s)[1];
      }
    } else {   // fp32 -> bf16
      const f32x4 x = reinterpret_cast<const f32x4 *>(s)[0], y = reinterpret_cast<const f32x4 *>(s)[1];
      bf16x8 o;
#pragma unroll
      for (int e = 0; e < 4; ++e) { o[e] = (bf16_t)x[e]; o[4 + e] = (bf16_t)y[e]; }
      *reinterpret_cast<bf16x8 *>(d) = o;
    }
  }
}

template <typename SRC, typename DST> int launch_rows(const CopyArgs &a, hipStream_t st) {
  const int64_t total = (int64_t)a.heads * a.rows * a.chunks;
  const int64_t blocks = (total + 255) / 256;
  if (blocks > 0x7fffffff) return S1F_EUNSUPPORTED;
  CopyArgs args = a;
  void *params[] = {&args};
  const hipError_t e = hipLaunchKernel(reinterpret_cast<const void *>(&rows_kernel<SRC, DST>), dim3((unsigned)blocks),
                                       dim3(256), params, 0, st);
  return e == hipSuccess ? S1F_OK : S1F_EDEVICE;
}

bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15) == 0; }

int check(const s1f_desc *d, int64_t seg_off, int64_t seg_len, int64_t sb, int64_t sh, int64_t ss) {
  if (!d) return S1F_EINVAL;
  if (d->batch < 1 || d->n_kv_heads < 1 || d->reserved != 0) return S1F_EINVAL;
  if (d->dtype != S1F_F32 && d->dtype != S1F_BF16) return S1F_EUNSUPPORTED;
  if (d->head_dim < 8 || d->head_dim % 8 != 0) return S1F_EUNSUPPORTED;
  if (d->kv_stride_s < d->head_dim || ss < d->head_dim) return S1F_EINVAL;
  if ((d->kv_stride_b | d->kv_stride_h | d->kv_stride_s | sb | sh | ss) % 8 != 0) return S1F_EINVAL;
  if (seg_off < 0 || seg_len < 1 || seg_off + seg_len > d->kv_capacity) return S1F_ERANGE;
  if (seg_len > (int64_t(1) << 30)) return S1F_ERANGE;
  return S1F_OK;
}

}  // namespace
}  // namespace s1f

using namespace s1f;

extern "C" int s1f_kv_append(const s1f_desc *desc, const void *k_seg, const void *v_seg, int64_t seg_stride_b,
                             int64_t seg_stride_h, int64_t seg_stride_s, int64_t seg_off, int64_t seg_len,
                             void *k_cache, void *v_cache, void *hip_stream) {
  const int rc = check(desc, seg_off, seg_len, seg_stride_b, seg_stride_h, seg_stride_s);
  if (rc != S1F_OK) return rc;
  if (!k_seg || !v_seg || !k_cache || !v_cache) return S1F_EINVAL;
  if (!aligned16(k_seg) || !aligned16(v_seg) || !aligned16(k_cache) || !aligned16(v_cache)) return S1F_EINVAL;
  const int64_t esz = desc->dtype == S1F_BF16 ? 2 : 4;
  CopyArgs a = {};
  a.src0 = k_seg; a.src1 = v_seg;
  a.dst0 = reinterpret_cast<char *>(k_cache) + seg_off * desc->kv_stride_s * esz;
  a.dst1 = reinterpret_cast<char *>(v_cache) + seg_off * desc->kv_stride_s * esz;
  a.src_sb = seg_stride_b; a.src_sh = seg_stride_h; a.src_ss = seg_stride_s;
  a.dst_sb = desc->kv_stride_b; a.dst_sh = desc->kv_stride_h; a.dst_ss = desc->kv_stride_s;
  a.rows = (int32_t)seg_len; a.heads = desc->n_kv_heads; a.chunks = desc->head_dim / 8;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  for (int b = 0; b < desc->batch; ++b) {   // one launch per batch entry (the workloads have one)
    CopyArgs ab = a;
    ab.src0 = reinterpret_cast<const char *>(a.src0) + b * a.src_sb * esz;
    ab.src1 = reinterpret_cast<const char *>(a.src1) + b * a.src_sb * esz;
    ab.dst0 = reinterpret_cast<char *>(a.dst0) + b * a.dst_sb * esz;
    ab.dst1 = reinterpret_cast<char *>(a.dst1) + b * a.dst_sb * esz;
    const int r = desc->dtype == S1F_BF16 ? launch_rows<bf16_t, bf16_t>(ab, st) : launch_rows<float, float>(ab, st);
    if (r != S1F_OK) return r;
  }
  return S1F_OK;
}

extern "C" int s1f_kv_grad_emit(const s1f_desc *desc, const float *dk_prefix_acc, const float *dv_prefix_acc,
                                int64_t seg_off, int64_t seg_len, void *dk_seg, void *dv_seg, int64_t seg_stride_b,
                                int64_t seg_stride_h, int64_t seg_stride_s, void *hip_stream) {
  const int rc = check(desc, seg_off, seg_len, seg_stride_b, seg_stride_h, seg_stride_s);
  if (rc != S1F_OK) return rc;
  if (!dk_prefix_acc || !dv_prefix_acc || !dk_seg || !dv_seg) return S1F_EINVAL;
  if (!aligned16(dk_prefix_acc) || !aligned16(dv_prefix_acc) || !aligned16(dk_seg) || !aligned16(dv_seg)) return S1F_EINVAL;
  const int64_t esz = desc->dtype == S1F_BF16 ? 2 : 4;
  CopyArgs a = {};
  a.src_sb = desc->kv_stride_b; a.src_sh = desc->kv_stride_h; a.src_ss = desc->kv_stride_s;
  a.dst_sb = seg_stride_b; a.dst_sh = seg_stride_h; a.dst_ss = seg_stride_s;
  a.rows = (int32_t)seg_len; a.heads = desc->n_kv_heads; a.chunks = desc->head_dim / 8;
  hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
  for (int b = 0; b < desc->batch; ++b) {   // one launch per batch entry
    CopyArgs ab = a;
    ab.src0 = dk_prefix_acc + seg_off * desc->kv_stride_s + b * a.src_sb;
    ab.src1 = dv_prefix_acc + seg_off * desc->kv_stride_s + b * a.src_sb;
    ab.dst0 = reinterpret_cast<char *>(dk_seg) + b * a.dst_sb * esz;
    ab.dst1 = reinterpret_cast<char *>(dv_seg) + b * a.dst_sb * esz;
    const int r = desc->dtype == S1F_BF16 ? launch_rows<float, bf16_t>(ab, st) : launch_rows<float, float>(ab, st);
    if (r != S1F_OK) return r;
  }
  return S1F_OK;
}
