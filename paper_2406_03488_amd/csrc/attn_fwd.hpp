// Forward of one segment: out = softmax(q k^T / sqrt(D), causal with the diagonal shifted by seg_off) v,
// lse = log-sum-exp of the scaled scores (Section 3.1, Eq. 3, restricted to the segment's rows).
//
// One workgroup (4 waves) owns BM = 128*NQ query rows of one head; wave w owns rows 32*NQ*w .. +32*NQ.
// The transposed products are computed so that a lane always holds ONE query (column ln) and the
// keys run over registers:
//     S^T[key][q] = sum_d K[key][d] Q[q][d]        A = K fragment from LDS, B = Q fragment (registers)
//     O^T[d][q]  += sum_key V[key][d] P^T[key][q]  A = V read transposed from LDS, B = P^T slab (registers)
// Row maximum and sum are then in-lane reductions plus one exchange with the partner lane (lane ^ 32).
// K/V tiles of BN keys are staged through registers into double-buffered, swizzled LDS tiles.
// Key tiles wholly above the shifted diagonal are never visited; tiles wholly below it skip masking.
#pragma once
#include "attn_device.hpp"

namespace s1f {

template <typename T, int D, int NQ, int BN> struct FwdCfg {
  static constexpr int BM = 128 * NQ;
  typedef LdsTile<T, BN, D> KT;
  static constexpr int LDS_BYTES = 4 * KT::BYTES;   // {K, V} x 2 buffers
};

template <typename T, int D, int NQ, int BN>
__global__ void __launch_bounds__(256) seg_attn_fwd_kernel(const AttnArgs a) {
  typedef Elem<T> E;
  typedef typename E::Frag Frag;
  typedef LdsTile<T, BN, D> KT;
  constexpr int EPL = E::EPL, KSTEP = 2 * EPL, NKS = D / KSTEP;
  constexpr int DB = KT::DPAD / 32, NSLAB = 16 / EPL, KB = BN / 32;
  constexpr int BM = 128 * NQ;
  static_assert(D % KSTEP == 0 && BN % 32 == 0, "shape");

  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, ln = lane & 31;
  const int qt = (int)gridDim.x - 1 - (int)blockIdx.x;   // later (heavier) row tiles are scheduled first
  const int h = blockIdx.y, b = blockIdx.z, hk = h / a.group;
  const int seg_off = a.seg_off, seg_len = a.seg_len, kv_len = seg_off + seg_len;
  const int row0 = qt * BM, wrow0 = row0 + wave * 32 * NQ;

  const T *qb = reinterpret_cast<const T *>(a.q) + b * a.q_sb + h * a.q_sh;
  const T *kbase = reinterpret_cast<const T *>(a.k) + b * a.kv_sb + hk * a.kv_sh;
  const T *vbase = reinterpret_cast<const T *>(a.v) + b * a.kv_sb + hk * a.kv_sh;

  Frag qf[NQ][NKS];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    int r = wrow0 + 32 * nq + ln;
    r = r < seg_len ? r : seg_len - 1;   // rows past the segment are computed on a copy and never stored
    const T *p = qb + (int64_t)r * a.q_ss + EPL * g;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) qf[nq][ks] = load_frag_global<T>(p + ks * KSTEP);
  }

  f32x16 o[NQ][DB];
  float m[NQ], l[NQ];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    m[nq] = -INFINITY;
    l[nq] = 0.f;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) o[nq][db][v] = 0.f;
  }

  const int last_row = (row0 + BM < seg_len ? row0 + BM : seg_len) - 1;
  const int n_kt = (seg_off + last_row) / BN + 1;            // tiles holding keys 0 .. seg_off+last_row
  const bool w_active = wrow0 < seg_len;
  const int w_last = (wrow0 + 32 * NQ < seg_len ? wrow0 + 32 * NQ : seg_len) - 1;
  const float c = a.scale * kLog2e;

  TileCopy<T, BN, D, 256> ck, cv;
  ck.load(kbase, a.kv_ss, kv_len, tid);
  cv.load(vbase, a.kv_ss, kv_len, tid);
  ck.store(smem, tid);
  cv.store(smem + KT::BYTES, tid);
  __syncthreads();

  for (int jt = 0; jt < n_kt; ++jt) {
    const char *kt = smem + (jt & 1) * 2 * KT::BYTES;
    const char *vt = kt + KT::BYTES;
    const int key0 = jt * BN;
    if (jt + 1 < n_kt) {
      const int nk0 = key0 + BN;
      ck.load(kbase + (int64_t)nk0 * a.kv_ss, a.kv_ss, kv_len - nk0, tid);
      cv.load(vbase + (int64_t)nk0 * a.kv_ss, a.kv_ss, kv_len - nk0, tid);
    }
    if (w_active && key0 <= seg_off + w_last) {
      f32x16 s[KB][NQ];
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
          for (int v = 0; v < 16; ++v) s[kb][nq][v] = 0.f;
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          const Frag kf = KT::nat_frag(kt, 32 * kb + ln, ks, g);
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) s[kb][nq] = mma(kf, qf[nq][ks], s[kb][nq]);
        }
      }
      if (key0 + BN - 1 > seg_off + wrow0) {   // the tile crosses the diagonal for some row of this wave
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) {
            const int lim = seg_off + wrow0 + 32 * nq + ln - (key0 + 32 * kb + 4 * g);   // visible iff 8*(v/4)+v%4 <= lim
#pragma unroll
            for (int v = 0; v < 16; ++v)
              if (8 * (v >> 2) + (v & 3) > lim) s[kb][nq][v] = -INFINITY;
          }
      }
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) {
        float mx = -INFINITY;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) mx = fmaxf(mx, s[kb][nq][v]);
        mx = fmaxf(mx, xor32(mx));
        const float m_new = fmaxf(m[nq], mx * c);
        const float alpha = exp2_fast(m[nq] - m_new);
        m[nq] = m_new;
        float rs = 0.f;
#pragma unroll
        for (int kb = 0; kb < KB; ++kb)
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const float p = exp2_fast(fmaf(s[kb][nq][v], c, -m_new));
            s[kb][nq][v] = p;
            rs += p;
          }
        l[nq] = l[nq] * alpha + rs;
#pragma unroll
        for (int db = 0; db < DB; ++db)
#pragma unroll
          for (int v = 0; v < 16; ++v) o[nq][db][v] *= alpha;
      }
#pragma unroll
      for (int kb = 0; kb < KB; ++kb)
#pragma unroll
        for (int t = 0; t < NSLAB; ++t) {
          Frag pf[NQ];
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) pf[nq] = block_slab<T>(s[kb][nq], t);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const Frag vf = KT::tr_frag(vt, 32 * kb, t, db, lane);
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) o[nq][db] = mma(vf, pf[nq], o[nq][db]);
          }
        }
    }
    if (jt + 1 < n_kt) {
      char *nk = smem + ((jt + 1) & 1) * 2 * KT::BYTES;
      ck.store(nk, tid);
      cv.store(nk + KT::BYTES, tid);
    }
    __syncthreads();
  }

  T *ob = reinterpret_cast<T *>(a.out_w) + b * a.q_sb + h * a.q_sh;
  float *lse = a.lse + ((int64_t)b * a.n_q_heads + h) * seg_len;
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const float lt = l[nq] + xor32(l[nq]);
    const float inv = 1.f / lt;
    const int r = wrow0 + 32 * nq + ln;
    if (r < seg_len) {
      T *orow = ob + (int64_t)r * a.q_ss;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int d0 = 32 * db + 8 * vq + 4 * g;
          if (d0 < D)
            store4<T>(orow + d0, o[nq][db][4 * vq] * inv, o[nq][db][4 * vq + 1] * inv, o[nq][db][4 * vq + 2] * inv,
                      o[nq][db][4 * vq + 3] * inv);
        }
      if (g == 0) lse[r] = (m[nq] + __builtin_amdgcn_logf(lt)) * kLn2;
    }
  }
}

}  // namespace s1f
