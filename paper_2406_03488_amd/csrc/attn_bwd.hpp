// Backward of one segment (derivative of Section 3.1, Eq. 3; accumulation per Section 3.2):
//   p_ij = exp(s_ij - lse_i),  delta_i = dO_i . O_i,  dp_ij = dO_i . v_j,  ds_ij = p_ij (dp_ij - delta_i)
//   dq_i = scale * sum_j ds_ij k_j      dk_j += scale * sum_i ds_ij q_i      dv_j += sum_i p_ij dO_i
//
// Two kernels, neither uses atomics:
//   seg_attn_bwd_dq_kernel    owns query rows (same decomposition as the forward), loops over key tiles,
//                             also writes delta for the second kernel;
//   seg_attn_bwd_dkdv_kernel  owns key rows, loops over the query heads of its K/V group and over the
//                             segment's query tiles, and adds its result into the fp32 prefix accumulators
//                             (each accumulator element is touched by exactly one lane of one workgroup).
// The probabilities are recomputed in both (7 matrix products in total instead of 5) in exchange for
// deterministic sums and no dQ workspace.
#pragma once
#include "attn_device.hpp"

namespace s1f {

template <typename T, int D, int NQ, int BN> struct BwdDqCfg {
  static constexpr int BM = 128 * NQ;
  typedef LdsTile<T, BN, D> KT;
  static constexpr int LDS_BYTES = 4 * KT::BYTES;   // {K, V} x 2 buffers
};

// Lane = one query (column ln); keys run over registers.
//   S^T[key][q]  = K Q^T      A = K (LDS),            B = Q (registers)
//   dP^T[key][q] = V dO^T     A = V (LDS),            B = dO (registers)
//   dQ^T[d][q]  += K^T dS^T   A = K read transposed,  B = dS^T slab (registers)
template <typename T, int D, int NQ, int BN, int OCC>
__global__ void __launch_bounds__(256, OCC) seg_attn_bwd_dq_kernel(const AttnArgs a) {
  typedef Elem<T> E;
  typedef typename E::Frag Frag;
  typedef LdsTile<T, BN, D> KT;
  constexpr int EPL = E::EPL, KSTEP = 2 * EPL, NKS = D / KSTEP;
  constexpr int DB = KT::DPAD / 32, NSLAB = 16 / EPL, KB = BN / 32;
  constexpr int BM = 128 * NQ;

  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, ln = lane & 31;
  int qt, bh;
  decode_workgroup(blockIdx.x, a.n_tiles, a.n_bh, qt, bh);
  qt = a.n_tiles - 1 - qt;   // later (heavier) row tiles are scheduled first
  const int h = bh % a.n_q_heads, b = bh / a.n_q_heads, hk = h / a.group;
  const int seg_off = a.seg_off, seg_len = a.seg_len, kv_len = seg_off + seg_len;
  const int row0 = qt * BM, wrow0 = row0 + wave * 32 * NQ;

  const int64_t qoff = b * a.q_sb + h * a.q_sh;
  const T *qb = reinterpret_cast<const T *>(a.q) + qoff;
  const T *dob = reinterpret_cast<const T *>(a.dout) + qoff;
  const T *ob = reinterpret_cast<const T *>(a.out) + qoff;
  const T *kbase = reinterpret_cast<const T *>(a.k) + b * a.kv_sb + hk * a.kv_sh;
  const T *vbase = reinterpret_cast<const T *>(a.v) + b * a.kv_sb + hk * a.kv_sh;
  const int64_t lse_off = ((int64_t)b * a.n_q_heads + h) * seg_len;

  Frag qf[NQ][NKS], dof[NQ][NKS];
  float lse2[NQ], delta[NQ];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int r = wrow0 + 32 * nq + ln;
    const int rc = r < seg_len ? r : seg_len - 1;
    const int64_t off = (int64_t)rc * a.q_ss + EPL * g;
    float part = 0.f;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      qf[nq][ks] = load_frag_global<T>(qb + off + ks * KSTEP);
      dof[nq][ks] = load_frag_global<T>(dob + off + ks * KSTEP);
      part += frag_dot<T>(dof[nq][ks], load_frag_global<T>(ob + off + ks * KSTEP));
    }
    delta[nq] = sum_xor32(part);
    lse2[nq] = a.lse[lse_off + rc] * kLog2e;
    if (r < seg_len && g == 0) a.delta[lse_off + r] = delta[nq];
  }

  f32x16 dq[NQ][DB];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) dq[nq][db][v] = 0.f;

  const int last_row = (row0 + BM < seg_len ? row0 + BM : seg_len) - 1;
  const int n_kt = (seg_off + last_row) / BN + 1;
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
      const bool diag = key0 + BN - 1 > seg_off + wrow0;
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        f32x16 s[NQ], dp[NQ];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
          for (int v = 0; v < 16; ++v) { s[nq][v] = 0.f; dp[nq][v] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          const Frag kf = KT::nat_frag(kt, 32 * kb + ln, ks, g);
          const Frag vf = KT::nat_frag(vt, 32 * kb + ln, ks, g);
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) {
            s[nq] = mma(kf, qf[nq][ks], s[nq]);
            dp[nq] = mma(vf, dof[nq][ks], dp[nq]);
          }
        }
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq) {
          const int lim = diag ? seg_off + wrow0 + 32 * nq + ln - (key0 + 32 * kb + 4 * g) : 64;
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            float p = exp2_fast(fmaf(s[nq][v], c, -lse2[nq]));
            if (8 * (v >> 2) + (v & 3) > lim) p = 0.f;
            s[nq][v] = p * (dp[nq][v] - delta[nq]);   // dS^T
          }
        }
#pragma unroll
        for (int t = 0; t < NSLAB; ++t) {
          Frag dsf[NQ];
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) dsf[nq] = block_slab<T>(s[nq], t);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const Frag ktf = KT::tr_frag(kt, 32 * kb, t, db, lane);
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) dq[nq][db] = mma(ktf, dsf[nq], dq[nq][db]);
          }
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

  T *dqb = reinterpret_cast<T *>(a.dq) + qoff;
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int r = wrow0 + 32 * nq + ln;
    if (r < seg_len) {
      T *row = dqb + (int64_t)r * a.q_ss;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int d0 = 32 * db + 8 * vq + 4 * g;
          if (d0 < D)
            store4<T>(row + d0, dq[nq][db][4 * vq] * a.scale, dq[nq][db][4 * vq + 1] * a.scale,
                      dq[nq][db][4 * vq + 2] * a.scale, dq[nq][db][4 * vq + 3] * a.scale);
        }
    }
  }
}

template <typename T, int D, int NK, int BQ> struct BwdDkdvCfg {
  static constexpr int BNW = 128 * NK;                 // keys per workgroup
  typedef LdsTile<T, BQ, D> QT;
  static constexpr int STAT_BYTES = 2 * BQ * 4;        // lse*log2(e) and delta of the tile's rows
  static constexpr int BUF_BYTES = 2 * QT::BYTES + STAT_BYTES;
  static constexpr int LDS_BYTES = 2 * BUF_BYTES;      // double buffered
};

// Lane = one key (column ln); queries run over registers.
//   S[q][key]  = Q K^T         A = Q (LDS),              B = K (registers)
//   dP[q][key] = dO V^T        A = dO (LDS),             B = V (registers)
//   dV^T[d][key] += dO^T P     A = dO read transposed,   B = P slab (registers)
//   dK^T[d][key] += Q^T dS     A = Q read transposed,    B = dS slab (registers)
template <typename T, int D, int NK, int BQ>
__global__ void __launch_bounds__(256) seg_attn_bwd_dkdv_kernel(const AttnArgs a) {
  typedef Elem<T> E;
  typedef typename E::Frag Frag;
  typedef BwdDkdvCfg<T, D, NK, BQ> Cfg;
  typedef LdsTile<T, BQ, D> QT;
  constexpr int EPL = E::EPL, KSTEP = 2 * EPL, NKS = D / KSTEP;
  constexpr int DB = QT::DPAD / 32, NSLAB = 16 / EPL, QB = BQ / 32;
  static_assert(BQ % 32 == 0 && 2 * BQ <= 256, "query tile");

  extern __shared__ __attribute__((aligned(16))) char smem[];
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63, g = lane >> 5, ln = lane & 31;
  int kt, bh;
  decode_workgroup(blockIdx.x, a.n_tiles, a.n_bh, kt, bh);   // early key tiles see every query row: heaviest first
  const int n_kv_heads = a.n_q_heads / a.group;
  const int hk = bh % n_kv_heads, b = bh / n_kv_heads;
  const int seg_off = a.seg_off, seg_len = a.seg_len, kv_len = seg_off + seg_len;
  const int j0 = kt * Cfg::BNW;                    // first key of the workgroup
  const int wkey0 = j0 + wave * 32 * NK;           // first key of the wave

  const int64_t kvoff = b * a.kv_sb + hk * a.kv_sh;
  const T *kbase = reinterpret_cast<const T *>(a.k) + kvoff;
  const T *vbase = reinterpret_cast<const T *>(a.v) + kvoff;

  Frag kf[NK][NKS], vf[NK][NKS];
#pragma unroll
  for (int nk = 0; nk < NK; ++nk) {
    int key = wkey0 + 32 * nk + ln;
    key = key < kv_len ? key : kv_len - 1;     // keys past the prefix are computed on a copy and never stored
    const int64_t off = (int64_t)key * a.kv_ss + EPL * g;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      kf[nk][ks] = load_frag_global<T>(kbase + off + ks * KSTEP);
      vf[nk][ks] = load_frag_global<T>(vbase + off + ks * KSTEP);
    }
  }
  f32x16 dk[NK][DB], dv[NK][DB];
#pragma unroll
  for (int nk = 0; nk < NK; ++nk)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) { dk[nk][db][v] = 0.f; dv[nk][db][v] = 0.f; }

  // First query row that can see any key of this workgroup, and the tile holding it.
  const int r_first = j0 > seg_off ? j0 - seg_off : 0;
  const int qt_first = r_first / BQ;
  const int n_qt = (seg_len + BQ - 1) / BQ;
  const int per_head = n_qt - qt_first;            // >= 1 because j0 < kv_len
  const int n_it = per_head * a.group;
  const float c = a.scale * kLog2e;
  const bool w_active = wkey0 < kv_len;

  TileCopy<T, BQ, D, 256> cq, cdo;
  float stat = 0.f;   // one lse2 or delta value staged by threads 0 .. 2*BQ-1

  auto issue = [&](int it) {
    const int hq = hk * a.group + it / per_head;
    const int r0 = (qt_first + it % per_head) * BQ;
    const int64_t qoff = b * a.q_sb + hq * a.q_sh + (int64_t)r0 * a.q_ss;
    cq.load(reinterpret_cast<const T *>(a.q) + qoff, a.q_ss, seg_len - r0, tid);
    cdo.load(reinterpret_cast<const T *>(a.dout) + qoff, a.q_ss, seg_len - r0, tid);
    if (tid < 2 * BQ) {
      const int rr = r0 + (tid % BQ);
      const int64_t so = ((int64_t)b * a.n_q_heads + hq) * seg_len + (rr < seg_len ? rr : seg_len - 1);
      stat = tid < BQ ? a.lse[so] * kLog2e : a.delta[so];
    }
  };
  auto commit = [&](int buf) {
    char *base = smem + buf * Cfg::BUF_BYTES;
    cq.store(base, tid);
    cdo.store(base + QT::BYTES, tid);
    if (tid < 2 * BQ) reinterpret_cast<float *>(base + 2 * QT::BYTES)[tid] = stat;
  };

  issue(0);
  commit(0);
  __syncthreads();

  for (int it = 0; it < n_it; ++it) {
    const char *base = smem + (it & 1) * Cfg::BUF_BYTES;
    const char *qtile = base, *dotile = base + QT::BYTES;
    const float *lse2s = reinterpret_cast<const float *>(base + 2 * QT::BYTES);
    const float *deltas = lse2s + BQ;
    const int r0 = (qt_first + it % per_head) * BQ;
    if (it + 1 < n_it) issue(it + 1);

    if (w_active && wkey0 <= seg_off + r0 + BQ - 1) {
#pragma unroll
      for (int qb = 0; qb < QB; ++qb) {
        const int rb = r0 + 32 * qb;   // first row of this 32-row block
        if (wkey0 > seg_off + rb + 31 || rb >= seg_len) continue;
        f32x16 s[NK], dp[NK];
#pragma unroll
        for (int nk = 0; nk < NK; ++nk)
#pragma unroll
          for (int v = 0; v < 16; ++v) { s[nk][v] = 0.f; dp[nk][v] = 0.f; }
#pragma unroll
        for (int ks = 0; ks < NKS; ++ks) {
          const Frag qa = QT::nat_frag(qtile, 32 * qb + ln, ks, g);
          const Frag da = QT::nat_frag(dotile, 32 * qb + ln, ks, g);
#pragma unroll
          for (int nk = 0; nk < NK; ++nk) {
            s[nk] = mma(qa, kf[nk][ks], s[nk]);
            dp[nk] = mma(da, vf[nk][ks], dp[nk]);
          }
        }
        // rows of register v: rb + 8*(v/4) + 4*g + v%4
        f32x4 l2[4], dl[4];
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          l2[vq] = *reinterpret_cast<const f32x4 *>(lse2s + 32 * qb + 8 * vq + 4 * g);
          dl[vq] = *reinterpret_cast<const f32x4 *>(deltas + 32 * qb + 8 * vq + 4 * g);
        }
        const bool edge = (wkey0 + 32 * NK - 1 > seg_off + rb) || (rb + 32 > seg_len);
#pragma unroll
        for (int nk = 0; nk < NK; ++nk) {
          const int key = wkey0 + 32 * nk + ln;
          // visible iff key <= seg_off + row and row < seg_len, row = rb + 4g + 8*(v/4) + v%4
          const int lo = edge ? key - seg_off - rb - 4 * g : -64;     // need 8*(v/4)+v%4 >= lo
          const int hi = edge ? seg_len - rb - 4 * g : 64;            // and  8*(v/4)+v%4 <  hi
#pragma unroll
          for (int v = 0; v < 16; ++v) {
            const int rr = 8 * (v >> 2) + (v & 3);
            float p = exp2_fast(fmaf(s[nk][v], c, -l2[v >> 2][v & 3]));
            if (rr < lo || rr >= hi) p = 0.f;
            s[nk][v] = p;
            dp[nk][v] = p * (dp[nk][v] - dl[v >> 2][v & 3]);
          }
        }
#pragma unroll
        for (int t = 0; t < NSLAB; ++t) {
          Frag pf[NK], dsf[NK];
#pragma unroll
          for (int nk = 0; nk < NK; ++nk) {
            pf[nk] = block_slab<T>(s[nk], t);
            dsf[nk] = block_slab<T>(dp[nk], t);
          }
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const Frag dot = QT::tr_frag(dotile, 32 * qb, t, db, lane);
            const Frag qtf = QT::tr_frag(qtile, 32 * qb, t, db, lane);
#pragma unroll
            for (int nk = 0; nk < NK; ++nk) {
              dv[nk][db] = mma(dot, pf[nk], dv[nk][db]);
              dk[nk][db] = mma(qtf, dsf[nk], dk[nk][db]);
            }
          }
        }
      }
    }
    if (it + 1 < n_it) commit((it + 1) & 1);
    __syncthreads();
  }

  float *dkb = a.dk_acc + kvoff, *dvb = a.dv_acc + kvoff;
#pragma unroll
  for (int nk = 0; nk < NK; ++nk) {
    const int key = wkey0 + 32 * nk + ln;
    if (key < kv_len) {
      float *dkr = dkb + (int64_t)key * a.kv_ss, *dvr = dvb + (int64_t)key * a.kv_ss;
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int d0 = 32 * db + 8 * vq + 4 * g;
          if (d0 < D) {
            f32x4 x = *reinterpret_cast<f32x4 *>(dkr + d0), y = *reinterpret_cast<f32x4 *>(dvr + d0);
#pragma unroll
            for (int e = 0; e < 4; ++e) {
              x[e] += dk[nk][db][4 * vq + e] * a.scale;
              y[e] += dv[nk][db][4 * vq + e];
            }
            *reinterpret_cast<f32x4 *>(dkr + d0) = x;
            *reinterpret_cast<f32x4 *>(dvr + d0) = y;
          }
        }
    }
  }
}

}  // namespace s1f
