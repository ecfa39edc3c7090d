// Forward of one segment: out = softmax(q k^T / sqrt(D), causal with the diagonal shifted by seg_off) v,
// lse = log-sum-exp of the scaled scores (Section 3.1, Eq. 3, restricted to the segment's rows).
//
// One workgroup (NW waves) owns BM = 32*NQ*NW query rows of one head; wave w owns rows 32*NQ*w .. +32*NQ.
// The transposed products are computed so that a lane always holds ONE query (column ln) and the
// keys run over registers:
//     S^T[key][q] = sum_d K[key][d] Q[q][d]        A = K fragment from LDS, B = Q fragment (registers)
//     O^T[d][q]  += sum_key V[key][d] P^T[key][q]  A = V read transposed from LDS, B = P^T slab (registers)
// Row maximum and sum are then in-lane reductions plus one exchange with the partner lane (lane ^ 32).
//
// K/V tiles of BN = 32*KB keys go from HBM straight into a 3-stage ring of swizzled LDS tiles (no register
// staging); tile j+2 is in flight while tiles j and j+1 are consumed, with one workgroup barrier per tile.
// The loop advances in steps of one 32-key block and is software-pipelined inside each wave: the score
// product of block k+1 (matrix pipe) is issued together with the row sums and operand packing of block k's
// probabilities (vector pipe), then the PV product of block k together with the maximum and the exponentials
// of block k+1 (see fwd_step).  Key blocks wholly above the shifted diagonal are never visited; blocks wholly
// below it run a step without any masking code.
#pragma once
#include "attn_device.hpp"


namespace s1f {

// Lazy rescaling: the running maximum m of a row is raised only when a new block makes its probabilities
// 2^(s*c - m) large, and the steady loop finds that out from their SUM, which it needs anyway, instead of from their
// maximum: a lane adds up the probabilities of its 16 keys of the block, and if that sum exceeds 2^kRescaleTau in
// any lane of the wave (infinity included: the exponentials are taken before anyone has looked), the loop is left,
// the block's row maxima are computed, the rows whose maximum exceeds m by more than kRescaleTau - 4 (a sum over 16
// keys above 2^tau needs one of them above 2^(tau-4)) take it as their new m, O and l are rescaled and the block's
// probabilities recomputed.  Otherwise every probability is at most 2^kRescaleTau, which fp32 sums and bf16
// operands hold without loss.  The accumulator rescale (a pass over every O register) and the maximum (a chain of
// its own through all 16 scores, plus a lane exchange) thereby leave the steady loop.
constexpr float kRescaleTau = 8.0f;
constexpr float kRescaleLimit = 256.0f;   // 2^kRescaleTau

template <typename T, int D, int NQ, int KB, int NW> struct FwdCfg {
  static constexpr int BM = 32 * NQ * NW;
  static constexpr int BN = 32 * KB;
  static constexpr int THREADS = 64 * NW;
  typedef LdsTile<T, BN, D> KT;
  static constexpr int STAGE_BYTES = 2 * KT::BYTES;      // K tile then V tile
  static constexpr int LDS_BYTES = 3 * STAGE_BYTES;
};

// Number of operand fragments a wave keeps in flight ahead of the matrix instruction that consumes them
// (LDS latency is three to four 32x32x16 MFMAs).
constexpr int kPrefetch = 2;

// S^T blocks of one 32-key block: s[nq] = K[block rows, :] Q^T   (prologue only; the loop uses fwd_step)
template <typename RD, typename T, int NQ, int NKS>
S1F_DEV void fwd_scores(f32x16 (&s)[NQ], const typename Elem<T>::Frag (&qf)[NQ][NKS], const RD &rd, lds_addr kblock) {
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
    for (int v = 0; v < 16; ++v) s[nq][v] = 0.f;
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) {
    const typename Elem<T>::Frag kf = rd.nat(kblock, ks);
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) s[nq] = mma(kf, qf[nq][ks], s[nq]);
  }
}

// Masks the scores of a block that crosses the diagonal.
//   lim0 = (absolute row of this lane's query in query block 0) - (first key of the block) - 4g
template <int NQ> S1F_DEV void fwd_mask(f32x16 (&s)[NQ], int lim0) {
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const int lim = lim0 + 32 * nq;   // register v is visible iff 8*(v/4) + v%4 <= lim
#pragma unroll
    for (int v = 0; v < 16; ++v) s[nq][v] = (8 * (v >> 2) + (v & 3) > lim) ? -INFINITY : s[nq][v];
  }
}

// Row maxima of a block in log2 units (each lane gets the maximum of its query's 32 scores).
template <int NQ> S1F_DEV void fwd_row_max(const f32x16 (&s)[NQ], float (&mx)[NQ], float c) {
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    float x = -INFINITY;
#pragma unroll
    for (int v = 0; v < 16; ++v) x = fmaxf(x, s[nq][v]);
    mx[nq] = max_xor32(x) * c;
  }
}

// Probabilities of a block from its scores, against the running maximum m (log2 units): p = 2^(s*c - m); rs = the
// sum over this lane's 16 keys.
template <int NQ>
S1F_DEV void fwd_probs(f32x16 (&p)[NQ], const f32x16 (&s)[NQ], const float (&m)[NQ], float c, float (&rs)[NQ]) {
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    rs[nq] = 0.f;
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      p[nq][v] = exp2_fast(fmaf(s[nq][v], c, -m[nq]));
      rs[nq] += p[nq][v];
    }
  }
}

// One pipelined step over block k, whose probabilities (against m) are in `p` and already counted in l:
//   phase 1   sn = scores of block k+1 (matrix pipe)  ||  p packed into operand slabs (vector pipe)
//   phase 2   O += P V of block k (matrix pipe)        ||  p = 2^(sn*c - m): block k+1's probabilities, and their sums rs
// The probabilities of block k+1 are computed against the CURRENT m, before anyone knows whether m has to be raised
// for them: the caller looks at rs afterwards (see kRescaleTau) and, in the rare case that it must raise m, rescales
// O and l and recomputes p from sn (which this step leaves untouched); otherwise it adds rs to l.  That way the
// loop carries the probabilities in the registers they were written to; carrying the SCORES of block k+1 over
// instead (exponentials at the start of the next step) cost a 16-register copy per step and measured 3 % slower.
// Operand fragments are read from LDS kPrefetch matrix instructions ahead of their use (the V fragments
// of phase 2 start arriving during the last slots of phase 1).  No scheduling fences: the compiler keeps the
// reads ahead by itself here, and with fences per slot the kernel measured 0.5-1 % slower.
//   mask_next: block k+1 crosses the diagonal of the wave's rows
//   lim0_next = (absolute row of this lane's query in query block 0) - (first key of block k+1) - 4g
template <typename RD, typename T, bool HAS_NEXT, int NQ, int NKS, int DB>
S1F_DEV void fwd_step(f32x16 (&p)[NQ], f32x16 (&sn)[NQ], f32x16 (&o)[NQ][DB], const float (&m)[NQ], float (&rs)[NQ],
                      const typename Elem<T>::Frag (&qf)[NQ][NKS], const RD &rd,
                      lds_addr kblock_next, lds_addr vblock, float c, bool mask_next, int lim0_next
                      ) {
  typedef typename Elem<T>::Frag Frag;
  constexpr int NSLAB = 16 / Elem<T>::EPL;
  constexpr int PF = kPrefetch;
  constexpr int NV = NSLAB * DB;   // V fragments of the block, in the order (slab, d-block)
  static_assert(NKS >= PF && NV >= PF, "prefetch ring deeper than the products");

  Frag vf[PF];
  Frag pf[NQ][NSLAB];
  if (HAS_NEXT) {
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
      for (int v = 0; v < 16; ++v) sn[nq][v] = 0.f;
    Frag kf[PF];
#pragma unroll
    for (int i = 0; i < PF; ++i) kf[i] = rd.nat(kblock_next, i);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) sn[nq] = mma(kf[ks % PF], qf[nq][ks], sn[nq]);
      if (ks + PF < NKS) {
        kf[ks % PF] = rd.nat(kblock_next, ks + PF);
      } else {   // the K ring drains: its slots go to the first V fragments
        const int i = ks + PF - NKS;
        vf[i] = rd.tr(vblock, i / DB, i % DB);
      }
    }
  } else {
#pragma unroll
    for (int i = 0; i < PF; ++i) vf[i] = rd.tr(vblock, i / DB, i % DB);
  }
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
    for (int t = 0; t < NSLAB; ++t) pf[nq][t] = block_slab<T>(p[nq], t);
  // Blocks that cross the diagonal of this wave's rows get their mask here, in a branch of its own that holds
  // no matrix instruction: two instances of the whole step (with and without mask code) in one loop body make
  // the compiler keep the output accumulators in two places and copy all 64 registers on every step.
  if (HAS_NEXT && mask_next) {
    asm volatile("" ::: "memory");   // keeps this a branch: turned into selects it would run on every step
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
      for (int v = 0; v < 16; ++v)
        if (8 * (v >> 2) + (v & 3) > lim0_next + 32 * nq) sn[nq][v] = -INFINITY;
  }

#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) rs[nq] = 0.f;
#pragma unroll
  for (int t = 0; t < NSLAB; ++t) {
#pragma unroll
    for (int db = 0; db < DB; ++db) {
      const int i = t * DB + db;
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) o[nq][db] = mma(vf[i % PF], pf[nq][t], o[nq][db]);
      if (i + PF < NV) vf[i % PF] = rd.tr(vblock, (i + PF) / DB, (i + PF) % DB);
      if (HAS_NEXT) {   // this slot's share of the next block's 16 probabilities per query block
#pragma unroll
        for (int v = 16 * i / NV; v < 16 * (i + 1) / NV; ++v)
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) {
            p[nq][v] = exp2_fast(fmaf(sn[nq][v], c, -m[nq]));
            rs[nq] += p[nq][v];
          }
      }
    }
  }
}

template <typename T, int D, int NQ, int KB, int NW, int OCC>
__global__ void __launch_bounds__(64 * NW, OCC) seg_attn_fwd_kernel(const AttnArgs a) {
  typedef Elem<T> E;
  typedef typename E::Frag Frag;
  typedef FwdCfg<T, D, NQ, KB, NW> Cfg;
  typedef typename Cfg::KT KT;
  constexpr int EPL = E::EPL, KSTEP = 2 * EPL, NKS = D / KSTEP;
  constexpr int DB = KT::DPAD / 32, BM = Cfg::BM, BN = Cfg::BN;
  static_assert(D % KSTEP == 0, "shape");

  extern __shared__ __attribute__((aligned(8192))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, ln = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const UnitChunk uc = split_unit(blockIdx.x, a.n_whole, a.n_split, a.n_split_units);
  int qt, bh;
  decode_workgroup(uc.unit, a.n_tiles, a.n_bh, a.tile_major, qt, bh);
  qt = a.n_tiles - 1 - qt;   // later (heavier) row tiles are scheduled first
  const int h = bh % a.n_q_heads, b = bh / a.n_q_heads, hk = h / a.group;
  const int seg_len = a.seg_len;
  const int row0 = qt * BM, wrow0 = row0 + wave * 32 * NQ;
  const int last_row = (row0 + BM < seg_len ? row0 + BM : seg_len) - 1;
  // This workgroup's 32-key blocks: all that hold keys 0 .. seg_off+last_row, or one chunk of them.  From here on
  // keys are counted from the chunk's first key: seg_off and kv_len are relative to it.
  int blk0, blk1;
  chunk_range(uc, (a.seg_off + row0) / 32, (a.seg_off + last_row) / 32 + 1, blk0, blk1);
  const int seg_off = a.seg_off - 32 * blk0, kv_len = seg_off + seg_len;
  const int n_blk = blk1 - blk0;
  const int n_kt = (n_blk + KB - 1) / KB;

  const T *qb = reinterpret_cast<const T *>(a.q) + b * a.q_sb + h * a.q_sh;
  const int64_t kv_first = b * a.kv_sb + hk * a.kv_sh + (int64_t)(32 * blk0) * a.kv_ss;
  const T *kbase = reinterpret_cast<const T *>(a.k) + kv_first;
  const T *vbase = reinterpret_cast<const T *>(a.v) + kv_first;

  const lds_addr lds0 = to_lds_addr(smem);
  // The wave's share of a tile's copy is issued in KB parts, one per 32-key step, so that the waves of the
  // workgroup do not queue behind each other's copies right after the barrier.
  constexpr int PER_STEP = (2 * BN * KT::RS / (64 * NW)) / KB;   // copy instructions per wave and step
  typedef AsyncTilePairU<T, BN, D, NW, (PER_STEP < 4 ? PER_STEP : 4)> LD;
  static_assert(LD::PARTS % KB == 0, "the copy splits evenly over the 32-key steps");
  LD ld;
  ld.init(wave, lane, a.kv_ss);
  auto issue_part = [&](int jt, int step_part) {
#pragma unroll
    for (int p = 0; p < LD::PARTS / KB; ++p)
      ld.issue_part(step_part * (LD::PARTS / KB) + p, kbase, vbase, a.kv_ss, jt * BN, kv_len,
                    lds0 + (jt % 3) * Cfg::STAGE_BYTES, wave, lane);
  };
  // The same for the tile whose first row `krow`/`vrow` point at and whose ring stage is known: the steady loop
  // keeps these running instead of deriving them from the tile number on every step.
  auto issue_part_at = [&](const T *krow, const T *vrow, int rows_left, int stage, int step_part) {
#pragma unroll
    for (int p = 0; p < LD::PARTS / KB; ++p)
      ld.issue_part(step_part * (LD::PARTS / KB) + p, krow, vrow, a.kv_ss, 0, rows_left,
                    lds0 + stage * Cfg::STAGE_BYTES, wave, lane);
  };
  auto issue = [&](int jt) {
#pragma unroll
    for (int p = 0; p < KB; ++p) issue_part(jt, p);
  };
  issue(0);
  if (n_kt > 1) issue(1);

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
  const float c = a.scale * kLog2e;

  FragReader<KT, T> rd;
  rd.init(lane);
  constexpr int BLOCK_BYTES = 32 * KT::RS * 16;

  wait_async_tiles();
  __syncthreads();
  f32x16 s[NQ], sn[NQ];
  float mx[NQ];
  fwd_scores<FragReader<KT, T>, T, NQ, NKS>(s, qf, rd, lds0);
  if (31 > seg_off + wrow0) fwd_mask(s, seg_off + wrow0 + ln - 4 * g);
  fwd_row_max(s, mx, c);
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) m[nq] = mx[nq];   // key 0 is visible to every row: finite
  float rs[NQ];
  fwd_probs(s, s, m, c, rs);   // from here on `s` holds the probabilities of the current block, l their sums
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) l[nq] = rs[nq];

  // The steady loop never touches O except through the matrix pipe.  When some row of the wave has to
  // raise its running maximum the loop is left, O and l are rescaled, and the loop is entered again.
  typedef FragReader<KT, T> RD;
  int k = 0;
  // Ring stages of the tiles holding block k (st_cur) and block k + 1 (st_next), and the tile that the next copy
  // fills: its first K and V rows, the rows of the prefix from there on, its stage.
  int st_cur = 0, st_next = KB == 1 ? 1 : 0;
  int jt_iss = 2, st_iss = 2, rows_iss = kv_len - 2 * BN;
  const T *k_iss = kbase + (int64_t)(2 * BN) * a.kv_ss, *v_iss = vbase + (int64_t)(2 * BN) * a.kv_ss;
  while (true) {
    bool raise_any = false;
    while (k + 1 < n_blk) {
      const int kb = k % KB;
      if (kb == KB - 1) {
        wait_async_tiles();   // this wave's part of the next tile has landed (it was issued a whole tile ago)
        __syncthreads();      // ... and everyone's; every wave has also finished reading the previous tile
      }
      // the tile two ahead of block k's (for kb = KB-1; the later parts follow in the steps of the next tile) goes
      // to the stage of the tile before block k's
      {
        const int part = (kb + 1) % KB;
        const bool copying = KB == 1 || k > 0;   // tiles 0 and 1 were copied whole before the loop
        if (copying && jt_iss < n_kt) issue_part_at(k_iss, v_iss, rows_iss, st_iss, part);
        if (copying && part == KB - 1) {   // that tile's copy is complete: move on to the following one
          ++jt_iss;
          st_iss = st_iss == 2 ? 0 : st_iss + 1;
          rows_iss -= BN;
          k_iss += (int64_t)BN * a.kv_ss;
          v_iss += (int64_t)BN * a.kv_ss;
        }
      }
      const lds_addr vblock = lds0 + st_cur * Cfg::STAGE_BYTES + KT::BYTES + kb * BLOCK_BYTES;
      const int kn = k + 1;
      const lds_addr kblock_next = lds0 + st_next * Cfg::STAGE_BYTES + (kn % KB) * BLOCK_BYTES;
      const int lim0n = seg_off + wrow0 + ln - 32 * kn - 4 * g;
      // the last block always crosses the diagonal; earlier ones do if their last key is past the wave's first row
      const bool mask_next = kn + 1 == n_blk || 32 * kn + 31 > seg_off + wrow0;
      fwd_step<RD, T, true>(s, sn, o, m, rs, qf, rd, kblock_next, vblock, c, mask_next, lim0n);
      k = kn;
      st_cur = st_next;
      if ((k + 1) % KB == 0) st_next = st_next == 2 ? 0 : st_next + 1;
      bool raise = false;
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) raise = raise || !(rs[nq] <= kRescaleLimit);
      if (__builtin_amdgcn_ballot_w64(raise) != 0) { raise_any = true; break; }
#pragma unroll
      for (int nq = 0; nq < NQ; ++nq) l[nq] += rs[nq];
    }
    if (!raise_any) break;
    fwd_row_max(sn, mx, c);
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      const float m_up = mx[nq] > m[nq] + (kRescaleTau - 4.f) ? mx[nq] : m[nq];
      const float alpha = exp2_fast(m[nq] - m_up);   // exactly 1 for rows that keep their maximum
      m[nq] = m_up;
      l[nq] *= alpha;
#pragma unroll
      for (int db = 0; db < DB; ++db) o[nq][db] = o[nq][db] * alpha;
    }
    fwd_probs(s, sn, m, c, rs);   // the current block's probabilities again, against the raised maxima
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) l[nq] += rs[nq];
  }
  {   // last block: no next scores to compute
    const lds_addr vblock = lds0 + st_cur * Cfg::STAGE_BYTES + KT::BYTES + (k % KB) * BLOCK_BYTES;
    fwd_step<RD, T, false>(s, sn, o, m, rs, qf, rd, vblock, vblock, c, false, 0);
  }

  if (uc.slot >= 0) {   // a chunk: unnormalised output rows, running maximum and row sum go to the workspace
    float *po = a.part + (int64_t)uc.slot * (BM * D);
    float *pml = a.part_ml + (int64_t)uc.slot * (BM * 2);
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      const float lt = sum_xor32(l[nq]);
      const int rl = wave * 32 * NQ + 32 * nq + ln;   // row within the unit
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int d0 = 32 * db + 8 * vq + 4 * g;
          if (d0 < D)
            store4<float>(po + rl * D + d0, o[nq][db][4 * vq], o[nq][db][4 * vq + 1], o[nq][db][4 * vq + 2],
                          o[nq][db][4 * vq + 3]);
        }
      if (g == 0) {
        pml[2 * rl] = m[nq];
        pml[2 * rl + 1] = lt;
      }
    }
    return;
  }
  T *ob = reinterpret_cast<T *>(a.out_w) + b * a.q_sb + h * a.q_sh;
  float *lse = a.lse + ((int64_t)b * a.n_q_heads + h) * seg_len;
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq) {
    const float lt = sum_xor32(l[nq]);
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

// Merges the chunks of the units that seg_attn_fwd_kernel split along the keys: with m_c, l_c, o_c the running
// maximum (log2 units), row sum and unnormalised output row of chunk c,
//   m = max_c m_c,  l = sum_c l_c 2^(m_c - m),  out = sum_c o_c 2^(m_c - m) / l,  lse = (m + log2 l) ln 2.
// A thread handles 4 consecutive head_dim elements of one row; a workgroup MergeRows<D>::RG rows of one split unit
// (grid: split units x groups of RG rows).  All chunk loads of a thread are independent of each other.
template <int D> struct MergeRows {
  static constexpr int C4 = D / 4;          // threads per row
  static constexpr int RG = 256 / C4;       // rows per workgroup
  static constexpr int groups(int bm) { return (bm + RG - 1) / RG; }
};
template <typename T, int D, int BM>
__global__ void __launch_bounds__(256) seg_attn_fwd_merge_kernel(const AttnArgs a) {
  typedef MergeRows<D> MR;
  const int unit = (int)blockIdx.x / MR::groups(BM), rg = (int)blockIdx.x % MR::groups(BM);
  const int rl = rg * MR::RG + (int)threadIdx.x / MR::C4, c4 = (int)threadIdx.x % MR::C4;
  int qt, bh;
  decode_workgroup(a.n_whole + unit, a.n_tiles, a.n_bh, a.tile_major, qt, bh);
  qt = a.n_tiles - 1 - qt;
  const int h = bh % a.n_q_heads, b = bh / a.n_q_heads;
  const int r = qt * BM + rl, S = a.n_split;
  if ((int)threadIdx.x >= MR::RG * MR::C4 || rl >= BM || r >= a.seg_len) return;
  int slot0, slot_step;
  chunk_slots(unit, a.n_split_units, slot0, slot_step);
  const float *po = a.part + (int64_t)slot0 * (BM * D) + rl * D + 4 * c4;
  const float *pml = a.part_ml + (int64_t)slot0 * (BM * 2) + 2 * rl;
  float mc[kMaxChunks], lc[kMaxChunks];
  f32x4 oc[kMaxChunks];
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const bool on = c < S;
    mc[c] = on ? pml[(int64_t)c * slot_step * (BM * 2)] : -INFINITY;
    lc[c] = on ? pml[(int64_t)c * slot_step * (BM * 2) + 1] : 0.f;
    oc[c] = on ? *reinterpret_cast<const f32x4 *>(po + (int64_t)c * slot_step * (BM * D)) : f32x4{0.f, 0.f, 0.f, 0.f};
  }
  float m = mc[0];
#pragma unroll
  for (int c = 1; c < kMaxChunks; ++c) m = fmaxf(m, mc[c]);
  float l = 0.f;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c) {
    const float w = exp2_fast(mc[c] - m);   // 0 for the chunks past S
    l += w * lc[c];
    acc += w * oc[c];
  }
  const float inv = 1.f / l;
  T *ob = reinterpret_cast<T *>(a.out_w) + b * a.q_sb + h * a.q_sh;
  store4<T>(ob + (int64_t)r * a.q_ss + 4 * c4, acc[0] * inv, acc[1] * inv, acc[2] * inv, acc[3] * inv);
  if (c4 == 0) a.lse[((int64_t)b * a.n_q_heads + h) * a.seg_len + r] = (m + __builtin_amdgcn_logf(l)) * kLn2;
}

}  // namespace s1f
