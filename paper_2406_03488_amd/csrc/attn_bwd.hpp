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
  static constexpr int STAGE_BYTES = 2 * KT::BYTES;    // K tile, V tile right behind it
  static constexpr int LDS_BYTES = 2 * STAGE_BYTES;    // two stages
  static_assert(STAGE_BYTES % 8192 == 0, "stages must keep the 8 KiB alignment of the fragment reader");
};

// Lane = one query (column ln); keys run over registers.
//   S^T[key][q]  = K Q^T      A = K (LDS),            B = Q (registers)
//   dP^T[key][q] = V dO^T     A = V (LDS),            B = dO (registers)
//   dQ^T[d][q]  += K^T dS^T   A = K read transposed,  B = dS^T slab (registers)
// The accumulators of the first two products start from the row statistics (-lse/scale and -delta, the
// same in every register of a lane) so that p = exp2(c * s) and dS = p * dp need no further operand.
// K/V tiles are copied HBM -> LDS asynchronously, one tile ahead of their use.
template <typename T, int D, int NQ, int BN, int OCC>
__global__ void __launch_bounds__(256, OCC) seg_attn_bwd_dq_kernel(const AttnArgs a) {
  typedef Elem<T> E;
  typedef typename E::Frag Frag;
  typedef BwdDqCfg<T, D, NQ, BN> Cfg;
  typedef LdsTile<T, BN, D> KT;
  typedef FragReader<KT, T> RD;
  constexpr int EPL = E::EPL, KSTEP = 2 * EPL, NKS = D / KSTEP;
  constexpr int DB = KT::DPAD / 32, NSLAB = 16 / EPL, KB = BN / 32;
  constexpr int BM = 128 * NQ;
  constexpr int BLOCK_BYTES = 32 * KT::RS * 16;
  constexpr int PF = NKS >= 3 ? 3 : 2;   // operand fragments in flight ahead of their use

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
  // This workgroup's key tiles: all that hold keys 0 .. seg_off+last_row, or one chunk of them.  From here on keys
  // are counted from the chunk's first key: seg_off and kv_len are relative to it.
  int kt0, kt1;
  chunk_range(uc, (a.seg_off + row0) / BN, (a.seg_off + last_row) / BN + 1, kt0, kt1);
  const int seg_off = a.seg_off - BN * kt0, kv_len = seg_off + seg_len;
  const int n_kt = kt1 - kt0;

  const int64_t qoff = b * a.q_sb + h * a.q_sh;
  const T *qb = reinterpret_cast<const T *>(a.q) + qoff;
  const T *dob = reinterpret_cast<const T *>(a.dout) + qoff;
  const T *ob = reinterpret_cast<const T *>(a.out) + qoff;
  const int64_t kv_first = b * a.kv_sb + hk * a.kv_sh + (int64_t)(BN * kt0) * a.kv_ss;
  const T *kbase = reinterpret_cast<const T *>(a.k) + kv_first;
  const T *vbase = reinterpret_cast<const T *>(a.v) + kv_first;
  const int64_t lse_off = ((int64_t)b * a.n_q_heads + h) * seg_len;
  const lds_addr lds0 = to_lds_addr(smem);
  AsyncTilePairU<T, BN, D, 4> ld;
  ld.init(wave, lane, a.kv_ss);
  RD rd;
  rd.init(lane);
  ld.issue(kbase, vbase, a.kv_ss, 0, kv_len, lds0, wave, lane);

  Frag qf[NQ][NKS], dof[NQ][NKS];
  float nl[NQ], nd[NQ];   // -lse/scale and -delta of the lane's rows
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
    nd[nq] = -sum_xor32(part);
    nl[nq] = -a.lse[lse_off + rc] / a.scale;
    if (r < seg_len && g == 0 && uc.chunk == 0) {   // row statistics for the dK/dV kernel
      a.delta[lse_off + r] = nl[nq];
      a.delta[a.ws_plane + lse_off + r] = nd[nq];
    }
  }

  f32x16 dq[NQ][DB];
#pragma unroll
  for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int v = 0; v < 16; ++v) dq[nq][db][v] = 0.f;

  const bool w_active = wrow0 < seg_len;
  const int w_last = (wrow0 + 32 * NQ < seg_len ? wrow0 + 32 * NQ : seg_len) - 1;
  const float c = a.scale * kLog2e;
  wait_async_tiles();
  __syncthreads();

  for (int jt = 0; jt < n_kt; ++jt) {
    const lds_addr ktile = lds0 + (jt & 1) * Cfg::STAGE_BYTES;   // the V tile lies KT::BYTES behind it
    const int key0 = jt * BN;
    // the other stage was last read before the barrier that ended the previous iteration
    if (jt + 1 < n_kt) ld.issue(kbase, vbase, a.kv_ss, key0 + BN, kv_len, lds0 + ((jt + 1) & 1) * Cfg::STAGE_BYTES, wave, lane);
    if (w_active && key0 <= seg_off + w_last) {
#pragma unroll
      for (int kb = 0; kb < KB; ++kb) {
        const int kb0 = key0 + 32 * kb;
        if (kb0 > seg_off + w_last) continue;
        const lds_addr kblock = ktile + kb * BLOCK_BYTES;
        f32x16 s[NQ], dp[NQ];
#pragma unroll
        for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
          for (int v = 0; v < 16; ++v) { s[nq][v] = nl[nq]; dp[nq][v] = nd[nq]; }
        // K and V fragments are read from LDS PF steps ahead of the matrix instructions that use them
        {
          Frag kf[PF], vf[PF];
#pragma unroll
          for (int i = 0; i < PF; ++i) rd.nat2(kblock, KT::BYTES, i, kf[i], vf[i]);
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int ks = 0; ks < NKS; ++ks) {
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) {
              s[nq] = mma(kf[ks % PF], qf[nq][ks], s[nq]);
              dp[nq] = mma(vf[ks % PF], dof[nq][ks], dp[nq]);
            }
            if (ks + PF < NKS) rd.nat2(kblock, KT::BYTES, ks + PF, kf[ks % PF], vf[ks % PF]);
            __builtin_amdgcn_sched_barrier(0);
          }
        }
        // register v holds key kb0 + 8*(v/4) + 4*g + v%4, visible to row r iff key <= seg_off + r; only
        // the blocks on the diagonal need the test
        if (kb0 + 31 > seg_off + wrow0) {
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) {
            const int lim = seg_off + wrow0 + 32 * nq + ln - (kb0 + 4 * g);
#pragma unroll
            for (int v = 0; v < 16; ++v) {
              float p = exp2_fast(s[nq][v] * c);
              if (8 * (v >> 2) + (v & 3) > lim) p = 0.f;
              s[nq][v] = p * dp[nq][v];   // dS^T
            }
          }
        } else {
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq)
#pragma unroll
            for (int v = 0; v < 16; ++v) s[nq][v] = exp2_fast(s[nq][v] * c) * dp[nq][v];
        }
#pragma unroll
        for (int t = 0; t < NSLAB; ++t) {
          Frag dsf[NQ];
#pragma unroll
          for (int nq = 0; nq < NQ; ++nq) dsf[nq] = block_slab<T>(s[nq], t);
#pragma unroll
          for (int db = 0; db < DB; ++db) {
            const Frag ktf = rd.tr(kblock, t, db);
#pragma unroll
            for (int nq = 0; nq < NQ; ++nq) dq[nq][db] = mma(ktf, dsf[nq], dq[nq][db]);
          }
        }
      }
    }
    wait_async_tiles();   // this wave's part of the next tile has landed
    __syncthreads();
  }

  if (uc.slot >= 0) {   // a chunk: its unscaled share of the unit's dQ rows goes to the workspace
    float *pd = a.part + (int64_t)uc.slot * (BM * D);
#pragma unroll
    for (int nq = 0; nq < NQ; ++nq) {
      const int rl = wave * 32 * NQ + 32 * nq + ln;   // row within the unit
#pragma unroll
      for (int db = 0; db < DB; ++db)
#pragma unroll
        for (int vq = 0; vq < 4; ++vq) {
          const int d0 = 32 * db + 8 * vq + 4 * g;
          if (d0 < D)
            store4<float>(pd + rl * D + d0, dq[nq][db][4 * vq], dq[nq][db][4 * vq + 1], dq[nq][db][4 * vq + 2],
                          dq[nq][db][4 * vq + 3]);
        }
    }
    return;
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

// Sums the chunks of the units that seg_attn_bwd_dq_kernel split along the keys: dq = scale * sum_c part_c.
// Thread and grid layout as in seg_attn_fwd_merge_kernel.
template <typename T, int D, int BM>
__global__ void __launch_bounds__(256) seg_attn_bwd_dq_merge_kernel(const AttnArgs a) {
  constexpr int C4 = D / 4, RG = 256 / C4, GROUPS = (BM + RG - 1) / RG;
  const int unit = (int)blockIdx.x / GROUPS, rg = (int)blockIdx.x % GROUPS;
  const int rl = rg * RG + (int)threadIdx.x / C4, c4 = (int)threadIdx.x % C4;
  int qt, bh;
  decode_workgroup(a.n_whole + unit, a.n_tiles, a.n_bh, a.tile_major, qt, bh);
  qt = a.n_tiles - 1 - qt;
  const int h = bh % a.n_q_heads, b = bh / a.n_q_heads;
  const int r = qt * BM + rl, S = a.n_split;
  if ((int)threadIdx.x >= RG * C4 || rl >= BM || r >= a.seg_len) return;
  int slot0, slot_step;
  chunk_slots(unit, a.n_split_units, slot0, slot_step);
  const float *pd = a.part + (int64_t)slot0 * (BM * D) + rl * D + 4 * c4;
  f32x4 pc[kMaxChunks];
#pragma unroll
  for (int c = 0; c < kMaxChunks; ++c)
    pc[c] = c < S ? *reinterpret_cast<const f32x4 *>(pd + (int64_t)c * slot_step * (BM * D)) : f32x4{0.f, 0.f, 0.f, 0.f};
  f32x4 acc = pc[0];
#pragma unroll
  for (int c = 1; c < kMaxChunks; ++c) acc += pc[c];
  T *dqb = reinterpret_cast<T *>(a.dq) + b * a.q_sb + h * a.q_sh;
  store4<T>(dqb + (int64_t)r * a.q_ss + 4 * c4, acc[0] * a.scale, acc[1] * a.scale, acc[2] * a.scale, acc[3] * a.scale);
}

// dK/dV kernel.  NW waves of 32 keys each; Q/dO tiles of 32 rows travel through a ring of NST LDS stages.
// DIST: a tile's copy is issued DIST iterations before the iteration that consumes it.
// LAG:  with LAG = 1 the upper half of the waves runs one phase behind the lower half (see the kernel), which
// keeps each tile alive for one more iteration.
template <typename T, int D, int NW, int DIST, int LAG> struct BwdDkdvCfg {
  static constexpr int BQ = 32;                        // rows per Q/dO tile
  static constexpr int BNW = 32 * NW;                  // keys per workgroup
  static constexpr int THREADS = 64 * NW;
  static constexpr int NST = DIST + LAG + 1;           // ring stages
  typedef LdsTile<T, BQ, D> QT;
  static constexpr int STAGE_BYTES = 2 * QT::BYTES;    // Q tile, dO tile right behind it
  static constexpr int STAT_BYTES = 2 * BQ * 4;        // -lse/scale and -delta of the tile's rows
  typedef PaddedRows<T, BNW, D> VT;                    // the workgroup's V rows
  static constexpr int LDS_BYTES = NST * STAGE_BYTES + VT::BYTES + NST * STAT_BYTES;   // stages, V, statistics
  static_assert(STAGE_BYTES % 8192 == 0, "stages must keep the 8 KiB alignment of the fragment reader");
  static_assert(DIST >= 1 && LAG >= 0 && LAG <= 1 && NW % 4 == 0, "schedule");
};

// Lane = one key (column ln); queries run over registers.
//   S[q][key]  = Q K^T         A = Q (LDS),              B = K (registers)
//   dP[q][key] = dO V^T        A = dO (LDS),             B = V (LDS)
//   dV^T[d][key] += dO^T P     A = dO read transposed,   B = P slab (registers)
//   dK^T[d][key] += Q^T dS     A = Q read transposed,    B = dS slab (registers)
// The wave's K fragments, its dK and dV accumulators and the block's S and dP fill the register budget of
// two waves per SIMD; its V rows are therefore read from LDS (copied there once, in padded rows).
// Q/dO tiles and their row statistics are copied HBM -> LDS asynchronously (no staging registers).
//
// A wave's work on one tile has three phases: B (S and dP on the matrix pipe), C (exp and dS on the vector
// pipe), D (dV and dK on the matrix pipe).  Two waves share a SIMD, and one's vector phase should meet the other's
// matrix phases instead of both queueing for the same pipe.  Either the two belong to different workgroups (NW = 4,
// WGS = 2: two workgroups per compute unit with barriers of their own, which also overlaps one's prologue and
// epilogue with the other's loop; the shape the library launches for bf16), or to the two halves of one workgroup
// (NW = 8) whose upper half, with LAG = 1, runs the sequence one phase late (C and D of the previous tile, then B of
// the current one).
template <typename T, int D, int NW, int DIST, int LAG, int WGS = 1>   // WGS: workgroups meant to share a compute unit
__global__ void __launch_bounds__(64 * NW, WGS * NW / 4) seg_attn_bwd_dkdv_kernel(const AttnArgs a) {
  typedef Elem<T> E;
  typedef typename E::Frag Frag;
  typedef BwdDkdvCfg<T, D, NW, DIST, LAG> Cfg;
  typedef typename Cfg::QT QT;
  typedef FragReader<QT, T> RD;
  constexpr int EPL = E::EPL, KSTEP = 2 * EPL, NKS = D / KSTEP;
  constexpr int DB = QT::DPAD / 32, NSLAB = 16 / EPL, BQ = Cfg::BQ, NST = Cfg::NST;
  constexpr int PF = 2;              // steps by which operand fragments are read ahead in phase B ...
  constexpr int PFD = 2;             // ... and in phase D (deeper rings spill at two waves per SIMD and run slower)
  constexpr int NV = NSLAB * DB;     // (slab, d-block) steps of the second pair of products
  static_assert(NKS >= PF && NV >= PFD && PFD >= PF, "prefetch ring deeper than the products");

  extern __shared__ __attribute__((aligned(8192))) char smem[];
  const int tid = threadIdx.x, lane = tid & 63, g = lane >> 5, ln = lane & 31;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  int kt, bh;
  decode_workgroup(blockIdx.x, a.n_tiles, a.n_bh, a.tile_major, kt, bh);   // early key tiles see every query row: heaviest first
  const int n_kv_heads = a.n_q_heads / a.group;
  const int hk = bh % n_kv_heads, b = bh / n_kv_heads;
  const int seg_off = a.seg_off, seg_len = a.seg_len, kv_len = seg_off + seg_len;
  const int j0 = kt * Cfg::BNW;                    // first key of the workgroup
  const int wkey0 = j0 + wave * 32;                // first key of the wave

  const int64_t kvoff = b * a.kv_sb + hk * a.kv_sh;
  const T *kbase = reinterpret_cast<const T *>(a.k) + kvoff;
  const T *vbase = reinterpret_cast<const T *>(a.v) + kvoff;

  // First query row that can see any key of this workgroup, and the tile holding it.  Iteration `it` covers
  // tile qt_first + it % per_head of query head hk * group + it / per_head.
  const int r_first = j0 > seg_off ? j0 - seg_off : 0;
  const int qt_first = r_first / BQ;
  const int n_qt = (seg_len + BQ - 1) / BQ;
  const int per_head = n_qt - qt_first;            // >= 1 because j0 < kv_len
  const int n_it = per_head * a.group;
  const float c = a.scale * kLog2e;
  const bool w_active = wkey0 < kv_len;

  const lds_addr lds0 = to_lds_addr(smem);
  const lds_addr vtile = lds0 + NST * Cfg::STAGE_BYTES;
  const lds_addr stats0 = vtile + Cfg::VT::BYTES;
  AsyncTilePairU<T, BQ, D, NW> ld;
  ld.init(wave, lane, a.q_ss);
  RD rd;
  rd.init(lane);

  // Tile cursors (row offset of the tile, its query head, its ring stage), advanced once per iteration.
  struct Cursor {
    int r0, hq, stage;
  };
  auto advance = [&](Cursor &t) {
    t.r0 += BQ;
    if (t.r0 >= n_qt * BQ) { t.r0 = qt_first * BQ; ++t.hq; }
    t.stage = t.stage + 1 == NST ? 0 : t.stage + 1;
  };
  auto issue = [&](const Cursor &t) {   // rows past the segment re-read its last row
    const int64_t qoff = b * a.q_sb + t.hq * a.q_sh;
    ld.issue(reinterpret_cast<const T *>(a.q) + qoff, reinterpret_cast<const T *>(a.dout) + qoff, a.q_ss, t.r0, seg_len,
             lds0 + t.stage * Cfg::STAGE_BYTES, wave, lane);
    if (wave < 2 * BQ / 64) {   // lane `lane` copies entry 64*wave + lane of {-lse/scale [BQ], -delta [BQ]}
      const int st_idx = wave * 64 + fresh(lane), rr = t.r0 + st_idx % BQ;
      const unsigned st_plane = (unsigned)((st_idx / BQ) * a.ws_plane);
      const float *sb = a.delta + ((int64_t)b * a.n_q_heads + t.hq) * seg_len;     // wave-uniform
      const unsigned so = (st_plane + (unsigned)(rr < seg_len ? rr : seg_len - 1)) * 4u;
      const unsigned dst = stats0 + (unsigned)(t.stage * Cfg::STAT_BYTES + wave * 256);
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dword %1, %2" : : "s"(dst), "v"(so), "s"(sb) : "m0");
    }
  };

  // V rows of the workgroup's keys -> LDS (rows past the prefix are zero: their products are never stored)
  Cfg::VT::template copy<Cfg::THREADS>(smem + NST * Cfg::STAGE_BYTES, vbase + (int64_t)j0 * a.kv_ss, a.kv_ss, kv_len - j0, tid);
  // K fragments of the wave's keys stay in registers for the whole kernel.
  Frag kf[NKS];
  {
    int key = wkey0 + ln;
    key = key < kv_len ? key : kv_len - 1;     // keys past the prefix are computed on a copy and never stored
    const int64_t off = (int64_t)key * a.kv_ss + EPL * g;
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) kf[ks] = load_frag_global<T>(kbase + off + ks * KSTEP);
  }
  Cursor t_iss = {qt_first * BQ, hk * a.group, 0};   // next tile to copy
  for (int i = 0; i < DIST; ++i) {
    if (i < n_it) issue(t_iss);
    advance(t_iss);
  }
  f32x16 dk[DB], dv[DB];
#pragma unroll
  for (int db = 0; db < DB; ++db)
#pragma unroll
    for (int v = 0; v < 16; ++v) { dk[db][v] = 0.f; dv[db][v] = 0.f; }
#pragma unroll
  for (int ks = 0; ks < NKS; ++ks) settle(kf[ks]);
  const lds_addr vrow = Cfg::VT::lane_base(vtile, wave * 32 + ln, g);   // the lane's row of V
  wait_async_tiles();
  __syncthreads();

  // State of the tile in flight.  Operand fragments are read from LDS PF steps ahead of the matrix
  // instruction that consumes them (the compiler, left alone, reads each one right before its use and
  // exposes the LDS latency on every step); the scheduling fences keep that order.
  struct State {
    f32x16 s, dp;
    Frag qa[PF], da[PF], va[PF], tq[PFD], tdo[PFD];
  };
  auto active = [&](const Cursor &t) { return w_active && wkey0 <= seg_off + t.r0 + 31; };

  // Phase B: the accumulators start from the row statistics instead of zero (register v holds row
  // r0 + 8*(v/4) + 4*g + v%4), so that s = q.k - lse/scale and dp = dO.v - delta come out of the matrix
  // pipe ready for p = exp2(c*s) and dS = p*dp.
  // The matrix phases run at a raised wave priority, the vector phase at the default one: when the two waves of a
  // SIMD both have instructions ready, the one feeding the matrix pipe goes first (1.3 % of the kernel, measured).
  auto phase_b = [&](State &z, const Cursor &t) {
    __builtin_amdgcn_s_setprio(2);
    const lds_addr qblock = lds0 + t.stage * Cfg::STAGE_BYTES;   // the dO block lies QT::BYTES behind it
    const lds_addr st = stats0 + (unsigned)(t.stage * Cfg::STAT_BYTES + 16 * g);
#pragma unroll
    for (int vq = 0; vq < 4; ++vq) {
      const f32x4 nl = lds_load<f32x4>(st + 32 * vq);
      const f32x4 nd = lds_load<f32x4>(st + 4 * BQ + 32 * vq);
#pragma unroll
      for (int e = 0; e < 4; ++e) { z.s[4 * vq + e] = nl[e]; z.dp[4 * vq + e] = nd[e]; }
    }
#pragma unroll
    for (int i = 0; i < PF; ++i) {
      rd.nat2(qblock, QT::BYTES, i, z.qa[i], z.da[i]);
      z.va[i] = Cfg::VT::frag(vrow, i);
    }
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int ks = 0; ks < NKS; ++ks) {
      z.s = mma(z.qa[ks % PF], kf[ks], z.s);
      z.dp = mma(z.da[ks % PF], z.va[ks % PF], z.dp);
      if (ks + PF < NKS) {
        rd.nat2(qblock, QT::BYTES, ks + PF, z.qa[ks % PF], z.da[ks % PF]);
        z.va[ks % PF] = Cfg::VT::frag(vrow, ks + PF);
      } else {   // the rings drain: start on the operands of phase D
        const int i = ks + PF - NKS;
        rd.tr2(qblock, QT::BYTES, i / DB, i % DB, z.tq[i], z.tdo[i]);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  // Phase C.  Visible iff key <= seg_off + row and row < seg_len, row = r0 + 4g + 8*(v/4) + v%4; blocks that
  // lie wholly below the diagonal and inside the segment (nearly all of them) skip the test.
  auto phase_c = [&](State &z, const Cursor &t) {
    __builtin_amdgcn_s_setprio(0);
    const lds_addr qblock = lds0 + t.stage * Cfg::STAGE_BYTES;
#pragma unroll
    for (int i = PF; i < PFD; ++i) rd.tr2(qblock, QT::BYTES, i / DB, i % DB, z.tq[i], z.tdo[i]);   // rest of phase D's ring
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int v = 0; v < 16; ++v) {
      const float p = exp2_fast(z.s[v] * c);
      z.s[v] = p;
      z.dp[v] = p * z.dp[v];
    }
    // Tiles on the diagonal or at the end of the segment: entries above the diagonal and rows past the segment are
    // set to zero afterwards, in a branch that holds nothing else (whatever the exponential made of them, infinity
    // included, is overwritten).  One instance of the arithmetic above keeps p and dS in place: with a masked and an
    // unmasked copy of it the compiler moved all 16 dS registers on every step.
    const bool edge = (wkey0 + 31 > seg_off + t.r0) || (t.r0 + 32 > seg_len);
    if (edge) {
      asm volatile("" ::: "memory");   // keeps this a branch
      const int fl = fresh(lane), fg = fl >> 5;
      const int lo = wkey0 + (fl & 31) - seg_off - t.r0 - 4 * fg;   // need 8*(v/4)+v%4 >= lo
      const int hi = seg_len - t.r0 - 4 * fg;                       // and  8*(v/4)+v%4 <  hi
#pragma unroll
      for (int v = 0; v < 16; ++v) {
        const int rr = 8 * (v >> 2) + (v & 3);
        if (rr < lo || rr >= hi) {
          z.s[v] = 0.f;
          z.dp[v] = 0.f;
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);
  };
  auto phase_d = [&](State &z, const Cursor &t) {
    __builtin_amdgcn_s_setprio(2);
    const lds_addr qblock = lds0 + t.stage * Cfg::STAGE_BYTES;
    Frag pf, dsf;
#pragma unroll
    for (int i = 0; i < NV; ++i) {
      const int sl = i / DB, db = i % DB;
      if (db == 0) {
        pf = block_slab<T>(z.s, sl);
        dsf = block_slab<T>(z.dp, sl);
      }
      dv[db] = mma(z.tdo[i % PFD], pf, dv[db]);
      dk[db] = mma(z.tq[i % PFD], dsf, dk[db]);
      if (i + PFD < NV) rd.tr2(qblock, QT::BYTES, (i + PFD) / DB, (i + PFD) % DB, z.tq[i % PFD], z.tdo[i % PFD]);
      __builtin_amdgcn_sched_barrier(0);
    }
  };

  // End of an iteration: the wave's share of the NEXT tile must have landed.  With DIST = 2 the copy issued at the top
  // of this iteration (PER instructions, one more for the statistics on wave 0) belongs to the tile after it and
  // stays in flight across the barrier.
  constexpr int kCopyInsts = AsyncTilePairU<T, BQ, D, NW>::PER;
  auto wait_next_tile = [&](bool issued_this_iteration) {
    if (DIST >= 2 && issued_this_iteration) {
      if (wave < 2 * BQ / 64) wait_async_tiles_but_last<kCopyInsts + 1>();
      else wait_async_tiles_but_last<kCopyInsts>();
    } else {
      wait_async_tiles();
    }
  };
  Cursor cur = {qt_first * BQ, hk * a.group, 0};   // tile of the current iteration
  const bool late = LAG > 0 && wave >= NW / 2;
  if (!late) {
    for (int it = 0; it < n_it; ++it) {
      // the stage this copy overwrites was last read before the barrier that ended the previous iteration
      if (it + DIST < n_it) issue(t_iss);
      advance(t_iss);
      if (active(cur)) {
        State z;
        phase_b(z, cur);
        phase_c(z, cur);
        phase_d(z, cur);
      }
      advance(cur);
      wait_next_tile(it + DIST < n_it);   // this wave's part of tile it+1 has landed
      __syncthreads();
    }
  } else {
    State z;
    Cursor prev = cur;
    for (int it = 0; it < n_it; ++it) {
      if (it + DIST < n_it) issue(t_iss);
      advance(t_iss);
      if (it > 0 && active(prev)) {
        phase_c(z, prev);
        phase_d(z, prev);
      }
      if (active(cur)) phase_b(z, cur);
      prev = cur;
      advance(cur);
      wait_next_tile(it + DIST < n_it);
      __syncthreads();
    }
    if (active(prev)) {
      phase_c(z, prev);
      phase_d(z, prev);
    }
  }

  // Epilogue: acc[key][d] += result, each element touched by exactly one lane of the grid.  In the accumulators a
  // lane holds ONE key and 4-element pieces of its row 32 bytes apart: read-modify-write straight from there would
  // touch 64 different cache lines per instruction.  Each wave therefore passes its 32 x D block through LDS (its
  // own region; rows padded by 16 bytes so that the row-per-lane writes spread over all banks) and updates the
  // accumulators row by row, LPR lanes side by side on one row.
  __syncthreads();   // the late half's last phases still read the tile ring that the regions below overlay
  float *dkb = a.dk_acc + kvoff, *dvb = a.dv_acc + kvoff;
  constexpr int ROWB = QT::DPAD * 4 + 16;           // bytes per staged row
  constexpr int LPR = D / 4;                        // lanes per row (16 bytes each)
  constexpr int RPI = 64 / LPR;                     // rows per instruction
  constexpr int NI = (32 + RPI - 1) / RPI;          // instructions per block
  static_assert(NW * 32 * ROWB <= Cfg::LDS_BYTES, "the epilogue's staging regions must fit the kernel's LDS");
  char *region = smem + wave * (32 * ROWB);
  const int row_in = lane / LPR, col = lane % LPR;
#pragma unroll
  for (int which = 0; which < 2; ++which) {
    const f32x16(&acc)[DB] = which == 0 ? dk : dv;
    const float mul = which == 0 ? a.scale : 1.f;
    float *base = which == 0 ? dkb : dvb;
#pragma unroll
    for (int db = 0; db < DB; ++db)
#pragma unroll
      for (int vq = 0; vq < 4; ++vq) {
        const int d0 = 32 * db + 8 * vq + 4 * g;
        *reinterpret_cast<f32x4 *>(region + ln * ROWB + d0 * 4) =
            f32x4{acc[db][4 * vq] * mul, acc[db][4 * vq + 1] * mul, acc[db][4 * vq + 2] * mul, acc[db][4 * vq + 3] * mul};
      }
    f32x4 cur[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int r = i * RPI + row_in, key = wkey0 + r;
      if (row_in < RPI && r < 32 && key < kv_len)
        cur[i] = *reinterpret_cast<const f32x4 *>(base + (int64_t)key * a.kv_ss + 4 * col);
    }
#pragma unroll
    for (int i = 0; i < NI; ++i) {
      const int r = i * RPI + row_in, key = wkey0 + r;
      if (row_in < RPI && r < 32 && key < kv_len) {
        const f32x4 add = *reinterpret_cast<const f32x4 *>(region + r * ROWB + 16 * col);
        *reinterpret_cast<f32x4 *>(base + (int64_t)key * a.kv_ss + 4 * col) = cur[i] + add;
      }
    }
  }
}

}  // namespace s1f
