// Device-side building blocks shared by the three attention kernels (gfx950 / CDNA4 only).
//
// Vocabulary used throughout:
//   wave      64 lanes; lane = 32*g + ln with g in {0,1}, ln in 0..31
//   block     a 32x32 fp32 MFMA result held as 16 registers per lane: register v of lane (g, ln) is
//             element (row 8*(v/4) + 4*g + v%4, column ln)
//   fragment  what one lane feeds to one MFMA as A (row ln) or B (column ln) operand: EPL consecutive
//             elements of the contraction index starting at EPL*g; one MFMA contracts KSTEP = 2*EPL
//   slab      KSTEP consecutive MFMA contraction slots taken from a block's ROW index, so that a block
//             can be fed back as an operand without any cross-lane movement: slot (g, e) of slab t is
//             block row r(t, g, e) = 8*((EPL*t+e)/4) + 4*g + (EPL*t+e)%4, i.e. register EPL*t + e.
//             The other operand is read from LDS in the same row order.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace s1f {

typedef __bf16 bf16_t;
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef __bf16 bf16x4 __attribute__((ext_vector_type(4)));
typedef short s16x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));

#define S1F_DEV __device__ __forceinline__
#define S1F_LDS(ptr_type, p) ((__attribute__((address_space(3))) ptr_type *)(p))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;

template <typename T> struct Elem;
template <> struct Elem<float> {
  static constexpr int EPL = 1;    // elements per lane per MFMA operand
  static constexpr int CE = 4;     // elements per 16-byte chunk
  typedef float Frag;
};
template <> struct Elem<bf16_t> {
  static constexpr int EPL = 8;
  static constexpr int CE = 8;
  typedef bf16x8 Frag;
};

// D(32x32) += A(32xKSTEP) * B(KSTEPx32)
S1F_DEV f32x16 mma(bf16x8 a, bf16x8 b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0); }
S1F_DEV f32x16 mma(float a, float b, f32x16 c) { return __builtin_amdgcn_mfma_f32_32x32x2f32(a, b, c, 0, 0, 0); }

S1F_DEV float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }   // v_exp_f32; exp2(-inf) = 0
// The lane's own value and the value held by its partner lane (lane ^ 32), in unspecified order.
// v_permlane32_swap exchanges the upper half of its first operand with the lower half of its second, so
// with both operands equal to x the register pair ends up as (own, partner) in the lower half-wave and
// (partner, own) in the upper one.  Written as assembly: with two identical operands the compiler's
// builtin hands back its first result for both.  The leading s_nop covers the wait states the
// instruction needs after a vector write of its operands.
S1F_DEV void own_and_partner(float x, float &a, float &b) {
  a = x;
  b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1" : "+v"(a), "+v"(b));
}
S1F_DEV float max_xor32(float x) {
  float a, b;
  own_and_partner(x, a, b);
  return fmaxf(a, b);
}
S1F_DEV float sum_xor32(float x) {
  float a, b;
  own_and_partner(x, a, b);
  return a + b;
}

template <typename T> S1F_DEV typename Elem<T>::Frag load_frag_global(const T *p);
template <> S1F_DEV float load_frag_global<float>(const float *p) { return *p; }
template <> S1F_DEV bf16x8 load_frag_global<bf16_t>(const bf16_t *p) { return *reinterpret_cast<const bf16x8 *>(p); }

template <typename T> S1F_DEV float frag_dot(typename Elem<T>::Frag a, typename Elem<T>::Frag b);
template <> S1F_DEV float frag_dot<float>(float a, float b) { return a * b; }
template <> S1F_DEV float frag_dot<bf16_t>(bf16x8 a, bf16x8 b) {
  float s = 0.f;
#pragma unroll
  for (int e = 0; e < 8; ++e) s += (float)a[e] * (float)b[e];
  return s;
}

// Slab t of a block as an MFMA operand (rounds to bf16 in bf16 mode).
template <typename T> S1F_DEV typename Elem<T>::Frag block_slab(const f32x16 &c, int t);
template <> S1F_DEV float block_slab<float>(const f32x16 &c, int t) { return c[t]; }
template <> S1F_DEV bf16x8 block_slab<bf16_t>(const f32x16 &c, int t) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)c[8 * t + e];
  return r;
}

constexpr int pow2_at_least(int x) { int p = 1; while (p < x) p *= 2; return p; }

// A [ROWS x D] tile of T in LDS, rows of RS 16-byte chunks, chunk c of row r stored at position
// c ^ swz(r).  The swizzle makes both access patterns below bank-conflict free without padding:
// 16 lanes reading the same chunk of 16 consecutive rows, and 32 lanes reading 4 consecutive rows x 4
// consecutive chunks (the transposing read).
template <typename T, int ROWS_, int D_> struct LdsTile {
  static constexpr int ROWS = ROWS_;
  static constexpr int D = D_;
  static constexpr int CE = Elem<T>::CE;
  static constexpr int DPAD = (D + 31) / 32 * 32;
  static constexpr int CPR = D / CE;                       // chunks per row holding data
  static constexpr int RS = pow2_at_least(DPAD / CE);      // row stride in chunks
  static constexpr int BYTES = ROWS * RS * 16;
  static_assert(D % CE == 0, "head_dim must be a whole number of 16-byte chunks");
  static_assert(RS >= 8, "row too short for the swizzle");

  S1F_DEV static int swz(int r) {
    if (RS >= 16) return ((r & 3) << 2) | ((r >> 2) & 3);
    return (((r >> 1) & 1) << 2) | ((r >> 2) & 3);
  }
  S1F_DEV static int chunk_off(int r, int c) { return (r * RS + (c ^ swz(r))) * 16; }   // bytes

  // Operand fragment with the contraction running along D: lane reads row `row`, elements
  // [KSTEP*ks + EPL*g, +EPL).
  S1F_DEV static typename Elem<T>::Frag nat_frag(const char *tile, int row, int ks, int g);
  // Operand fragment with the contraction running along the tile's rows (slab t of the 32-row block
  // starting at row32), for operand index (row for A, column for B) d = 32*db + ln.
  S1F_DEV static typename Elem<T>::Frag tr_frag(const char *tile, int row32, int t, int db, int lane);
};

template <typename Tile> struct TileOps;

template <int ROWS, int D> struct TileOps<LdsTile<float, ROWS, D>> {
  typedef LdsTile<float, ROWS, D> TL;
  S1F_DEV static float nat(const char *tile, int row, int ks, int g) {
    const int d = 2 * ks + g;
    return *reinterpret_cast<const float *>(tile + TL::chunk_off(row, d >> 2) + 4 * (d & 3));
  }
  S1F_DEV static float tr(const char *tile, int row32, int t, int db, int lane) {
    const int g = lane >> 5, ln = lane & 31;
    const int row = row32 + 8 * (t >> 2) + 4 * g + (t & 3);
    const int d = 32 * db + ln;
    return *reinterpret_cast<const float *>(tile + TL::chunk_off(row, d >> 2) + 4 * (d & 3));
  }
};

template <int ROWS, int D> struct TileOps<LdsTile<bf16_t, ROWS, D>> {
  typedef LdsTile<bf16_t, ROWS, D> TL;
  S1F_DEV static bf16x8 nat(const char *tile, int row, int ks, int g) {
    return *reinterpret_cast<const bf16x8 *>(tile + TL::chunk_off(row, 2 * ks + g));
  }
  // ds_read_b64_tr_b16: within each group of 16 lanes, lane i supplies the address of 4 consecutive
  // 16-bit elements (row i/4 of a 4x16 matrix, columns 4*(i%4)..+3) and lane n receives column n of
  // that matrix (4 rows).  Two reads give the 8 contraction slots of a slab: rows 16t+4g+{0..3} and
  // 16t+8+4g+{0..3} of the 32-row block, for column d = 32*db + 16*(b&1) + n, b = lane/16.
  S1F_DEV static bf16x8 tr(const char *tile, int row32, int t, int db, int lane) {
    const int i = lane & 15, b = lane >> 4, g = lane >> 5;
    const int c = 4 * db + 2 * (b & 1) + ((i & 3) >> 1);
    const int sub = (i & 1) * 8;
    const int r0 = row32 + 16 * t + 4 * g + (i >> 2);
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(S1F_LDS(s16x4, tile + TL::chunk_off(r0, c) + sub));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(S1F_LDS(s16x4, tile + TL::chunk_off(r0 + 8, c) + sub));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
  }
};

template <typename T, int ROWS, int D>
S1F_DEV typename Elem<T>::Frag LdsTile<T, ROWS, D>::nat_frag(const char *tile, int row, int ks, int g) {
  return TileOps<LdsTile<T, ROWS, D>>::nat(tile, row, ks, g);
}
template <typename T, int ROWS, int D>
S1F_DEV typename Elem<T>::Frag LdsTile<T, ROWS, D>::tr_frag(const char *tile, int row32, int t, int db, int lane) {
  return TileOps<LdsTile<T, ROWS, D>>::tr(tile, row32, t, db, lane);
}

// LDS addresses are handled as 32-bit byte offsets (lds_addr) so that address arithmetic, including the
// XOR of the swizzle, stays in the LDS address space.
typedef unsigned lds_addr;
S1F_DEV lds_addr to_lds_addr(const void *p) { return (lds_addr)(uintptr_t)S1F_LDS(const char, p); }
template <typename V> S1F_DEV V lds_load(lds_addr a) {
  return *reinterpret_cast<const __attribute__((address_space(3))) V *>((uintptr_t)a);
}
S1F_DEV const char *lds_generic(lds_addr a) {
  return (const char *)reinterpret_cast<const __attribute__((address_space(3))) char *>((uintptr_t)a);
}

// Returns x through an opaque barrier: values derived from the result are recomputed where they are used
// instead of being kept in registers across a loop (the kernels run at the register limit of two waves
// per SIMD, and the compiler otherwise hoists every loop-invariant lane value it can find).
S1F_DEV int fresh(int x) {
  asm volatile("" : "+v"(x));
  return x;
}

// Reads operand fragments of 32-row blocks out of an LdsTile.  The swizzle depends on the row modulo 16
// only, so for a block starting at a multiple of 16 rows every address is (block base: uniform) combined
// with a lane part computed once, here.  `block` below is the LDS address of the block's first row.
template <typename TL, typename T> struct FragReader;

template <int ROWS, int D> struct FragReader<LdsTile<bf16_t, ROWS, D>, bf16_t> {
  typedef LdsTile<bf16_t, ROWS, D> TL;
  static constexpr int NKS = D / 16, DB = TL::DPAD / 32;
  static constexpr int ROW_BYTES = TL::RS * 16;
  // With 256-byte rows (RS == 16) the swizzle is an XOR on address bits 4..7 that no other term touches,
  // so one lane value per access pattern is enough: fragment ks / d-block db is reached by XOR-ing a
  // compile-time constant into it.  `block` must then be aligned to 8 KiB (the kernels' LDS bases are).
  // Shorter rows keep one precomputed offset per fragment.
  static constexpr bool XOR_FORM = TL::RS == 16;
  unsigned nat_x, tr_x;
  unsigned nat_off[XOR_FORM ? 1 : NKS];
  unsigned tr_off[XOR_FORM ? 1 : DB][2];
  S1F_DEV void init(int lane) {
    const int g = lane >> 5, ln = lane & 31, i = lane & 15, b = lane >> 4;
    const int r0 = 4 * g + (i >> 2), cl = 2 * (b & 1) + ((i & 3) >> 1);
    nat_x = TL::chunk_off(ln, g);                    // fragment ks: nat_x ^ (32 * ks)
    tr_x = TL::chunk_off(r0, cl) + (i & 1) * 8;      // d-block db, row half hh: tr_x ^ (64 * db) ^ (hh * (32 + 2048))
    if (!XOR_FORM) {
#pragma unroll
      for (int ks = 0; ks < NKS; ++ks) nat_off[ks] = TL::chunk_off(ln, 2 * ks + g);
#pragma unroll
      for (int db = 0; db < DB; ++db) {
        tr_off[db][0] = TL::chunk_off(r0, 4 * db + cl) + (i & 1) * 8;
        tr_off[db][1] = TL::chunk_off(r0 + 8, 4 * db + cl) + (i & 1) * 8;
      }
    }
  }
  // contraction along D: row ln of the block, elements [16 ks + 8 g, +8)
  S1F_DEV bf16x8 nat(lds_addr block, int ks) const {
    if (XOR_FORM) return lds_load<bf16x8>((block + nat_x) ^ (unsigned)(32 * ks));
    return lds_load<bf16x8>(block + nat_off[ks]);
  }
  // contraction along the block's rows (slab t), operand index d = 32 db + ln.
  // ds_read_b64_tr_b16: within each group of 16 lanes, lane i supplies the address of 4 consecutive
  // 16-bit elements (row i/4 of a 4x16 matrix, columns 4*(i%4)..+3) and lane n receives column n of
  // that matrix (4 rows).  Two reads give the 8 contraction slots of a slab: rows 16t+4g+{0..3} and
  // 16t+8+4g+{0..3} of the block, for column d = 32*db + 16*(b&1) + n, b = lane/16.
  S1F_DEV bf16x8 tr(lds_addr block, int t, int db) const {
    lds_addr p0, p1;
    if (XOR_FORM) {
      p0 = ((block + tr_x) ^ (unsigned)(64 * db)) + t * 16 * ROW_BYTES;
      p1 = ((block + tr_x) ^ (unsigned)((64 * db) ^ (32 + 2048))) + t * 16 * ROW_BYTES;
    } else {
      p0 = block + t * 16 * ROW_BYTES + tr_off[db][0];
      p1 = block + t * 16 * ROW_BYTES + tr_off[db][1];
    }
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        reinterpret_cast<__attribute__((address_space(3))) s16x4 *>((uintptr_t)p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        reinterpret_cast<__attribute__((address_space(3))) s16x4 *>((uintptr_t)p1));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
  }
  // The same fragment of two blocks `delta` bytes apart (delta a multiple of 8 KiB in the XOR form): the
  // swizzled address is computed once and the second read differs in its immediate offset only.
  S1F_DEV void nat2(lds_addr block, unsigned delta, int ks, bf16x8 &x, bf16x8 &y) const {
    if (XOR_FORM) {
      const lds_addr p = (block + nat_x) ^ (unsigned)(32 * ks);
      x = lds_load<bf16x8>(p);
      y = lds_load<bf16x8>(p + delta);
    } else {
      x = nat(block, ks);
      y = nat(block + delta, ks);
    }
  }
  S1F_DEV static bf16x8 tr_pair(lds_addr p0, lds_addr p1) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        reinterpret_cast<__attribute__((address_space(3))) s16x4 *>((uintptr_t)p0));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
        reinterpret_cast<__attribute__((address_space(3))) s16x4 *>((uintptr_t)p1));
    typedef short s16x8 __attribute__((ext_vector_type(8)));
    s16x8 r = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
    return __builtin_bit_cast(bf16x8, r);
  }
  S1F_DEV void tr2(lds_addr block, unsigned delta, int t, int db, bf16x8 &x, bf16x8 &y) const {
    if (XOR_FORM) {
      const lds_addr q0 = (block + tr_x) ^ (unsigned)(64 * db);
      const lds_addr q1 = (block + tr_x) ^ (unsigned)((64 * db) ^ (32 + 2048));
      const unsigned o = t * 16 * ROW_BYTES;
      x = tr_pair(q0 + o, q1 + o);
      y = tr_pair(q0 + (o + delta), q1 + (o + delta));
    } else {
      x = tr(block, t, db);
      y = tr(block + delta, t, db);
    }
  }
};

template <int ROWS, int D> struct FragReader<LdsTile<float, ROWS, D>, float> {
  typedef LdsTile<float, ROWS, D> TL;
  static constexpr int ROW_BYTES = TL::RS * 16;
  int lane_;
  S1F_DEV void init(int lane) { lane_ = lane; }
  S1F_DEV float nat(lds_addr block, int ks) const { return TL::nat_frag(lds_generic(block), lane_ & 31, ks, lane_ >> 5); }
  S1F_DEV float tr(lds_addr block, int t, int db) const { return TL::tr_frag(lds_generic(block), 0, t, db, lane_); }
  S1F_DEV void nat2(lds_addr block, unsigned delta, int ks, float &x, float &y) const {
    x = nat(block, ks);
    y = nat(block + delta, ks);
  }
  S1F_DEV void tr2(lds_addr block, unsigned delta, int t, int db, float &x, float &y) const {
    x = tr(block, t, db);
    y = tr(block + delta, t, db);
  }
};

// Asynchronous copy of two [ROWS x D] tiles (say a K tile and the V tile right behind it in LDS) from global
// memory straight into LdsTiles (no register staging) by the NW waves of a workgroup.  One
// global_load_lds_dwordx4 moves 16 bytes per lane into 1 KiB of consecutive LDS: lane l lands at
// M0 + immediate offset + 16*l, and the immediate offset is added to the global address as well.  The
// instruction that fills 16-byte slots [64*n, 64*n+64) of a tile makes lane l fetch the chunk that the
// swizzle places in slot 64*n + l.  Each wave fills one contiguous range of the pair of tiles, and up to
// four of its instructions share one value of M0 (told apart by the immediate offset): rewriting M0
// between copies makes them complete one after the other instead of overlapping.  They are written as
// assembly so that the compiler's wait-count pass does not tie later LDS reads of OTHER ring stages to
// these copies; callers order the copies against their readers with wait_async_tiles() + a workgroup
// barrier.  Completion is tracked by the wave's vmcnt.
// The rows of a tile lie `row_stride` apart from one wave-uniform base per tensor: the address is (scalar
// base of the tile) + (32-bit lane offset fixed at init), one register per instruction.  Rows past
// `rows_total` re-read the last valid row (callers mask them); slots of padding columns (head_dim 80)
// re-read a valid chunk of the same row.  (ROWS - 1) * row_stride * sizeof(T) + row bytes must fit 32 bits.
template <typename T, int ROWS, int D, int NW, int GMAX = 4> struct AsyncTilePairU {
  typedef LdsTile<T, ROWS, D> TL;
  static constexpr int SLOTS = ROWS * TL::RS;
  static constexpr int PER = 2 * SLOTS / (64 * NW);
  static constexpr int G = PER < GMAX ? PER : GMAX;    // instructions per group (one value of M0 each)
  static_assert((2 * SLOTS) % (64 * NW) == 0 && SLOTS % (64 * G) == 0, "tiles must split evenly over the waves");
  static_assert(PER % G == 0 && (G == 1 || G == 2 || G == 4), "instructions are issued in groups of one, two or four");
  unsigned voff[PER];   // byte offset of this lane's chunk from the first row of its tile

  S1F_DEV static int slot_row(int wave, int i, int lane) { return (((wave * PER + i) * 64 + lane) % SLOTS) / TL::RS; }

  S1F_DEV void init(int wave, int lane, int64_t row_stride) {
#pragma unroll
    for (int i = 0; i < PER; ++i) {
      const int slot = ((wave * PER + i) * 64 + lane) % SLOTS;
      const int r = slot / TL::RS, pos = slot % TL::RS;
      int c = pos ^ TL::swz(r);
      if (TL::CPR < TL::RS && c >= TL::CPR) c &= TL::RS / 2 - 1;
      voff[i] = (unsigned)((r * row_stride + c * TL::CE) * (int64_t)sizeof(T));
    }
  }

  template <int N>
  S1F_DEV static void issue_group(unsigned dst_, const char *tb_, unsigned o0, unsigned o1, unsigned o2, unsigned o3) {
    // both are wave-uniform by construction; say so where the compiler cannot prove it
    const unsigned dst = __builtin_amdgcn_readfirstlane(dst_);
    const uint64_t tbits = reinterpret_cast<uint64_t>(tb_);
    const char *tb = reinterpret_cast<const char *>(
        ((uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(tbits >> 32)) << 32) |
        (uint64_t)(unsigned)__builtin_amdgcn_readfirstlane((int)(unsigned)tbits));
    if (N == 1)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" : : "s"(dst), "v"(o0), "s"(tb) : "m0");
    else if (N == 2)
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %3\n\t"
                   "global_load_lds_dwordx4 %2, %4 offset:1024"
                   : : "s"(dst), "v"(o0), "v"(o1), "s"(tb), "s"(tb - 1024) : "m0");
    else
      asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %5\n\t"
                   "global_load_lds_dwordx4 %2, %6 offset:1024\n\t"
                   "global_load_lds_dwordx4 %3, %7 offset:2048\n\t"
                   "global_load_lds_dwordx4 %4, %8 offset:3072"
                   : : "s"(dst), "v"(o0), "v"(o1), "v"(o2), "v"(o3), "s"(tb), "s"(tb - 1024), "s"(tb - 2048), "s"(tb - 3072)
                   : "m0");
  }

  // base0/base1: row 0 of the two tensors (wave-uniform); tile_row0: first row of the tile; stage: LDS
  // address of the first tile (the second follows it)
  S1F_DEV void issue(const T *base0, const T *base1, int64_t row_stride, int tile_row0, int rows_total, lds_addr stage,
                     int wave, int lane) const {
#pragma unroll
    for (int p = 0; p < PARTS; ++p) issue_part(p, base0, base1, row_stride, tile_row0, rows_total, stage, wave, lane);
  }
  // One group of up to four of the wave's instructions (0 <= part < PARTS).  Issuing the parts at different
  // points of a tile's computation keeps a wave from queueing behind the copies of its whole workgroup.
  static constexpr int PARTS = PER / G;
  S1F_DEV void issue_part(int part, const T *base0, const T *base1, int64_t row_stride, int tile_row0, int rows_total,
                          lds_addr stage, int wave, int lane) const {
#pragma unroll
    for (int p = 0; p < PARTS; ++p) {
      if (p != part) continue;
      const int i = p * G;
      unsigned off[G];
#pragma unroll
      for (int j = 0; j < G; ++j) off[j] = voff[i + j];
      if (tile_row0 + ROWS > rows_total) {   // the segment ends inside this tile
#pragma unroll
        for (int j = 0; j < G; ++j) {
          const int over = tile_row0 + slot_row(wave, i + j, fresh(lane)) - (rows_total - 1);
          if (over > 0) off[j] -= (unsigned)(over * row_stride * (int64_t)sizeof(T));
        }
      }
      const bool second = (wave * PER + i) * 64 >= SLOTS;     // wave-uniform, the same for the whole group
      const char *tb = reinterpret_cast<const char *>((second ? base1 : base0) + (int64_t)tile_row0 * row_stride);
      const unsigned dst = stage + (unsigned)((wave * PER + i) * 1024);
      issue_group<G>(dst, tb, off[0], off[G > 1 ? 1 : 0], off[G > 2 ? 2 : 0], off[G > 2 ? 3 : 0]);
    }
  }
};

// A [ROWS x D] tile in LDS whose rows are 16 bytes longer than their data: lane ln reading row ln (both
// half-waves, one 16-byte chunk apart) is bank-conflict free without a swizzle, and the fragments along
// D of one lane differ by a compile-time offset only (one address register, no per-fragment arithmetic).
// Used for operands that are copied once through registers and never read transposed.
template <typename T, int ROWS, int D> struct PaddedRows {
  static constexpr int CE = Elem<T>::CE, CPR = D / CE;
  static constexpr int ROW_BYTES = CPR * 16 + 16;
  static constexpr int BYTES = ROWS * ROW_BYTES;
  // rows [0, rows_valid) of `base` (row stride in elements) -> tile; the rest is zero-filled
  template <int NT> S1F_DEV static void copy(char *tile, const T *base, int64_t row_stride, int rows_valid, int tid) {
    constexpr int TOTAL = ROWS * CPR;
    static_assert(TOTAL % NT == 0, "tile must split evenly over the threads");
#pragma unroll
    for (int i = 0; i < TOTAL / NT; ++i) {
      const int id = tid + i * NT, r = id / CPR, c = id % CPR;
      u32x4 v = {0u, 0u, 0u, 0u};
      if (r < rows_valid) v = *reinterpret_cast<const u32x4 *>(base + (int64_t)r * row_stride + c * CE);
      *reinterpret_cast<u32x4 *>(tile + r * ROW_BYTES + c * 16) = v;
    }
  }
  // address of the fragment (row, contraction step 0) of lane (ln, g); step ks lies ks * KSTEP * sizeof(T) further
  S1F_DEV static lds_addr lane_base(lds_addr tile, int row, int g) {
    return tile + (unsigned)(row * ROW_BYTES + g * Elem<T>::EPL * (int)sizeof(T));
  }
  S1F_DEV static typename Elem<T>::Frag frag(lds_addr lane_base_addr, int ks) {
    return lds_load<typename Elem<T>::Frag>(lane_base_addr + (unsigned)(ks * 2 * Elem<T>::EPL * (int)sizeof(T)));
  }
};

// Marks a value loaded from memory as used here.  The compiler then waits for the load at this point
// instead of at the first real use; kernels call it on operands fetched before their main loop, whose
// first use inside the loop would otherwise put a vmcnt wait there that also waits (on every iteration)
// for the asynchronous tile copies in flight.
template <typename V> S1F_DEV void settle(V &v) { asm volatile("" : "+v"(v)); }

// Wait until every asynchronous tile copy issued by this wave has landed (vmcnt(0), other counters untouched).
S1F_DEV void wait_async_tiles() { asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); }
// The same, except that the wave's N most recent copy instructions may still be in flight (loads complete in order).
template <int N> S1F_DEV void wait_async_tiles_but_last() { asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory"); }

// Store 4 consecutive head_dim elements of one row.
template <typename T> S1F_DEV void store4(T *p, float a, float b, float c, float d);
template <> S1F_DEV void store4<float>(float *p, float a, float b, float c, float d) {
  *reinterpret_cast<f32x4 *>(p) = f32x4{a, b, c, d};
}
template <> S1F_DEV void store4<bf16_t>(bf16_t *p, float a, float b, float c, float d) {
  bf16x4 r = {(bf16_t)a, (bf16_t)b, (bf16_t)c, (bf16_t)d};
  *reinterpret_cast<bf16x4 *>(p) = r;
}

// Workgroup id -> (tile, batch*head).  The hardware hands consecutive workgroup ids to the 8 XCDs in turn,
// and each XCD has its own L2.  All tiles of one (batch, head) stream the same K/V prefix (or the same
// Q/dO segment), so they are given ids that land on one XCD: the shared operand is then fetched from HBM once
// per XCD instead of once per workgroup.  An XCD takes n_bh / 8 CONSECUTIVE (batch, head) pairs, so that query
// heads sharing a K/V head share an XCD as well.  Within an XCD the ids run head by head (`tile_major` = 0: best
// when the tiles of a launch take about the same time, i.e. behind a long prefix) or tile by tile over the XCD's
// heads (`tile_major` = 1: the light tiles of every head come last, which shortens the end of a launch whose
// tiles differ a lot, i.e. the first segments; and heads that share K/V rows walk them together).  Falls back to
// the plain order when the number of (batch, head) pairs is not a multiple of 8.
S1F_DEV void decode_workgroup(int id, int n_tiles, int n_bh, int tile_major, int &tile, int &bh) {
  if ((n_bh & 7) == 0) {
    const int xcd = id & 7, slot = id >> 3;
    const int per_xcd = n_bh >> 3;
    const int first = xcd * per_xcd;
    if (tile_major) {
      bh = first + slot % per_xcd;
      tile = slot / per_xcd;
    } else {
      bh = first + slot / n_tiles;
      tile = slot % n_tiles;
    }
  } else {
    bh = id / n_tiles;
    tile = id % n_tiles;
  }
}

// Key-split.  The workgroups of a launch are handed to the chip's workgroup slots in id order; when the last
// round of units fills only part of the slots, the launch ends with most of the chip idle for the length of one
// unit (a row tile against its whole prefix).  The host may therefore cut each of the LAST units of a launch into
// n_split chunks along the keys, which then run side by side; every chunk leaves a partial result in a workspace and a
// small second kernel merges them.  The keys that every row of the unit sees in full (`full`, counted in pieces of the
// kernel's step) are dealt out evenly; the last chunk also takes the pieces on the diagonal.
// In: workgroup id.  Out: unit id, the chunk's piece range [begin, end) and its index in the workspace (-1: whole).
constexpr int kMaxChunks = 8;   // most chunks a unit is ever cut into
struct UnitChunk {
  int unit, chunk, n_chunks, slot;
};
// Chunk-major order: the ids past n_whole first run through one chunk of every split unit, then through the next
// chunk, so that the workgroups that start one after the other walk the SAME keys of neighbouring row tiles and
// share them in the L2 (in unit-major order, a unit's chunks side by side, the workgroups of one key range start
// too far apart for that: 1.5 to 1.7 times the reads from memory over a 32K-token step).  The chunk that holds the diagonal goes first: it is
// the longest.  A chunk keeps its unit's XCD (workgroup ids go to the XCDs in turn, and decode_workgroup ties a unit
// to the XCD of its id) whenever n_whole and the number of split units are multiples of 8, which they are when the
// heads are pinned to XCDs.
S1F_DEV UnitChunk split_unit(int id, int n_whole, int n_split, int n_split_units) {
  if (id < n_whole) return UnitChunk{id, 0, 1, -1};
  const int j = id - n_whole, pass = j / n_split_units, idx = j - pass * n_split_units;
  const int chunk = n_split - 1 - pass;
  return UnitChunk{n_whole + idx, chunk, n_split, chunk * n_split_units + idx};
}
// Workspace index of chunk 0 of split unit number `unit_idx` (counted from n_whole), and the index step to its next chunk.
S1F_DEV void chunk_slots(int unit_idx, int n_split_units, int &first, int &step) {
  first = unit_idx;
  step = n_split_units;
}
S1F_DEV void chunk_range(const UnitChunk &u, int full, int total, int &begin, int &end) {
  begin = u.chunk * full / u.n_chunks;
  end = u.chunk + 1 < u.n_chunks ? (u.chunk + 1) * full / u.n_chunks : total;
}

// Arguments common to the three kernels (all strides in elements of the tensor they index).
struct AttnArgs {
  const void *q, *k, *v, *out, *dout;   // out: written by fwd, read by bwd
  void *out_w, *dq;
  float *lse;                            // [batch, Hq, seg_len]
  float *delta;                          // workspace (bwd): two planes [batch, Hq, seg_len], ws_plane floats apart:
                                         // -lse/scale, then -delta = -rowsum(dO * O)
  int64_t ws_plane;
  float *dk_acc, *dv_acc;
  int64_t q_sb, q_sh, q_ss;
  int64_t kv_sb, kv_sh, kv_ss;
  int32_t seg_off, seg_len;
  int32_t n_q_heads, group;              // group = Hq / Hkv
  int32_t n_tiles, n_bh;                 // launch shape: tiles per (batch, head) and number of (batch, head) pairs
  int32_t tile_major;                    // order of the workgroups within an XCD (see decode_workgroup)
  float scale;                           // 1/sqrt(head_dim)
  // Key-split of the last units of a launch (forward and dQ kernels; see split_unit): workgroup ids below n_whole
  // are whole units; the n_split_units units after them are cut into n_split chunks each.
  int32_t n_whole, n_split, n_split_units;
  float *part;                           // partial results of the chunks: [chunk][split unit][rows per unit][head_dim]
  float *part_ml;                        // forward only: running maximum (log2 units) and row sum, [..][rows per unit][2]
  int64_t part_cap;                      // host side only: most bytes of partial results a launch may plan for
};

}  // namespace s1f
