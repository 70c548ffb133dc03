// In-register unpack + de-quantise of one lane's share of a weight chunk.
//
// This is the "reinterpret, then vectorised cast" half of the paper's weight
// pipeline (Sections "Key Ideas" steps 3-4 and "Efficient Casting"): the bytes
// a lane loaded ARE its codes, and turning them into fp16/bf16 MFMA operands
// uses only shifts, masks and packed arithmetic inside the lane -- no exchange
// with other lanes and no trip through LDS.  The instruction choices below are
// gfx950's (v_and_or_b32, packed-half add/mul, v_fma_mix_f32, v_cvt_pk_bf16_f32)
// rather than the PRMT/LOP3 sequences the paper uses on NVIDIA hardware.
#pragma once
#include <type_traits>

#include "qg_common.h"

namespace qg {

typedef _Float16 h2_t __attribute__((ext_vector_type(2)));
typedef __bf16 b2_t __attribute__((ext_vector_type(2)));
typedef float f2_t __attribute__((ext_vector_type(2)));

__device__ __forceinline__ uint32_t u32(h2_t v) { return __builtin_bit_cast(uint32_t, v); }
__device__ __forceinline__ h2_t as_h2(uint32_t v) { return __builtin_bit_cast(h2_t, v); }

// (a & mask) | orv in one VALU op.  The mask lives in a scalar register, the
// OR operand in a vector register (gfx9 VOP3 reads at most one scalar).
__device__ __forceinline__ uint32_t and_or(uint32_t a, uint32_t mask, uint32_t orv) {
  uint32_t d;
  asm("v_and_or_b32 %0, %1, %2, %3" : "=v"(d) : "v"(a), "s"(mask), "v"(orv));
  return d;
}

template <int S>
__device__ __forceinline__ uint32_t shr(uint32_t x) {
  if constexpr (S == 0) return x;
  else return x >> S;
}
// shift left for S > 0, right for S < 0
template <int S>
__device__ __forceinline__ uint32_t shl_signed(uint32_t x) {
  if constexpr (S == 0) return x;
  else if constexpr (S > 0) return x << S;
  else return x >> (-S);
}

// ---- where pair t lives in the lane's two 16-bit streams -----------------------
template <int BITS>
struct Lay {
  static constexpr int RAW = 4 * BITS;
  // number of codes taken from one shifted view of a register: their bits must
  // fit below bit 10 (the fp16 mantissa), capped at 4 to bound the constants
  static constexpr int WN = (10 / BITS) > 4 ? 4 : (10 / BITS);
  static constexpr uint32_t CODE = (1u << BITS) - 1u;
};

template <int BITS, int T>
struct Pos {
  static constexpr int bit = T * BITS;
  static constexpr int h = bit >> 4;                 // register index
  static constexpr int p = bit & 15;                 // offset inside each 16-bit half
  static constexpr bool straddle = (p + BITS > 16);  // spills into register h+1
  static constexpr int n1 = 16 - p;                  // bits in register h when straddling
  static constexpr int p0 = (BITS - (16 * h) % BITS) % BITS;  // first code starting in h
  static constexpr int idx = (p - p0) / BITS;
  static constexpr int WN = Lay<BITS>::WN;
  static constexpr int widx = straddle ? 0 : idx % WN;         // position inside the view
  static constexpr int s = straddle ? p : p0 + (idx / WN) * WN * BITS;  // view shift
  static constexpr int pp = widx * BITS;                       // offset inside the view
  static_assert(straddle || (p - s == pp && pp + BITS <= 10), "window arithmetic");
};

// fp16 pattern of 2^(10-pp): OR-ing a code placed at mantissa bit pp onto it
// gives the half-precision number 2^(10-pp) + code exactly.
__host__ __device__ constexpr uint32_t magic16(int pp) { return (uint32_t)(25 - pp) << 10; }
__host__ __device__ constexpr uint32_t dup16(uint32_t x) { return x | (x << 16); }

// =============================== integer codes ==================================
// Extract pair T as (2^(10-pp) + q_lo, 2^(10-pp) + q_hi) in packed fp16.
template <int BITS, int T>
__device__ __forceinline__ uint32_t int_pair_magic(const uint32_t (&r)[4 * BITS], const uint32_t (&magic)[Lay<BITS>::WN]) {
  typedef Pos<BITS, T> P;
  if constexpr (!P::straddle) {
    return and_or(shr<P::s>(r[P::h]), dup16(Lay<BITS>::CODE << P::pp), magic[P::widx]);
  } else {
    constexpr int n1 = P::n1;
    uint32_t x = and_or(shr<P::p>(r[P::h]), dup16((1u << n1) - 1u), magic[0]);
    return and_or(r[P::h + 1] << n1, dup16(Lay<BITS>::CODE & ~((1u << n1) - 1u)), x);
  }
}

// ================================ float codes ===================================
// Extract pair T as raw fp16 patterns sign | E (low-aligned in the 5-bit
// exponent field) | M (top-aligned in the mantissa).  The true value is that
// half-precision number times 2^(15 - bias), applied by the caller.
template <int BITS, int EB, int MB, int T>
__device__ __forceinline__ uint32_t float_pair_raw(const uint32_t (&r)[4 * BITS]) {
  typedef Pos<BITS, T> P;
  constexpr uint32_t MAGMASK = dup16(((1u << (BITS - 1)) - 1u) << (10 - MB));
  constexpr uint32_t SIGN = 0x80008000u;
  if constexpr (!P::straddle) {
    uint32_t mag = shl_signed<(10 - MB) - P::p>(r[P::h]) & MAGMASK;
    return and_or(r[P::h] << (16 - P::p - BITS), SIGN, mag);
  } else {
    constexpr int n1 = P::n1;
    uint32_t y = (r[P::h] >> P::p) & dup16((1u << n1) - 1u);
    y = and_or(r[P::h + 1] << n1, dup16(Lay<BITS>::CODE & ~((1u << n1) - 1u)), y);
    uint32_t mag = (y << (10 - MB)) & MAGMASK;
    return and_or(y << (16 - BITS), SIGN, mag);
  }
}

// ===================== float codes with a hardware convert ======================
// Pair T as two exact half-precision values (every e2m1 / e3m2 / e4m3 value is
// representable in fp16).  e3m2 converts a whole k-step (32 codes in 6 registers)
// at once; the compiler merges the identical calls made for the 16 pairs of a step.
typedef _Float16 h32_t __attribute__((ext_vector_type(32)));
typedef uint32_t u6_t __attribute__((ext_vector_type(6)));
template <int WT, int T>
__device__ __forceinline__ h2_t natural_pair(const uint32_t (&r)[4 * wt_bits(WT)]) {
  if constexpr (WT == 13) {
    return __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(r[T / 2], 1.0f, (T % 2) == 1);
  } else if constexpr (WT == 9) {
    return __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(r[T / 4], 1.0f, T % 4);
  } else {
    static_assert(WT == 11, "no hardware convert for this type");
    constexpr int G = T / 16;
    const u6_t six = {r[6 * G + 0], r[6 * G + 1], r[6 * G + 2], r[6 * G + 3], r[6 * G + 4], r[6 * G + 5]};
    const h32_t all = __builtin_amdgcn_cvt_scalef32_pk32_f16_bf6(six, 1.0f);   // "bf6" is e3m2 ("fp6" is e2m3)
    return (h2_t){all[2 * (T % 16)], all[2 * (T % 16) + 1]};
  }
}

// The same converts with a power-of-two block scale (an 8-bit exponent, the shared scale of the
// microscaling types): the hardware multiplies by 2^(exponent of `scale`) while it converts, so
// the de-quantised pair is ONE instruction.  OUT_BF16 picks the 16-bit type of the result.
// Only the two-values-per-instruction converts exist per (scale, pair): e2m1 and e4m3 (the
// 6-bit convert takes one scale for 32 values, which here belong to four columns).
template <int WT, int T, int OUT_BF16>
__device__ __forceinline__ uint32_t natural_pair_mx(const uint32_t (&r)[4 * wt_bits(WT)], float scale) {
  static_assert(WT == 13 || WT == 9, "block-scaled converts exist for e4m3 and e2m1");
  if constexpr (WT == 13) {
    if constexpr (OUT_BF16) return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(r[T / 2], scale, (T % 2) == 1));
    else                    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(r[T / 2], scale, (T % 2) == 1));
  } else {
    if constexpr (OUT_BF16) return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(r[T / 4], scale, T % 4));
    else                    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(r[T / 4], scale, T % 4));
  }
}

// One k-step of 32 rows is one scale block: the lane's four columns have one scale byte each
// (s4, low byte = first column).  2^(e - 127) as fp32 is the byte moved into the exponent field
// (e in 1 .. 254).
struct MxConsts {
  float s[4];
  __device__ __forceinline__ void make(uint32_t s4) {
#pragma unroll
    for (int nt = 0; nt < 4; ++nt) s[nt] = __builtin_bit_cast(float, ((s4 >> (8 * nt)) & 0xffu) << 23);
  }
};
template <int WT, int OUT_BF16, int J, int NT>
__device__ __forceinline__ void frag_mx(const uint32_t (&r)[4 * wt_bits(WT)], const MxConsts& gc, uint32_t (&out)[4]) {
  constexpr int T0 = LayoutOf<0>::t0(J, NT);
  out[0] = natural_pair_mx<WT, T0 + 0, OUT_BF16>(r, gc.s[NT]);
  out[1] = natural_pair_mx<WT, T0 + 1, OUT_BF16>(r, gc.s[NT]);
  out[2] = natural_pair_mx<WT, T0 + 2, OUT_BF16>(r, gc.s[NT]);
  out[3] = natural_pair_mx<WT, T0 + 3, OUT_BF16>(r, gc.s[NT]);
}

// ============================ per-group constants ================================
// sraw: the lane's 16-bit scales (its NTL adjacent columns, low bits first), zraw:
// its zero-point bytes.  Built once per (chunk, group), used by 8 or 16 pairs each.
template <int WT, int ROUTE, int LY = 0, bool LUT = wt_is_lut(WT)>
struct Decoder;

// ---- integers, fp16 route:  w = ((2^e + q) - (2^e + z')) * s ------------------
template <int WT, int LY>
struct Decoder<WT, ROUTE_F16, LY, false> {
  static constexpr int NTL = LayoutOf<LY>::NT;     // columns per lane
  static constexpr int BITS = wt_bits(WT);
  static constexpr bool IS_FLOAT = wt_is_float(WT);
  static constexpr bool NATURAL = wt_natural(WT);
  static constexpr int EB = wt_ebits(WT), MB = wt_mbits(WT);
  static constexpr int WN = Lay<BITS>::WN;
  static constexpr int RAW = 4 * BITS;
  static constexpr bool HAS_META = true;           // scales / zero-points are loaded with every chunk
  static constexpr bool IS_MX = false;
  static constexpr bool IS_LUT = false;

  struct Consts {
    h2_t s[NTL];
    h2_t c[WN][NTL];   // integers: 2^(10-pp) + z'   (floats: unused)
  };
  struct Uniform {
    uint32_t magic[WN];
    __device__ __forceinline__ void init() {
#pragma unroll
      for (int w = 0; w < WN; ++w) magic[w] = dup16(magic16(w * BITS));
    }
  };

  // constants of one of the lane's columns (callers that spread the work over
  // several places build column by column)
  static __device__ __forceinline__ void make_col(Consts& gc, int nt, uint2 sraw, uint32_t zraw, int zbias, int /*scale_bf16*/) {
    const uint32_t sw = (nt >> 1) ? sraw.y : sraw.x;
    const uint32_t s16 = (nt & 1) ? (sw >> 16) : (sw & 0xffffu);
    gc.s[nt] = as_h2(s16 | (s16 << 16));
    if constexpr (!IS_FLOAT) {
      uint32_t z = ((zraw >> (8 * nt)) & 0xffu) + (uint32_t)zbias;   // < 1024
      h2_t c0 = as_h2(dup16(0x6400u) | z | (z << 16));               // 1024 + z', exact
      gc.c[0][nt] = c0;
#pragma unroll
      for (int w = 1; w < WN; ++w) {
        const _Float16 d = (_Float16)(float)((1 << (10 - w * BITS)) - 1024);
        gc.c[w][nt] = c0 + (h2_t){d, d};                             // exact: integers < 2048
      }
    }
  }
  static __device__ __forceinline__ void make_consts(Consts& gc, uint2 sraw, uint32_t zraw, int zbias, int scale_bf16) {
#pragma unroll
    for (int nt = 0; nt < NTL; ++nt) make_col(gc, nt, sraw, zraw, zbias, scale_bf16);
  }

  // The same pair in three separately schedulable phases (extract / centre or
  // re-bias / scale-and-round), so that a caller can slot them between matrix
  // instructions.
  typedef uint32_t Ext;
  typedef h2_t Mid;
  template <int T>
  static __device__ __forceinline__ uint32_t pair_e(const uint32_t (&r)[RAW], const Uniform& u) {
    if constexpr (NATURAL) return u32(natural_pair<WT, T>(r));
    else if constexpr (!IS_FLOAT) return int_pair_magic<BITS, T>(r, u.magic);
    else return float_pair_raw<BITS, EB, MB, T>(r);
  }
  template <int T>
  static __device__ __forceinline__ Mid pair_s(uint32_t x, const Consts& gc, int nt) {
    if constexpr (NATURAL) return as_h2(x);
    else if constexpr (!IS_FLOAT) return as_h2(x) - gc.c[Pos<BITS, T>::widx][nt];
    else {
      constexpr int ADJ = 15 - ((1 << (EB - 1)) - 1);
      const _Float16 a = (_Float16)(float)(1 << ADJ);
      return as_h2(x) * (h2_t){a, a};
    }
  }
  static __device__ __forceinline__ uint32_t pair_p(Mid m, const Consts& gc, int nt) { return u32(m * gc.s[nt]); }

  // one register (two values) of the MFMA operand: pair T, which belongs to sub-tile nt
  template <int T>
  static __device__ __forceinline__ uint32_t pair(const uint32_t (&r)[RAW], const Consts& gc, const Uniform& u, int nt) {
    if constexpr (NATURAL) {
      return u32(natural_pair<WT, T>(r) * gc.s[nt]);          // exact value, one rounding multiply
    } else if constexpr (!IS_FLOAT) {
      uint32_t x = int_pair_magic<BITS, T>(r, u.magic);
      return u32((as_h2(x) - gc.c[Pos<BITS, T>::widx][nt]) * gc.s[nt]);
    } else {
      constexpr int ADJ = 15 - ((1 << (EB - 1)) - 1);
      const _Float16 a = (_Float16)(float)(1 << ADJ);
      const h2_t adj = {a, a};
      return u32((as_h2(float_pair_raw<BITS, EB, MB, T>(r)) * adj) * gc.s[nt]);
    }
  }

  // the four registers (8 values) lane feeds to the MFMA for k-step J, sub-tile NT
  template <int J, int NT>
  static __device__ __forceinline__ void frag(const uint32_t (&r)[RAW], const Consts& gc, const Uniform& u, uint32_t (&out)[4]) {
    constexpr int T0 = LayoutOf<LY>::t0(J, NT);
    if constexpr (NATURAL) {
      out[0] = pair<T0 + 0>(r, gc, u, NT);
      out[1] = pair<T0 + 1>(r, gc, u, NT);
      out[2] = pair<T0 + 2>(r, gc, u, NT);
      out[3] = pair<T0 + 3>(r, gc, u, NT);
    } else if constexpr (!IS_FLOAT) {
      uint32_t x0 = int_pair_magic<BITS, T0 + 0>(r, u.magic);
      uint32_t x1 = int_pair_magic<BITS, T0 + 1>(r, u.magic);
      uint32_t x2 = int_pair_magic<BITS, T0 + 2>(r, u.magic);
      uint32_t x3 = int_pair_magic<BITS, T0 + 3>(r, u.magic);
      out[0] = u32((as_h2(x0) - gc.c[Pos<BITS, T0 + 0>::widx][NT]) * gc.s[NT]);
      out[1] = u32((as_h2(x1) - gc.c[Pos<BITS, T0 + 1>::widx][NT]) * gc.s[NT]);
      out[2] = u32((as_h2(x2) - gc.c[Pos<BITS, T0 + 2>::widx][NT]) * gc.s[NT]);
      out[3] = u32((as_h2(x3) - gc.c[Pos<BITS, T0 + 3>::widx][NT]) * gc.s[NT]);
    } else {
      // value = raw * 2^(15-bias) exactly (every supported format fits fp16),
      // then one rounding multiply by the scale
      constexpr int ADJ = 15 - ((1 << (EB - 1)) - 1);
      const _Float16 a = (_Float16)(float)(1 << ADJ);
      const h2_t adj = {a, a};
      out[0] = u32((as_h2(float_pair_raw<BITS, EB, MB, T0 + 0>(r)) * adj) * gc.s[NT]);
      out[1] = u32((as_h2(float_pair_raw<BITS, EB, MB, T0 + 1>(r)) * adj) * gc.s[NT]);
      out[2] = u32((as_h2(float_pair_raw<BITS, EB, MB, T0 + 2>(r)) * adj) * gc.s[NT]);
      out[3] = u32((as_h2(float_pair_raw<BITS, EB, MB, T0 + 3>(r)) * adj) * gc.s[NT]);
    }
  }
};

// ---- bf16 route:  w = bf16_rne( fma(x, s, -(2^e + z') * s) ), all exact in fp32 --
template <int WT, int LY>
struct Decoder<WT, ROUTE_BF16, LY, false> {
  static constexpr int NTL = LayoutOf<LY>::NT;     // columns per lane
  static constexpr int BITS = wt_bits(WT);
  static constexpr bool IS_FLOAT = wt_is_float(WT);
  static constexpr bool NATURAL = wt_natural(WT);
  static constexpr int EB = wt_ebits(WT), MB = wt_mbits(WT);
  static constexpr int WN = Lay<BITS>::WN;
  static constexpr int RAW = 4 * BITS;
  static constexpr bool HAS_META = true;           // scales / zero-points are loaded with every chunk
  static constexpr bool IS_MX = false;
  static constexpr bool IS_LUT = false;

  struct Consts {
    float s[NTL];     // integers: scale; floats: scale * 2^(15-bias)
    float ncs[WN][NTL];  // integers: -(2^(10-pp) + z') * s, exact (<= 22 bits)
  };
  struct Uniform {
    uint32_t magic[WN];
    __device__ __forceinline__ void init() {
#pragma unroll
      for (int w = 0; w < WN; ++w) magic[w] = dup16(magic16(w * BITS));
    }
  };

  static __device__ __forceinline__ void make_col(Consts& gc, int nt, uint2 sraw, uint32_t zraw, int zbias, int scale_bf16) {
    const uint32_t sw = (nt >> 1) ? sraw.y : sraw.x;
    const uint32_t s16 = (nt & 1) ? (sw >> 16) : (sw & 0xffffu);
    // widen the 16-bit scale exactly; both forms are computed and one is
    // selected with a mask so that no branch lands in the pipelined loops
    const uint32_t from_h = __builtin_bit_cast(uint32_t, (float)__builtin_bit_cast(_Float16, (uint16_t)s16));
    const uint32_t sel = scale_bf16 ? 0xffffffffu : 0u;
    float s = __builtin_bit_cast(float, ((s16 << 16) & sel) | (from_h & ~sel));
    if constexpr (!IS_FLOAT) {
      gc.s[nt] = s;
      float z = (float)(int)(((zraw >> (8 * nt)) & 0xffu) + (uint32_t)zbias);
#pragma unroll
      for (int w = 0; w < WN; ++w) gc.ncs[w][nt] = -((float)(1 << (10 - w * BITS)) + z) * s;
    } else if constexpr (NATURAL) {
      gc.s[nt] = s;
    } else {
      constexpr int ADJ = 15 - ((1 << (EB - 1)) - 1);
      gc.s[nt] = s * (float)(1 << ADJ);
    }
  }
  static __device__ __forceinline__ void make_consts(Consts& gc, uint2 sraw, uint32_t zraw, int zbias, int scale_bf16) {
#pragma unroll
    for (int nt = 0; nt < NTL; ++nt) make_col(gc, nt, sraw, zraw, zbias, scale_bf16);
  }

  static __device__ __forceinline__ uint32_t pk_bf16(float lo, float hi) {
    f2_t f = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, b2_t));
  }

  typedef uint32_t Ext;
  typedef f2_t Mid;
  template <int T>
  static __device__ __forceinline__ uint32_t pair_e(const uint32_t (&r)[RAW], const Uniform& u) {
    if constexpr (NATURAL) return u32(natural_pair<WT, T>(r));
    else if constexpr (!IS_FLOAT) return int_pair_magic<BITS, T>(r, u.magic);
    else return float_pair_raw<BITS, EB, MB, T>(r);
  }
  template <int T>
  static __device__ __forceinline__ Mid pair_s(uint32_t xb, const Consts& gc, int nt) {
    h2_t x = as_h2(xb);
    if constexpr (!IS_FLOAT) {
      constexpr int w = Pos<BITS, T>::widx;
      return (f2_t){__builtin_fmaf((float)x.x, gc.s[nt], gc.ncs[w][nt]), __builtin_fmaf((float)x.y, gc.s[nt], gc.ncs[w][nt])};
    } else {
      // x * s as fma(x, s, -0): one mixed-precision op; adding -0 keeps the sign of a zero product
      return (f2_t){__builtin_fmaf((float)x.x, gc.s[nt], -0.0f), __builtin_fmaf((float)x.y, gc.s[nt], -0.0f)};
    }
  }
  static __device__ __forceinline__ uint32_t pair_p(Mid m, const Consts&, int) { return pk_bf16(m.x, m.y); }

  // one register (two values) of the MFMA operand: pair T, which belongs to sub-tile nt
  template <int T>
  static __device__ __forceinline__ uint32_t pair(const uint32_t (&r)[RAW], const Consts& gc, const Uniform& u, int nt) {
    if constexpr (!IS_FLOAT) {
      h2_t x = as_h2(int_pair_magic<BITS, T>(r, u.magic));
      constexpr int w = Pos<BITS, T>::widx;
      return pk_bf16(__builtin_fmaf((float)x.x, gc.s[nt], gc.ncs[w][nt]),
                     __builtin_fmaf((float)x.y, gc.s[nt], gc.ncs[w][nt]));
    } else {
      h2_t x;
      if constexpr (NATURAL) x = natural_pair<WT, T>(r);
      else x = as_h2(float_pair_raw<BITS, EB, MB, T>(r));
      return pk_bf16(__builtin_fmaf((float)x.x, gc.s[nt], -0.0f), __builtin_fmaf((float)x.y, gc.s[nt], -0.0f));
    }
  }

  template <int J, int NT>
  static __device__ __forceinline__ void frag(const uint32_t (&r)[RAW], const Consts& gc, const Uniform& u, uint32_t (&out)[4]) {
    constexpr int T0 = LayoutOf<LY>::t0(J, NT);
    if constexpr (!IS_FLOAT) {
#define QG_ONE(V)                                                                         \
  {                                                                                       \
    h2_t x = as_h2(int_pair_magic<BITS, T0 + V>(r, u.magic));                            \
    constexpr int w = Pos<BITS, T0 + V>::widx;                                            \
    out[V] = pk_bf16(__builtin_fmaf((float)x.x, gc.s[NT], gc.ncs[w][NT]),                 \
                     __builtin_fmaf((float)x.y, gc.s[NT], gc.ncs[w][NT]));                \
  }
      QG_ONE(0) QG_ONE(1) QG_ONE(2) QG_ONE(3)
#undef QG_ONE
    } else {
      out[0] = pair<T0 + 0>(r, gc, u, NT);
      out[1] = pair<T0 + 1>(r, gc, u, NT);
      out[2] = pair<T0 + 2>(r, gc, u, NT);
      out[3] = pair<T0 + 3>(r, gc, u, NT);
    }
  }
};

// ===================================== codebook lookup ==========================================
// The paper's closing section says a lookup instruction would accommodate codebook quantisation:
// a code is an index into a table of 2^BITS levels.  Here the lookup is one LDS read.  Up to 4 bits
// the table is indexed by a PAIR of codes (the two k values of one operand register, adjacent in
// the lane's bit stream) and returns both levels, already packed the way the matrix instruction
// reads them: a bit-field extract, an address and one 4-byte read per pair.  From 5 bits on a
// pair table would not fit; each code is looked up by itself with a 16-bit read into its half of
// the register.  Every entry is stored 32 times, entry e of copy c at dword 32*e + c, and lane l
// reads copy l % 32: the 32 lanes the LDS serves together then hit 32 different banks whatever
// their codes are.  The levels are half precision; the group scale multiplies them with the
// one rounding of the other types (fp16: packed-half multiply; bf16: exact fp32 product, hardware
// fp32 -> bf16 rounding).  No zero-points.
typedef __attribute__((address_space(3))) const uint32_t* lds_u32_ptr;
typedef __attribute__((address_space(3))) const _Float16* lds_h_ptr;

template <int WT, int ROUTE, int LY>
struct Decoder<WT, ROUTE, LY, true> {
  static_assert(LY == 0, "codebook indices exist on the first layout");
  static constexpr int NTL = 4;
  static constexpr int BITS = wt_bits(WT);
  static constexpr int RAW = 4 * BITS;
  static constexpr bool HAS_META = true;
  static constexpr bool IS_MX = false;
  static constexpr bool IS_LUT = true;
  static constexpr bool PAIRED = BITS <= 4;
  static constexpr int IDX_BITS = PAIRED ? 2 * BITS : BITS;
  static constexpr int ENTRIES = 1 << IDX_BITS;
  static constexpr int TABLE_DWORDS = ENTRIES * 32;        // 32 copies
  static constexpr int LEVELS = 1 << BITS;

  struct Consts {
    h2_t s[NTL];       // fp16 route
    float f[NTL];      // bf16 route
  };
  struct Uniform {
    uint32_t base;     // LDS byte address of entry 0 of the lane's copy
    __device__ __forceinline__ void init() { base = 0; }
    __device__ __forceinline__ void set_table(const uint32_t* table, int lane) {
      base = (uint32_t)(uintptr_t)(lds_u32_ptr)table + 4u * (uint32_t)(lane & 31);
    }
  };

  // Builds the replicated table from the 2^BITS levels, in two steps so that a kernel can start
  // its first weight loads in between: fetch() reads this thread's level (workgroups have at
  // least 256 threads, so one each covers the table), build() places it in `stage` (256 halves
  // of LDS) and writes the entries to `table` (TABLE_DWORDS dwords of LDS).  Every thread of the
  // workgroup calls both; build() contains two workgroup barriers.
  static __device__ __forceinline__ uint32_t fetch(const uint16_t* levels, int tid) {
    return levels[tid < LEVELS ? tid : 0];
  }
  static __device__ __forceinline__ void build(uint32_t* table, uint16_t* stage, uint32_t level, int tid, int nthreads) {
    if (tid < LEVELS) stage[tid] = (uint16_t)level;
    __syncthreads();
    for (int i = tid; i < TABLE_DWORDS; i += nthreads) {
      const int e = i >> 5;
      if constexpr (PAIRED) table[i] = (uint32_t)stage[e & (LEVELS - 1)] | ((uint32_t)stage[e >> BITS] << 16);
      else table[i] = stage[e];
    }
    __syncthreads();
  }

  static __device__ __forceinline__ void make_col(Consts& gc, int nt, uint2 sraw, uint32_t, int, int scale_bf16) {
    const uint32_t sw = (nt >> 1) ? sraw.y : sraw.x;
    const uint32_t s16 = (nt & 1) ? (sw >> 16) : (sw & 0xffffu);
    if constexpr (ROUTE == ROUTE_F16) {
      gc.s[nt] = as_h2(s16 | (s16 << 16));
    } else {
      const uint32_t from_h = __builtin_bit_cast(uint32_t, (float)__builtin_bit_cast(_Float16, (uint16_t)s16));
      const uint32_t sel = scale_bf16 ? 0xffffffffu : 0u;
      gc.f[nt] = __builtin_bit_cast(float, ((s16 << 16) & sel) | (from_h & ~sel));
    }
  }
  static __device__ __forceinline__ void make_consts(Consts& gc, uint2 sraw, uint32_t zraw, int zbias, int scale_bf16) {
#pragma unroll
    for (int nt = 0; nt < NTL; ++nt) make_col(gc, nt, sraw, zraw, zbias, scale_bf16);
  }

  // LDS address of the entry that element E (IDX_BITS wide) of the lane's bit stream selects
  template <int E>
  static __device__ __forceinline__ uint32_t entry_addr(const uint32_t (&r)[RAW], const Uniform& u) {
    constexpr int bit = E * IDX_BITS, w = bit >> 5, sh = bit & 31;
    uint32_t x;
    if constexpr (sh + IDX_BITS <= 32) x = shr<sh>(r[w]);
    else x = (r[w] >> sh) | (r[w + 1] << (32 - sh));
    return ((x & (uint32_t)(ENTRIES - 1)) << 7) + u.base;
  }

  // "extract" = the lookup itself: address arithmetic and the LDS read(s), whose results stay in
  // flight until "round" uses them (the tiled kernel places that five matrix instructions later);
  // "centre" has nothing to do; "round" = merge the two halves of a pair looked up code by code,
  // then the one rounding multiply by the scale.
  struct Two { _Float16 lo, hi; };
  typedef typename std::conditional<PAIRED, uint32_t, Two>::type Ext;
  typedef Ext Mid;
  template <int T>
  static __device__ __forceinline__ Ext pair_e(const uint32_t (&r)[RAW], const Uniform& u) {
    if constexpr (PAIRED) {
      return *reinterpret_cast<lds_u32_ptr>(entry_addr<T>(r, u));
    } else {
      Two v;
      v.lo = *reinterpret_cast<lds_h_ptr>(entry_addr<2 * T>(r, u));
      v.hi = *reinterpret_cast<lds_h_ptr>(entry_addr<2 * T + 1>(r, u));
      return v;
    }
  }
  template <int T>
  static __device__ __forceinline__ Mid pair_s(Ext x, const Consts&, int) { return x; }
  static __device__ __forceinline__ uint32_t pair_p(Mid m, const Consts& gc, int nt) {
    h2_t x;
    if constexpr (PAIRED) x = as_h2(m);
    else x = (h2_t){m.lo, m.hi};
    if constexpr (ROUTE == ROUTE_F16) {
      return u32(x * gc.s[nt]);
    } else {
      // level * scale is exact in fp32 (11 x 11 significant bits); adding -0 keeps the sign of a zero product
      f2_t f = {__builtin_fmaf((float)x.x, gc.f[nt], -0.0f), __builtin_fmaf((float)x.y, gc.f[nt], -0.0f)};
      return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, b2_t));
    }
  }
  template <int J, int NT>
  static __device__ __forceinline__ void frag(const uint32_t (&r)[RAW], const Consts& gc, const Uniform& u, uint32_t (&out)[4]) {
    constexpr int T0 = LayoutOf<0>::t0(J, NT);
    const Ext x0 = pair_e<T0 + 0>(r, u), x1 = pair_e<T0 + 1>(r, u), x2 = pair_e<T0 + 2>(r, u), x3 = pair_e<T0 + 3>(r, u);
    out[0] = pair_p(x0, gc, NT);
    out[1] = pair_p(x1, gc, NT);
    out[2] = pair_p(x2, gc, NT);
    out[3] = pair_p(x3, gc, NT);
  }
};

// ================= weights already de-quantised (the paper's prefill variant) ==================
// For prefill-sized batches the paper decodes the quantised weight to float16 once and runs a
// standard 16-bit matmul (Section "End-to-End Performance").  Here the de-quantiser can write its
// result in "fragment order" -- the 16-bit image of the first device layout: chunk (kc, nc) is
// 16 pieces of 1024 bytes, piece 4*j + nt holds, for lane l at bytes [16*l, 16*l + 16), the four
// registers the lane feeds to the matrix instruction for k-step j and sub-tile nt -- and the tiled
// kernel then runs with this pass-through "decoder": the same kernel with the unpack removed.
template <int ROUTE>
struct DenseDecoder {
  static constexpr int NTL = 4, BITS = 16, RAW = 64;
  static constexpr bool HAS_META = false;
  static constexpr bool IS_MX = false;
  static constexpr bool IS_LUT = false;
  struct Consts {};
  struct Uniform { __device__ __forceinline__ void init() {} };
  typedef uint32_t Ext;
  typedef uint32_t Mid;
  static __device__ __forceinline__ void make_col(Consts&, int, uint2, uint32_t, int, int) {}
  template <int T>
  static __device__ __forceinline__ uint32_t pair_e(const uint32_t (&r)[RAW], const Uniform&) { return r[T]; }
  template <int T>
  static __device__ __forceinline__ Mid pair_s(uint32_t x, const Consts&, int) { return x; }
  static __device__ __forceinline__ uint32_t pair_p(Mid m, const Consts&, int) { return m; }
  template <int J, int NT>
  static __device__ __forceinline__ void frag(const uint32_t (&r)[RAW], const Consts&, const Uniform&, uint32_t (&out)[4]) {
    constexpr int T0 = LayoutOf<0>::t0(J, NT);
    out[0] = r[T0]; out[1] = r[T0 + 1]; out[2] = r[T0 + 2]; out[3] = r[T0 + 3];
  }
};

// Block-scaled e2m1 / e4m3 in the three-phase form the tiled kernel deals out over its gaps:
// "extract" picks the register that holds the pair, "centre" is the one scaled hardware convert,
// "round" has nothing left to do.  The lane's four scale bytes of a 32-row block travel in the
// zero-point slot of the weight stage.
template <int WT, int ROUTE>
struct MxDecoder {
  static constexpr int NTL = 4, BITS = wt_bits(WT), RAW = 4 * BITS;
  static constexpr bool HAS_META = true;
  static constexpr bool IS_MX = true;
  static constexpr bool IS_LUT = false;
  static_assert(WT == 9 || WT == 13, "block-scaled converts exist for e2m1 and e4m3");
  struct Consts { float s[4]; };
  struct Uniform { __device__ __forceinline__ void init() {} };
  typedef uint32_t Ext;
  typedef uint32_t Mid;
  static __device__ __forceinline__ void make_col(Consts& gc, int nt, uint2, uint32_t s4, int, int) {
    gc.s[nt] = __builtin_bit_cast(float, ((s4 >> (8 * nt)) & 0xffu) << 23);
  }
  template <int T>
  static __device__ __forceinline__ uint32_t pair_e(const uint32_t (&r)[RAW], const Uniform&) { return r[WT == 13 ? T / 2 : T / 4]; }
  template <int T>
  static __device__ __forceinline__ Mid pair_s(uint32_t x, const Consts& gc, int nt) {
    constexpr int OUT_BF16 = (ROUTE == ROUTE_BF16);
    if constexpr (WT == 13) {
      if constexpr (OUT_BF16) return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp8(x, gc.s[nt], (T % 2) == 1));
      else                    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp8(x, gc.s[nt], (T % 2) == 1));
    } else {
      if constexpr (OUT_BF16) return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_bf16_fp4(x, gc.s[nt], T % 4));
      else                    return __builtin_bit_cast(uint32_t, __builtin_amdgcn_cvt_scalef32_pk_f16_fp4(x, gc.s[nt], T % 4));
    }
  }
  static __device__ __forceinline__ uint32_t pair_p(Mid m, const Consts&, int) { return m; }
  template <int J, int NT>
  static __device__ __forceinline__ void frag(const uint32_t (&r)[RAW], const Consts& gc, const Uniform& u, uint32_t (&out)[4]) {
    constexpr int T0 = LayoutOf<0>::t0(J, NT);
    out[0] = pair_s<T0 + 0>(pair_e<T0 + 0>(r, u), gc, NT);
    out[1] = pair_s<T0 + 1>(pair_e<T0 + 1>(r, u), gc, NT);
    out[2] = pair_s<T0 + 2>(pair_e<T0 + 2>(r, u), gc, NT);
    out[3] = pair_s<T0 + 3>(pair_e<T0 + 3>(r, u), gc, NT);
  }
};

template <int WT, int ROUTE, bool MX = false>
struct DecoderFor { typedef Decoder<WT, ROUTE, 0> type; };
template <int ROUTE>
struct DecoderFor<WT_DENSE16, ROUTE, false> { typedef DenseDecoder<ROUTE> type; };
template <int ROUTE>
struct DecoderFor<9, ROUTE, true> { typedef MxDecoder<9, ROUTE> type; };
template <int ROUTE>
struct DecoderFor<13, ROUTE, true> { typedef MxDecoder<13, ROUTE> type; };

}  // namespace qg
