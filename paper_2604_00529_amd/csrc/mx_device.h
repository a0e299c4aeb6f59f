// Device-side building blocks of the MX kernels (gfx950 only): element-format traits, the
// shared-scale rule of Eq. (1), element encode / decode (Eq. (2), Sec. 3.3 notation), the
// Slice-and-Scale element maps of Eq. (4) / Eq. (6), and bit packing.
//
// OCP element formats (E4M3, E3M2, E2M3, E2M1) go through the CDNA4 scaled conversion
// instructions, whose scale operand is an fp32 of which only the exponent field is used: the
// bit pattern (byte << 23) is exactly the E8M0 scale 2^(byte-127), byte 0 included.  Those
// instructions round to nearest even and saturate (FP8 only with MODE.FP16_OVFL set).  Integer
// elements, the non-OCP minifloats (E3M3, E2M2) and the non-default tie rules use integer code.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

#include "mx.h"

namespace mx {

typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef float f32x32 __attribute__((ext_vector_type(32)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x6 __attribute__((ext_vector_type(6)));
typedef short i16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x32 __attribute__((ext_vector_type(32)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Compile-time loop: the byte / word selectors of the conversion builtins must be constants.
template <int I, int N, typename F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (I < N) {
    f(std::integral_constant<int, I>{});
    static_for<I + 1, N>(f);
  }
}

enum { HW_NONE = 0, HW_FP8 = 1, HW_FP4 = 2, HW_FP6 = 3, HW_BF6 = 4 };

// ------------------------------------------------------------------ element traits
template <int ELEM>
struct Elem;

#define MX_DEF_INT(ID, B)                                          \
  template <>                                                      \
  struct Elem<ID> {                                                \
    static constexpr bool is_int = true;                           \
    static constexpr int bits = B, eta = 0, mu = 0, bias = 0;      \
    static constexpr int emax = B - 2; /* integer view, Eq. (4) */ \
    static constexpr int hw = HW_NONE;                             \
    static constexpr bool has_nan = false;                         \
  };
#define MX_DEF_FP(ID, ETA, MU, HW)                                                            \
  template <>                                                                                 \
  struct Elem<ID> {                                                                           \
    static constexpr bool is_int = false;                                                     \
    static constexpr int bits = 1 + ETA + MU, eta = ETA, mu = MU;                             \
    static constexpr int bias = (1 << (ETA - 1)) - 1;                                         \
    static constexpr int emax = 1 << (ETA - 1); /* exponent of the largest normal */          \
    static constexpr int hw = HW;                                                             \
    static constexpr bool has_nan = (ETA == 4 && MU == 3);                                    \
  };
MX_DEF_INT(MX_INT8, 8)
MX_DEF_INT(MX_INT7, 7)
MX_DEF_INT(MX_INT6, 6)
MX_DEF_INT(MX_INT5, 5)
MX_DEF_INT(MX_INT4, 4)
MX_DEF_INT(MX_INT3, 3)
MX_DEF_INT(MX_INT2, 2)
MX_DEF_FP(MX_FP8_E4M3, 4, 3, HW_FP8)
MX_DEF_FP(MX_FP7_E3M3, 3, 3, HW_NONE)
MX_DEF_FP(MX_FP6_E3M2, 3, 2, HW_BF6)
MX_DEF_FP(MX_FP6_E2M3, 2, 3, HW_FP6)
MX_DEF_FP(MX_FP5_E2M2, 2, 2, HW_NONE)
MX_DEF_FP(MX_FP4_E2M1, 2, 1, HW_FP4)
#undef MX_DEF_INT
#undef MX_DEF_FP

// ------------------------------------------------------------------ scales (Eq. (1))
__device__ __forceinline__ uint32_t abs_bits(float v) { return __float_as_uint(v) & 0x7FFFFFFFu; }

// E8M0 byte of a block from the largest |V_i| given as fp32 bits (sign cleared).  The integer
// order of those bit patterns is the order of the magnitudes, NaN / Inf sort above every finite
// value and mark the block with byte 255.  floor(log2) is the exponent field for normals and
// comes from the leading-zero count for fp32 subnormals; zero falls out as byte 0 by the clamp.
template <int EMAX>
__device__ __forceinline__ uint32_t scale_byte_from_amax(uint32_t a) {
  if (a >= 0x7F800000u) return 255u;
  int e = (a >> 23) ? (int)(a >> 23) - 127 : (31 - (int)__clz(a)) - 149;
  int s = e - EMAX;
  s = s < -127 ? -127 : s;
  s = s > 127 ? 127 : s;
  return (uint32_t)(s + 127);
}

// fp32 whose exponent field is the E8M0 byte: the form the scaled conversions take.
__device__ __forceinline__ float scale_operand(uint32_t byte) { return __uint_as_float(byte << 23); }

// Saturating FP8 conversion needs MODE.FP16_OVFL = 1 (otherwise values above the largest normal
// become NaN codes).  `dep` is any value every later address depends on: routing it through the
// statement keeps the conversions after the mode write.
__device__ __forceinline__ int set_fp8_saturation(int dep) {
  asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 23, 1), 1" : "+v"(dep));
  return dep;
}

// ------------------------------------------------------------------ 32-element FP6 conversions
// These instructions read 16 consecutive registers and write 6.  They are issued
// through inline assembly with an early-clobber destination and with every source lane defined,
// so that the register allocator can never overlay the destination, the scale or another operand
// on (otherwise unused) source lanes: with such overlays the results were wrong.
template <bool BF6>
__device__ __forceinline__ u32x6 cvt_2xpk16_fp6_f32(f32x16 a, f32x16 b, float s) {
  u32x6 d;
  if constexpr (BF6) asm("v_cvt_scalef32_2xpk16_bf6_f32 %0, %1, %2, %3" : "=&v"(d) : "v"(a), "v"(b), "v"(s));
  else asm("v_cvt_scalef32_2xpk16_fp6_f32 %0, %1, %2, %3" : "=&v"(d) : "v"(a), "v"(b), "v"(s));
  return d;
}
template <bool BF6>
__device__ __forceinline__ u32x6 cvt_pk32_fp6_f16(f16x32 a, float s) {
  u32x6 d;
  if constexpr (BF6) asm("v_cvt_scalef32_pk32_bf6_f16 %0, %1, %2" : "=&v"(d) : "v"(a), "v"(s));
  else asm("v_cvt_scalef32_pk32_fp6_f16 %0, %1, %2" : "=&v"(d) : "v"(a), "v"(s));
  return d;
}
// 32 FP6 codes (6 dwords) times the E8M0 scale -> 32 bf16 (16 dwords), exact for every code and scale byte
// (the products have at most 4 significant bits; subnormal results included -- enumerated on the GPU).
typedef uint32_t u32x16 __attribute__((ext_vector_type(16)));
template <bool BF6>
__device__ __forceinline__ u32x16 cvt_pk32_bf16_fp6(u32x6 a, float s) {
  u32x16 d;
  if constexpr (BF6) asm("v_cvt_scalef32_pk32_bf16_bf6 %0, %1, %2" : "=&v"(d) : "v"(a), "v"(s));
  else asm("v_cvt_scalef32_pk32_bf16_fp6 %0, %1, %2" : "=&v"(d) : "v"(a), "v"(s));
  return d;
}
// 32 bf16 values (16 dwords) divided by the E8M0 scale -> 32 FP6 codes (6 dwords): round to nearest even, saturating.
template <bool BF6>
__device__ __forceinline__ u32x6 cvt_pk32_fp6_bf16(u32x16 a, float s) {
  u32x6 d;
  if constexpr (BF6) asm("v_cvt_scalef32_pk32_bf6_bf16 %0, %1, %2" : "=&v"(d) : "v"(a), "v"(s));
  else asm("v_cvt_scalef32_pk32_fp6_bf16 %0, %1, %2" : "=&v"(d) : "v"(a), "v"(s));
  return d;
}
// ------------------------------------------------------------------ software element codecs
// clip_b(Round(V / X)) for integer elements, X = 2^-sh.  Half away from zero: with q2 = trunc(2r)
// (the conversion truncates toward zero; 2r is exact), Round(r) = (q2 + [q2 >= 0]) >> 1 with an
// arithmetic shift, for both signs.  Half to even: the hardware's round-to-nearest-even.
template <int BITS>
__device__ __forceinline__ uint32_t encode_int_scaled(float v, int sh, int tie) {
  constexpr int LIM = (1 << (BITS - 1)) - 1;
  int q;
  if (tie == MX_ROUND_HALF_EVEN) {
    q = (int)rintf(ldexpf(v, sh));
  } else {
    int q2 = (int)ldexpf(v, sh + 1);
    q = (q2 + 1 + (q2 >> 31)) >> 1;
  }
  q = q < -LIM ? -LIM : (q > LIM ? LIM : q);
  return (uint32_t)q & ((1u << BITS) - 1u);
}

// The same for sources with at most 8 significant bits (bf16), half away from zero only: V * 2^sh + copysign(1/2, V)
// is then exact in fp32 unless |V * 2^sh| < 2^-16 (where the sum still truncates to 0), so one fma and the
// truncating conversion give Round.  (An fp32 source can sit half an ulp below a tie and would round up twice.)
// `scale` = 2^sh, subnormal for sh = -127.  Returns the clipped integer, not yet masked.
template <int BITS>
__device__ __forceinline__ int round_int_narrow(float v, float scale) {
  constexpr int LIM = (1 << (BITS - 1)) - 1;
  float half = __uint_as_float((__float_as_uint(v) & 0x80000000u) | 0x3F000000u);
  int q = (int)fmaf(v, scale, half);
  return q < -LIM ? -LIM : (q > LIM ? LIM : q);
}

template <int BITS>
__device__ __forceinline__ uint32_t encode_int(float r, int tie) {
  return encode_int_scaled<BITS>(r, 0, tie);
}

template <int BITS>
__device__ __forceinline__ float decode_int(uint32_t c) {
  return (float)(((int)(c << (32 - BITS))) >> (32 - BITS));
}

// quantize_{eta,mu}(r) on the bits of r: round the fp32 significand to mu bits (ties by `tie`),
// re-bias, saturate; below the smallest normal round on the fixed subnormal grid.
template <int ETA, int MU>
__device__ __forceinline__ uint32_t encode_fp_sw(float r, int tie) {
  constexpr int BIAS = (1 << (ETA - 1)) - 1;
  constexpr bool HAS_NAN = (ETA == 4 && MU == 3);
  constexpr uint32_t MAXC = (1u << (ETA + MU)) - (HAS_NAN ? 2u : 1u);
  constexpr uint32_t E32MIN = (uint32_t)(1 - BIAS + 127);
  uint32_t u = __float_as_uint(r);
  uint32_t sign = u >> 31;
  u &= 0x7FFFFFFFu;
  bool away = (tie == MX_ROUND_HALF_AWAY);
  uint32_t mag;
  if ((u >> 23) >= E32MIN) {
    constexpr int SH = 23 - MU;
    uint32_t keep = u >> SH, rem = u & ((1u << SH) - 1u), half = 1u << (SH - 1);
    uint32_t up = (rem > half) || (rem == half && (away || (keep & 1u)));
    mag = keep + up - ((uint32_t)(127 - BIAS) << MU);
    mag = mag > MAXC ? MAXC : mag;
  } else {
    float s = ldexpf(__uint_as_float(u), MU - (1 - BIAS));  // |r| on the subnormal grid, < 2^mu
    float t = truncf(s);
    float f = s - t;
    uint32_t ti = (uint32_t)t;
    uint32_t up = (f > 0.5f) || (f == 0.5f && (away || (ti & 1u)));
    mag = ti + up;
  }
  return (sign << (ETA + MU)) | mag;
}

template <int ETA, int MU>
__device__ __forceinline__ float decode_fp_sw(uint32_t c) {
  constexpr int BIAS = (1 << (ETA - 1)) - 1;
  constexpr bool HAS_NAN = (ETA == 4 && MU == 3);
  uint32_t m = c & ((1u << MU) - 1u);
  uint32_t e = (c >> MU) & ((1u << ETA) - 1u);
  uint32_t s = (c >> (ETA + MU)) & 1u;
  float v;
  if (HAS_NAN && e == (1u << ETA) - 1u && m == (1u << MU) - 1u) return __uint_as_float(0x7FC00000u);
  if (e)
    v = __uint_as_float(((e + 127u - BIAS) << 23) | (m << (23 - MU)));
  else
    v = (float)m * __uint_as_float((uint32_t)(127 + 1 - BIAS - MU) << 23);
  return s ? -v : v;
}

template <int ELEM>
__device__ __forceinline__ uint32_t encode_sw(float r, int tie) {
  if constexpr (Elem<ELEM>::is_int)
    return encode_int<Elem<ELEM>::bits>(r, tie);
  else
    return encode_fp_sw<Elem<ELEM>::eta, Elem<ELEM>::mu>(r, tie);
}

template <int ELEM>
__device__ __forceinline__ float decode_sw(uint32_t c) {
  if constexpr (Elem<ELEM>::is_int)
    return decode_int<Elem<ELEM>::bits>(c);
  else
    return decode_fp_sw<Elem<ELEM>::eta, Elem<ELEM>::mu>(c);
}

// ------------------------------------------------------------------ chunk codecs
// A "chunk" is N consecutive elements of one block held by one lane (N = 4 or 8), already as
// fp32.  encode_chunk returns their codes as a little-endian bit string of N * bits bits
// (element 0 in the low bits).  HW selects the scaled conversion instructions (ties to even).
// NARROW: the values have at most 8 significant bits (they came from bf16).
template <int ELEM, bool HW, int N, bool NARROW = false>
__device__ __forceinline__ uint64_t encode_chunk(const float (&v)[N], uint32_t byte, int tie) {
  using E = Elem<ELEM>;
  static_assert(N == 4 || N == 8, "chunk of 4 or 8 elements");
  if constexpr (HW && E::hw == HW_FP8) {
    float s = scale_operand(byte);
    uint32_t w[N / 4];
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
      i16x2 o = {0, 0};
      o = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(o, v[4 * i], v[4 * i + 1], s, false);
      o = __builtin_amdgcn_cvt_scalef32_pk_fp8_f32(o, v[4 * i + 2], v[4 * i + 3], s, true);
      w[i] = __builtin_bit_cast(uint32_t, o);
    }
    if constexpr (N == 4) return w[0];
    else return (uint64_t)w[0] | ((uint64_t)w[1] << 32);
  } else if constexpr (HW && E::hw == HW_FP4) {
    float s = scale_operand(byte);
    uint32_t w = 0;
    static_for<0, N / 2>([&](auto i) {
      constexpr int I = decltype(i)::value;
      w = __builtin_amdgcn_cvt_scalef32_pk_fp4_f32(w, v[2 * I], v[2 * I + 1], s, I);
    });
    return w;
  } else if constexpr (HW && (E::hw == HW_FP6 || E::hw == HW_BF6)) {
    // 2xpk16 interleaves its operands: result element 2j is src0[j], element 2j+1 is src1[j].
    // Only the first N/2 entries of each operand carry data; the rest is zero.
    float s = scale_operand(byte);
    f32x16 ev = {}, od = {};
#pragma unroll
    for (int i = 0; i < N / 2; ++i) {
      ev[i] = v[2 * i];
      od[i] = v[2 * i + 1];
    }
    u32x6 p = cvt_2xpk16_fp6_f32<E::hw == HW_BF6>(ev, od, s);
    if constexpr (N == 4) return p[0] & 0xFFFFFFu;
    else return (uint64_t)p[0] | ((uint64_t)(p[1] & 0xFFFFu) << 32);
  } else {
    uint32_t lo = 0, hi = 0;
    int sh = 127 - (int)byte;
    if constexpr (E::is_int && NARROW) {
      if (tie != MX_ROUND_HALF_EVEN) {
        const float scale = ldexpf(1.0f, sh);
        int q[N];
#pragma unroll
        for (int i = 0; i < N; ++i) q[i] = round_int_narrow<E::bits>(v[i], scale);
        if constexpr (E::bits == 8) {
          // 4 low bytes -> one dword with byte permutes (no masks)
#pragma unroll
          for (int d = 0; d < N / 4; ++d) {
            uint32_t p01 = __builtin_amdgcn_perm((uint32_t)q[4 * d + 1], (uint32_t)q[4 * d], 0x0c0c0400u);
            uint32_t p23 = __builtin_amdgcn_perm((uint32_t)q[4 * d + 3], (uint32_t)q[4 * d + 2], 0x0c0c0400u);
            uint32_t w = __builtin_amdgcn_perm(p23, p01, 0x05040100u);
            if (d == 0) lo = w; else hi = w;
          }
        } else {
#pragma unroll
          for (int i = 0; i < N; ++i) {
            uint32_t c = (uint32_t)q[i] & ((1u << E::bits) - 1u);
            const int pos = i * E::bits;
            if (pos < 32) {
              lo |= c << pos;
              if (pos + E::bits > 32) hi |= c >> (32 - pos);
            } else {
              hi |= c << (pos - 32);
            }
          }
        }
        return (uint64_t)lo | ((uint64_t)hi << 32);
      }
    }
#pragma unroll
    for (int i = 0; i < N; ++i) {
      uint32_t c;
      if constexpr (E::is_int) {
        c = encode_int_scaled<E::bits>(v[i], sh, tie);
      } else {
        // V / X, exact (a result below fp32's normal range rounds to a value that still encodes as zero)
        c = encode_fp_sw<E::eta, E::mu>(ldexpf(v[i], sh), tie);
      }
      const int pos = i * E::bits;   // compile-time after unrolling
      if (pos < 32) {
        lo |= c << pos;
        if (pos + E::bits > 32) hi |= c >> (32 - pos);
      } else {
        hi |= c << (pos - 32);
      }
    }
    return (uint64_t)lo | ((uint64_t)hi << 32);
  }
}

// Inverse: N codes (bit string) times 2^(byte-127) as fp32.  byte == 255 is handled by callers.
template <int ELEM, bool HW, int N>
__device__ __forceinline__ void decode_chunk(uint64_t codes, uint32_t byte, float (&v)[N]) {
  using E = Elem<ELEM>;
  static_assert(N == 4 || N == 8, "chunk of 4 or 8 elements");
  if constexpr (HW && E::hw == HW_FP8) {
    float s = scale_operand(byte);
#pragma unroll
    for (int i = 0; i < N / 4; ++i) {
      uint32_t w = (uint32_t)(codes >> (32 * i));
      f32x2 a = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(w, s, false);
      f32x2 b = __builtin_amdgcn_cvt_scalef32_pk_f32_fp8(w, s, true);
      v[4 * i] = a.x; v[4 * i + 1] = a.y; v[4 * i + 2] = b.x; v[4 * i + 3] = b.y;
    }
  } else if constexpr (HW && E::hw == HW_FP4) {
    float s = scale_operand(byte);
    uint32_t w = (uint32_t)codes;
    static_for<0, N / 2>([&](auto i) {
      constexpr int I = decltype(i)::value;
      f32x2 a = __builtin_amdgcn_cvt_scalef32_pk_f32_fp4(w, s, I);
      v[2 * I] = a.x; v[2 * I + 1] = a.y;
    });
  } else if constexpr (HW && (E::hw == HW_FP6 || E::hw == HW_BF6)) {
    // A minifloat without Inf / NaN placed in the top of an fp32's exponent / mantissa fields reads as
    // its own value times 2^(bias - 127), subnormals included (both formats share the convention);
    // one ldexp undoes that and applies the block scale.  Exact: at most mu + 1 significant bits.
    int sh = (int)byte - 127 + (127 - E::bias);
#pragma unroll
    for (int i = 0; i < N; ++i) {
      uint32_t c = (uint32_t)(codes >> (i * 6));
      uint32_t f = ((c & 0x1Fu) << (23 - E::mu)) | ((c & 0x20u) << 26);
      v[i] = ldexpf(__uint_as_float(f), sh);
    }
  } else {
    int sh = (int)byte - 127;
#pragma unroll
    for (int i = 0; i < N; ++i) {
      uint32_t c = (uint32_t)(codes >> (i * E::bits)) & ((1u << E::bits) - 1u);
      v[i] = ldexpf(decode_sw<ELEM>(c), sh);
    }
  }
}

// ------------------------------------------------------------------ Slice-and-Scale element maps
// All work on 4 anchor codes held in the 4 bytes of one dword.

// E4M3 NaN codes (S.1111.111) inside an anchor are taken as +-448: turn 0x7F / 0xFF into 0x7E / 0xFE.
__device__ __forceinline__ uint32_t e4m3_nan_to_max(uint32_t x) {
  uint32_t t = x & 0x7F7F7F7Fu;
  uint32_t n = (t + 0x01010101u) & 0x80808080u;  // bit 7 of a byte set iff its low 7 bits are all ones
  return x - (n >> 7);
}

// Eq. (4): P_l = clip(Round(P_h / 2^De)) on 4 int8 codes at once; result: 4 two's-complement
// BL-bit codes, one per byte lane.  Rounding acts on the magnitude (half away from zero by
// default), which is the "round on the most significant dropped bit" of Sec. 3.3.
template <int BL>
__device__ __forceinline__ uint32_t slice_int8x4(uint32_t x, int tie) {
  constexpr int DE = 8 - BL;
  constexpr uint32_t ONES = 0x01010101u;
  constexpr uint32_t LOW = ((1u << BL) - 1u) * ONES;
  uint32_t sg = x & 0x80808080u;
  uint32_t s = sg >> 7;
  uint32_t mask = (sg - s) | sg;      // 0xFF in negative byte lanes
  uint32_t mag = (x ^ mask) + s;      // |P_h| per lane, 0..128, no carry between lanes
  uint32_t q;
  if constexpr (DE == 0) {
    q = mag;
  } else {
    constexpr uint32_t HALF = (1u << (DE - 1)) * ONES;
    constexpr uint32_t KEEP = (0xFFu >> DE) * ONES;
    if (tie == MX_ROUND_HALF_EVEN) {
      uint32_t odd = (mag >> DE) & ONES;
      q = ((mag + (HALF - ONES) + odd) >> DE) & KEEP;
    } else {
      q = ((mag + HALF) >> DE) & KEEP;
    }
  }
  q -= (q >> (BL - 1)) & ONES;        // clip: q is at most 2^(BL-1), one above the limit
  return (((q ^ mask) & LOW) + s) & LOW;
}

// Eq. (6) for one E4M3 code with a software target (non-OCP minifloat or non-default tie).
template <int TARGET>
__device__ __forceinline__ uint32_t slice_e4m3_sw(uint32_t code, int tie) {
  constexpr int DE = Elem<MX_FP8_E4M3>::emax - Elem<TARGET>::emax;
  float p = __builtin_amdgcn_cvt_f32_fp8(code, 0);
  return encode_fp_sw<Elem<TARGET>::eta, Elem<TARGET>::mu>(ldexpf(p, -DE), tie);
}

// ------------------------------------------------------------------ bit packing
// 4 * NIN codes, one per byte in in[0..NIN-1], to NIN * BITS / 8 dwords (little-endian bit string).
// NIN = 8 is a whole block, NIN = 4 half a block (even widths only).
template <int BITS, int NIN>
__device__ __forceinline__ void pack_bytes(const uint32_t (&in)[NIN], uint32_t (&out)[NIN * BITS / 8]) {
  static_assert((NIN * BITS) % 8 == 0, "piece must end on a dword boundary");
  if constexpr (BITS == 8) {
#pragma unroll
    for (int i = 0; i < NIN; ++i) out[i] = in[i];
  } else if constexpr (BITS == 4) {
#pragma unroll
    for (int i = 0; i < NIN / 2; ++i) {
      uint32_t a = in[2 * i] | (in[2 * i] >> 4);          // bytes 0 and 2 hold two nibbles each
      uint32_t b = in[2 * i + 1] | (in[2 * i + 1] >> 4);
      out[i] = __builtin_amdgcn_perm(b, a, 0x06040200u);  // {a.b0, a.b2, b.b0, b.b2}
    }
  } else if constexpr (BITS == 6) {
#pragma unroll
    for (int i = 0; i < NIN / 4; ++i) {
      uint32_t p[4];
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        uint32_t x = in[4 * i + j];
        p[j] = (x & 0x3Fu) | ((x >> 2) & 0xFC0u) | ((x >> 4) & 0x3F000u) | ((x >> 6) & 0xFC0000u);
      }
      out[3 * i] = p[0] | (p[1] << 24);
      out[3 * i + 1] = (p[1] >> 8) | (p[2] << 16);
      out[3 * i + 2] = (p[2] >> 16) | (p[3] << 8);
    }
  } else {
#pragma unroll
    for (int i = 0; i < NIN * BITS / 8; ++i) out[i] = 0;
#pragma unroll
    for (int i = 0; i < 4 * NIN; ++i) {
      uint32_t c = (in[i >> 2] >> (8 * (i & 3))) & ((1u << BITS) - 1u);
      const int pos = i * BITS, d = pos >> 5, sft = pos & 31;
      out[d] |= c << sft;
      if (sft + BITS > 32) out[d + 1] |= c >> (32 - sft);
    }
  }
}

template <int BITS>
__device__ __forceinline__ void pack_block_bytes(const uint32_t (&in)[8], uint32_t (&out)[BITS]) {
  pack_bytes<BITS, 8>(in, out);
}

// Store / load W consecutive dwords at a 4*W-byte stride per lane with the widest aligned accesses.
template <int W>
__device__ __forceinline__ void store_dwords(uint32_t* p, const uint32_t (&v)[W]) {
  if constexpr (W % 4 == 0) {
#pragma unroll
    for (int i = 0; i < W / 4; ++i) reinterpret_cast<u32x4*>(p)[i] = u32x4{v[4 * i], v[4 * i + 1], v[4 * i + 2], v[4 * i + 3]};
  } else if constexpr (W % 2 == 0) {
#pragma unroll
    for (int i = 0; i < W / 2; ++i) reinterpret_cast<u32x2*>(p)[i] = u32x2{v[2 * i], v[2 * i + 1]};
  } else if constexpr (W == 3) {
    // one 96-bit store (needs only dword alignment)
    typedef uint32_t u32x3 __attribute__((ext_vector_type(3)));
    typedef u32x3 __attribute__((aligned(4))) u32x3_a4;
    *reinterpret_cast<u32x3_a4*>(p) = u32x3{v[0], v[1], v[2]};
  } else {
#pragma unroll
    for (int i = 0; i < W; ++i) p[i] = v[i];
  }
}

template <int W>
__device__ __forceinline__ void load_dwords(const uint32_t* p, uint32_t (&v)[W]) {
  if constexpr (W % 4 == 0) {
#pragma unroll
    for (int i = 0; i < W / 4; ++i) {
      u32x4 t = reinterpret_cast<const u32x4*>(p)[i];
      v[4 * i] = t.x; v[4 * i + 1] = t.y; v[4 * i + 2] = t.z; v[4 * i + 3] = t.w;
    }
  } else if constexpr (W % 2 == 0) {
#pragma unroll
    for (int i = 0; i < W / 2; ++i) {
      u32x2 t = reinterpret_cast<const u32x2*>(p)[i];
      v[2 * i] = t.x; v[2 * i + 1] = t.y;
    }
  } else {
#pragma unroll
    for (int i = 0; i < W; ++i) v[i] = p[i];
  }
}

// Saturating add of De to 4 or more E8M0 bytes held in one dword: min(b + De, 254), 255 stays
// 255 (Eq. (4) / Eq. (6) scale step with the E8M0 range respected).
__device__ __forceinline__ uint32_t scale_add_x4(uint32_t x, uint32_t de) {
  constexpr uint32_t ONES = 0x01010101u, H = 0x80808080u, L = 0x7F7F7F7Fu;
  uint32_t lo = (x & L) + de * ONES;          // de < 128: no carry between lanes
  uint32_t sum = lo ^ (x & H);                // per-lane (b + de) mod 256
  uint32_t ovf = (x & lo & H) >> 7;           // lane overflowed past 255
  uint32_t was255 = (((x & L) + ONES) & x & H) >> 7;
  uint32_t is255 = (((sum & L) + ONES) & sum & H) >> 7;
  uint32_t sat = (ovf | is255) & ~was255;     // lanes that must read 254
  uint32_t full = (sat | was255);
  uint32_t m = (full << 8) - full;            // 0xFF in lanes to overwrite (lanes are 0 or 1: no borrow trouble)
  return (sum & ~m) | (m - sat);              // 0xFF - 1 = 0xFE where saturated, 0xFF where it was 255
}

}  // namespace mx
