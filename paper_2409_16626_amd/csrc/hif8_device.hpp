// Device-side HiF8 arithmetic for gfx950: bit-level rounding of binary32 patterns to the
// HiF8 grid, assembly of the sign | dot | exponent | mantissa byte, and expansion of a
// byte back to a binary32 pattern.  (arXiv 2409.16626: Sec. 2.1 Tables 1-3, Eq. (1), Eq. (2);
// Sec. 3.1 rounding half away from zero; Sec. 3.2 simplified stochastic rounding and Eq. (3).)
//
// Everything works on integer views of IEEE binary32 values:
//   a      magnitude pattern (sign stripped), never a NaN here
//   e      biased exponent a >> 23, E = e - 127
//   k(E)   mantissa bits HiF8 keeps in the binade of E: 3 for |E| <= 3, 2 for 4..7,
//          1 for 8..15, 0 below 2^-15 (denormal codes are pure powers of two)
// Adding the rounding carry to the kept part of the pattern propagates into the exponent
// by itself, and the value it reaches (2^(E+1)) is representable at every band edge, so
// rounding "at the width of the source binade" is rounding to the nearest HiF8 value.
#pragma once

#ifndef HIF8_DEVICE_HOST_SHIM  // a CPU test build supplies __device__, __forceinline__ and __clz itself
#include <hip/hip_runtime.h>
#endif
#include <stdint.h>

namespace hif8dev {

constexpr uint32_t kCodeInf = 0x6Fu;  // S 11 0111 1 : the 1.5 * 2^15 slot, read as Infinity
constexpr uint32_t kCodeMax = 0x6Eu;  // 0 11 0111 0 : 2^15, largest finite magnitude
constexpr uint32_t kCodeNaN = 0x80u;  // 1 0000 000
constexpr uint32_t kBitsOverflow = 0x47400000u;  // binary32 pattern of 1.5 * 2^15
constexpr uint32_t kBitsTwoM22 = 105u << 23;     // binary32 pattern of 2^-22 (smallest denormal code)

// rounding_mode bit-field as seen by kernels
constexpr uint32_t kRmTA = 0u;   // rounding half away from zero (Sec. 3.1)
constexpr uint32_t kRmHR = 1u;   // hybrid rounding (Eq. (3))
constexpr uint32_t kRmTE = 2u;   // rounding half to even (Sec. 3.1; comparison mode)
constexpr uint32_t kRmSSR = 3u;  // simplified SR in every binade (Sec. 3.2; comparison mode)
constexpr uint32_t kRmSR = 4u;   // standard SR with a counter-based threshold (Sec. 3.2; comparison mode)
constexpr uint32_t kFlagSat = 0x10u;
constexpr uint32_t kFlagNan2Zero = 0x20u;

// source kinds: which simplified SR applies and where the source format's LSB sits in the
// binary32 pattern being converted (Sec. 3.2: SR14 for FP32, SR2 for FP16 and BF16)
constexpr int kSrcF32 = 0;
constexpr int kSrcBF16 = 1;  // LSB = bit 16
constexpr int kSrcF16 = 2;   // LSB = bit 13

__device__ __forceinline__ uint32_t overflow_code(uint32_t mode) {
  return (mode & kFlagSat) ? kCodeMax : kCodeInf;
}
__device__ __forceinline__ uint32_t nan_code(uint32_t mode) {
  return (mode & kFlagNan2Zero) ? 0u : kCodeNaN;
}

// Mantissa bits kept for biased binary32 exponent e (Table 3 widths per |E|; Eq. (2): none).
// |E| = 0..3 -> 3, 4..7 -> 2, 8..15 -> 1, >= 16 -> 0, i.e. clamp(clz(|E|) - 27, 0, 3).
__device__ __forceinline__ uint32_t kept_bits(uint32_t e) {
  int d = (int)e - 127;
  uint32_t absE = (uint32_t)(d < 0 ? -d : d);
  int k = __clz((int)absE) - 27;  // __clz(0) == 32
  k = k < 0 ? 0 : k;
  k = k > 3 ? 3 : k;
  return (uint32_t)k;
}

// Rounds magnitude pattern `a` (finite or Inf, not NaN) to the HiF8 grid and returns the
// rounded binary32 pattern.  `ybits` is the full pattern being converted (threshold bits
// of the simplified SR come from it).
//   - Below 2^-22 the grid has a single step [0, 2^-22]; the value is first rewritten as a
//     pseudo pattern in the binade of biased exponent 103 whose 23 mantissa bits hold
//     floor(a / 2^-22 * 2^23), so that the same "discarded fraction" logic applies.  A carry
//     then lands on pattern 104 << 23, which pack_mag() reads as 2^-22; no carry leaves
//     exponent 103, which pack_mag() reads as zero.
//   - TA (Sec. 3.1): carry iff the top discarded bit is set  ==  F >= half.
//   - HR (Eq. (3)): TA where k == 3 (|E| < 4); elsewhere simplified SR: carry iff F >= T,
//     F = top 14 (FP32 source) or top 2 (16-bit source) discarded bits, T = low 14 bits of
//     the pattern, or {bit 16, 1}.  F = 0 never carries (T is raised to at least 1), which
//     keeps representable inputs fixed.
template <bool HR, int SRCK>
__device__ __forceinline__ uint32_t round_mag(uint32_t a, uint32_t ybits) {
  uint32_t ap = a;
  {
    uint32_t sig = (a & 0x7FFFFFu) | 0x800000u;
    uint32_t shift = 105u - (a >> 23);  // >= 1 whenever it is used
    uint32_t P = (shift > 24u) ? 0u : (sig >> (shift & 31u));
    ap = (a < kBitsTwoM22) ? ((103u << 23) | P) : a;
  }
  const uint32_t k = kept_bits(ap >> 23);
  const uint32_t sh = 23u - k;
  uint32_t F, T;
  if (SRCK != kSrcF32) {
    F = (ap >> (sh - 2u)) & 3u;
    T = 2u * ((ybits >> (SRCK == kSrcBF16 ? 16 : 13)) & 1u) + 1u;
    if (!HR || k == 3u) T = 2u;
  } else {
    F = (ap >> (sh - 14u)) & 0x3FFFu;
    T = ybits & 0x3FFFu;
    T = T < 1u ? 1u : T;
    if (!HR || k == 3u) T = 0x2000u;
  }
  const uint32_t t = (ap >> sh) + (F >= T ? 1u : 0u);
  return t << sh;
}

// Magnitude code (7 bits) of a rounded pattern r produced by round_mag(), i.e. a pattern
// whose value is on the HiF8 grid (or beyond it).  Field assembly per Tables 1-3:
//   dot 0001 (D=0): 0001 mmm            E = 0
//   dot 001  (D=1): 001 Se mmm          |E| = 1
//   dot 01   (D=2): 01 Se g mmm         |E| = 2 | g
//   dot 10   (D=3): 10 Se gg mm         |E| = 4 | gg
//   dot 11   (D=4): 11 Se ggg m         |E| = 8 | ggg
//   dot 0000 (DML): 0000 MMM            value 2^(MMM - 23)
// For D >= 2 the bits below the dot are {Se, low D-1 bits of |E|, 5-D mantissa bits} and
// (|E| << (5-D)) always has its leading one at bit 4, so masking with 0xF drops it.
__device__ __forceinline__ uint32_t pack_mag(uint32_t r, uint32_t ovf_code) {
  if (r >= kBitsOverflow) return ovf_code;
  const uint32_t e = r >> 23;
  if (e <= 103u) return 0u;
  if (e <= 111u) return e == 104u ? 1u : e - 104u;  // 2^-22 .. 2^-16 (104: carry out of the underflow step)
  const int E = (int)e - 127;
  const uint32_t absE = (uint32_t)(E < 0 ? -E : E);
  const uint32_t Se = E < 0 ? 1u : 0u;
  const uint32_t m3 = (r >> 20) & 7u;
  const uint32_t D = 32u - (uint32_t)__clz((int)absE);
  if (D == 0u) return 0x08u | m3;
  if (D == 1u) return 0x10u | (Se << 3) | m3;
  const uint32_t kW = 5u - D;
  return ((D - 1u) << 5) | (Se << 4) | ((absE << kW) & 0xFu) | (m3 >> (3u - kW));
}

// Full ALU encode of one binary32 pattern (already scaled).
template <bool HR, int SRCK>
__device__ __forceinline__ uint32_t encode_alu(uint32_t ybits, uint32_t mode) {
  const uint32_t a = ybits & 0x7FFFFFFFu;
  if (a > 0x7F800000u) return nan_code(mode);
  const uint32_t c = pack_mag(round_mag<HR, SRCK>(a, ybits), overflow_code(mode));
  return c ? (c | ((ybits >> 24) & 0x80u)) : 0u;
}

// ------------------------------------------------------------------------------------
// Comparison modes (Sec. 3.1 TE; Sec. 3.2 simplified SR everywhere, standard SR), written
// for clarity: these are not on the throughput path.
// ------------------------------------------------------------------------------------

// Threshold generator of standard SR (Sec. 3.2 asks for one uniform random number per element and names no
// source; a counter-based hash supplies it: no state, reproducible, independent of the launch shape).
// Threshold of element `index` under `seed`:
//   key pair   (k1, k2) = low and high half of splitmix64's output function applied to
//              seed + 0x9E3779B97F4A7C15 * (hi32(index) + 1): a non-linear function of the whole seed,
//              constant over 2^32 consecutive elements (the kernels compute it once per workgroup and again
//              only where a tensor crosses a multiple of 2^32 elements);
//   threshold  MurmurHash3's 32-bit finaliser over lo32(index) ^ k1, with k2 added between its two
//              multiplications: ten vector instructions per element.
// Two seeds give two different functions of the index, not one sequence in another order.
struct SrKey {
  uint32_t k1, k2;
};
__host__ __device__ __forceinline__ SrKey sr_key(uint64_t seed, uint32_t index_hi) {
  uint64_t z = seed + 0x9E3779B97F4A7C15ull * ((uint64_t)index_hi + 1ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z = z ^ (z >> 31);
  SrKey k;
  k.k1 = (uint32_t)z;
  k.k2 = (uint32_t)(z >> 32);
  return k;
}
__host__ __device__ __forceinline__ uint32_t sr_hash(uint32_t index_lo, const SrKey& k) {
  uint32_t x = index_lo ^ k.k1;
  x ^= x >> 16; x *= 0x85EBCA6Bu; x += k.k2;
  x ^= x >> 13; x *= 0xC2B2AE35u; x ^= x >> 16;
  return x;
}
__host__ __device__ __forceinline__ uint32_t sr_threshold(uint64_t seed, uint64_t index) {
  return sr_hash((uint32_t)index, sr_key(seed, (uint32_t)(index >> 32)));
}

// Rounded pattern of magnitude `a` (not NaN) under rounding method rm (any of the five), in
// the convention of round_mag(): exponent 103 reads as zero and 104 as 2^-22 in pack_mag().
//   TE : carry iff the discarded part is above half, or exactly half and the kept
//        significand is odd (with no kept mantissa bits the significand is 1: odd).
//        Below 2^-22 the lower neighbour is 0 (even), so only strictly more than half carries.
//   SR : carry iff t32 / 2^32 < discarded fraction.  With d discarded bits that is
//        (t32 >> (32 - d)) < discarded, exactly.  Below 2^-22 the fraction is sig / 2^s,
//        s = 128 - e >= 24.
//   TA / HR / SSR: the F >= T rule of round_mag(), SSR without the |E| < 4 exception.
template <int SRCK>
__device__ __forceinline__ uint32_t round_mag_any(uint32_t rm, uint32_t a, uint32_t ybits, uint32_t t32) {
  if (rm == kRmTA) return round_mag<false, SRCK>(a, ybits);
  if (rm == kRmHR) return round_mag<true, SRCK>(a, ybits);
  const uint32_t e = a >> 23;
  if (a < kBitsTwoM22) {
    // value = sig * 2^(e - 150) (subnormal binary32: sig = mantissa, e taken as 1)
    const uint32_t sig = e ? ((a & 0x7FFFFFu) | 0x800000u) : a;
    const uint32_t s = 128u - (e ? e : 1u);  // fraction of the 2^-22 step = sig / 2^s, s in [24, 127]
    bool carry;
    if (rm == kRmTE) {
      carry = (s == 24u) && (sig > 0x800000u);  // more than half of the step
    } else if (rm == kRmSR) {
      if (s < 32u) carry = t32 < (sig << (32u - s));
      else if (s < 56u) carry = t32 < ((sig + (1u << (s - 32u)) - 1u) >> (s - 32u));  // ceil(sig / 2^(s-32))
      else carry = (t32 == 0u) && (sig != 0u);
    } else {  // SSR: top 14 (or 2) bits of the fraction against the threshold bits
      uint32_t F, T;
      if (SRCK != kSrcF32) {
        F = (s - 2u < 32u) ? (sig >> (s - 2u)) : 0u;
        T = 2u * ((ybits >> (SRCK == kSrcBF16 ? 16 : 13)) & 1u) + 1u;
      } else {
        F = (s - 14u < 32u) ? (sig >> (s - 14u)) : 0u;
        T = ybits & 0x3FFFu;
        T = T < 1u ? 1u : T;
      }
      carry = F >= T;
    }
    return (carry ? 104u : 103u) << 23;
  }
  const uint32_t k = kept_bits(e);
  const uint32_t d = 23u - k;
  const uint32_t disc = a & ((1u << d) - 1u);
  bool carry;
  if (rm == kRmTE) {
    const uint32_t half = 1u << (d - 1u);
    const uint32_t n_odd = k ? ((a >> d) & 1u) : 1u;
    carry = disc > half || (disc == half && n_odd);
  } else if (rm == kRmSR) {
    carry = (t32 >> (32u - d)) < disc;
  } else {
    uint32_t F, T;
    if (SRCK != kSrcF32) {
      F = disc >> (d - 2u);
      T = 2u * ((ybits >> (SRCK == kSrcBF16 ? 16 : 13)) & 1u) + 1u;
    } else {
      F = disc >> (d - 14u);
      T = ybits & 0x3FFFu;
      T = T < 1u ? 1u : T;
    }
    carry = F >= T;
  }
  return ((a >> d) + (carry ? 1u : 0u)) << d;
}

// Standard SR, table-driven form for the streaming kernels.
//
// At or above 2^-22, with d discarded bits, the carry rule (t32 >> (32 - d)) < discarded is the carry out
// of discarded + ((2^d - 1) - (t32 >> (32 - d))): add the top d bits of the complemented threshold below
// the kept part and truncate,
//     r = (y + bfe(~t32, 32 - d, d)) & mask,      mask = ~(2^d - 1),
// on the whole pattern y (the sum stays below the sign bit: the magnitude is at most Inf's pattern, the
// addend below 2^23).  The result is on the HiF8 grid, where the TA table is the identity.  Exponent 255
// (Inf, and NaN, which the table turns into the code of the NaN option) takes a field of width 0: unchanged.
// Below 2^-22 the rule is t32 < |y| / 2^-22 * 2^32 = |y| * 2^54, a product that binary32 holds exactly
// (below 2^32; subnormal inputs included, denormals are not flushed), so with X = ceil of it as an integer
// the value carries to 2^-22 (written as exponent 104, which the TA table reads as 2^-22) iff t32 < X, and
// is zero otherwise (mask keeps the sign only).  The factor is 2^54 for those exponents and 0 for all others
// (X = 0: never; Inf * 0 = NaN converts to 0 as well).
struct SrExp {
  uint32_t off, width;  // field of ~t32 that is added
  uint32_t mask;
  float fmul;
};

__device__ __forceinline__ SrExp sr_exp_entry(uint32_t e) {
  SrExp h;
  h.off = 0u; h.width = 0u; h.mask = 0xFFFFFFFFu; h.fmul = 0.0f;
  if (e == 255u) return h;
  if (e <= 104u) {
    h.mask = 0x80000000u;
    union { uint32_t u; float f; } v;
    v.u = (127u + 54u) << 23;
    h.fmul = v.f;
    return h;
  }
  const uint32_t d = 23u - kept_bits(e);  // 20..23
  h.off = 32u - d; h.width = d; h.mask = 0xFFFFFFFFu << d;
  return h;
}

#ifdef HIF8_DEVICE_HOST_SHIM
__device__ __forceinline__ uint32_t bfe_u32(uint32_t x, uint32_t off, uint32_t width) {
  return width ? ((x >> off) & ((1u << width) - 1u)) : 0u;
}
__device__ __forceinline__ uint32_t ceil_to_u32(float p) {  // p >= 0 or NaN; NaN -> 0
  if (!(p == p)) return 0u;
  const double c = __builtin_ceil((double)p);
  return c >= 4294967295.0 ? 0xFFFFFFFFu : (uint32_t)c;
}
#else
__device__ __forceinline__ uint32_t bfe_u32(uint32_t x, uint32_t off, uint32_t width) {
  return __builtin_amdgcn_ubfe(x, off, width);
}
__device__ __forceinline__ uint32_t ceil_to_u32(float p) {  // v_cvt_u32_f32: NaN -> 0, saturating
  uint32_t r;
  asm("v_cvt_u32_f32 %0, %1" : "=v"(r) : "v"(__builtin_ceilf(p)));
  return r;
}
#endif

// Rounded binary32 pattern (sign kept) of pattern ybits under standard SR with threshold t32;
// p = table entry of ybits' exponent.  NaN patterns come back unchanged.
__device__ __forceinline__ uint32_t sr_round_bits(uint32_t ybits, uint32_t t32, const SrExp& p) {
  union { uint32_t u; float f; } mag;
  mag.u = ybits & 0x7FFFFFFFu;
  const uint32_t X = ceil_to_u32(mag.f * p.fmul);
  const uint32_t small = t32 < X ? (104u << 23) : 0u;
  return ((ybits + bfe_u32(~t32, p.off, p.width)) & p.mask) | small;
}

// Full encode of one binary32 pattern under any rounding method (element-wise paths).
template <int SRCK>
__device__ __forceinline__ uint32_t encode_any(uint32_t ybits, uint32_t mode, uint32_t t32) {
  const uint32_t a = ybits & 0x7FFFFFFFu;
  if (a > 0x7F800000u) return nan_code(mode);
  const uint32_t c = pack_mag(round_mag_any<SRCK>(mode & 0xFu, a, ybits, t32), overflow_code(mode));
  return c ? (c | ((ybits >> 24) & 0x80u)) : 0u;
}

// ------------------------------------------------------------------------------------
// Hybrid rounding, table-driven form for the streaming kernels, binary32 sources (SR14).
//
// With d discarded mantissa bits, "carry iff F14 >= T" (F14 the top 14 discarded bits, Sec. 3.2) is the
// carry out of the discarded field after adding 2^d - T * 2^(d-14), so the rounding is
//     r = (a + C - T' * mult) & mask,    C = 2^d,  mult = 2^(d-14),  mask = ~(2^d - 1),
// on the binary32 pattern a of |y|; the carry propagates into the exponent exactly as in TA.  T' is the
// threshold T = low 14 bits of the pattern clamped to a per-exponent range: [1, 2^14 - 1] where Eq. (3)
// asks for simplified SR (so that F = 0 never carries), [2^13, 2^13] where it asks for TA (|E| < 4).
// Below 2^-22 there is one step from 0 to 2^-22 and F14 = sig >> (10 + j) for exponent 104 - j (sig the
// 24-bit significand): with C = (j + 1) * 2^23 and mult = 2^(10+j) the sum is 104 * 2^23 + sig - T' * mult,
// i.e. at or above exponent 104 exactly when it carries; the mask then keeps the exponent only, which
// the TA table reads as 2^-22 (104, 105) or 0 (below).  T' is clamped to 2^(14-j) there (F14 is smaller
// than that, and the product stays below 2^24).  Exponents with F14 = 0 (E <= -37), at or above 2^16,
// Inf and NaN pass unchanged (T' = 0).  The multiply is a 24-bit one (full rate).
// ------------------------------------------------------------------------------------
struct HrExp {
  uint32_t C;
  int32_t negmult;  // -mult
  uint32_t mask;
  uint32_t lo, hi;  // clamp range of the threshold
};

__device__ __forceinline__ float pow2f(int x) {  // 2^x for x in [-126, 127]
  union { uint32_t u; float f; } v;
  v.u = (uint32_t)(x + 127) << 23;
  return v.f;
}

// ssr: simplified SR in every binade (no TA exception for |E| < 4)
__device__ __forceinline__ HrExp hr_exp_entry(uint32_t e, bool ssr = false) {
  HrExp h;
  h.C = 0u; h.negmult = 0; h.mask = 0xFFFFFFFFu; h.lo = 0u; h.hi = 0u;
  if (e >= 143u || e <= 90u) return h;
  if (e <= 104u) {
    const uint32_t j = 104u - e;
    h.C = (j + 1u) << 23;
    h.negmult = -(int32_t)(1u << (10u + j));
    h.mask = 0xFF800000u;
    h.lo = 1u;
    h.hi = 1u << (14u - j);
    return h;
  }
  const uint32_t k = kept_bits(e), d = 23u - k;
  const bool ta = (k == 3u) && !ssr;
  h.C = 1u << d;
  h.negmult = -(int32_t)(1u << (d - 14u));
  h.mask = 0xFFFFFFFFu << d;
  h.lo = ta ? 0x2000u : 1u;
  h.hi = ta ? 0x2000u : 0x3FFFu;
  return h;
}

#ifdef HIF8_DEVICE_HOST_SHIM
// host stand-ins for two hardware instructions (used by the CPU test build only)
__device__ __forceinline__ uint32_t med3_u32(uint32_t a, uint32_t lo, uint32_t hi) {
  return a < lo ? lo : (a > hi ? hi : a);
}
__device__ __forceinline__ int32_t mul_i24(int32_t a, int32_t b) { return a * b; }  // operands fit 24 bits
#else
__device__ __forceinline__ uint32_t med3_u32(uint32_t a, uint32_t lo, uint32_t hi) {
  uint32_t r;
  asm("v_med3_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(lo), "v"(hi));
  return r;
}
__device__ __forceinline__ int32_t mul_i24(int32_t a, int32_t b) { return __mul24(a, b); }
#endif

// Rounded binary32 pattern (sign kept) of pattern ybits under HR; p = table entry of ybits' exponent.
// The result is on the HiF8 grid (or at/above 1.5 * 2^15: overflow); NaN patterns come back unchanged.
template <int SRCK>
__device__ __forceinline__ uint32_t hr_round_bits(uint32_t ybits, const HrExp& p) {
  static_assert(SRCK == kSrcF32, "binary32 sources; 16-bit sources use hr16_round_sum");
  // on the whole pattern: the addend C - T' * mult never takes the magnitude below zero or up to the sign
  // bit (it is at least -2^24 where the magnitude is at least 96 * 2^23, below 2^24 elsewhere, and zero
  // from exponent 143 up), and every mask keeps the sign bit
  const uint32_t T = med3_u32(ybits & 0x3FFFu, p.lo, p.hi);
  return (ybits + p.C + (uint32_t)mul_i24((int32_t)T, p.negmult)) & p.mask;
}

// ------------------------------------------------------------------------------------
// HR / simplified SR for 16-bit sources (SR2), streaming form.  The two-bit test "top two
// discarded bits F2 >= T2" with T2 = {source LSB, 1} (Sec. 3.2), or F2 >= 2 where Eq. (3) asks for
// TA, is the carry out of the discarded field after adding (4 - T2) (resp. 2) at the position of
// its top two bits, so the rounding is one add and one mask on the binary32 pattern; the carry
// propagates into the exponent exactly as in TA.  Per exponent the table holds the addend for a
// source LSB of 0, the addend for an LSB of 1, and the mask.  Below 2^-22 there is one step from 0 to
// 2^-22 (fraction bits F2 = {1, m22} for E = -23, 01 for E = -24, 00 below): the addends move the
// pattern to exponent 104 or above when it carries and leave it below otherwise, which the TA table
// then reads as 2^-22 and 0.  From 2^16 up (and for Inf) nothing is added: overflow whatever the rounding.
// ------------------------------------------------------------------------------------
struct HrExp16 {
  uint32_t add0;  // source LSB 0: T2 = 1
  uint32_t add1;  // source LSB 1: T2 = 3
  uint32_t mask;
};

__device__ __forceinline__ HrExp16 hr16_exp_entry(uint32_t e, bool ssr = false) {
  HrExp16 h;
  h.add0 = 0u; h.add1 = 0u; h.mask = 0xFFFFFFFFu;
  if (e >= 143u || e <= 102u) return h;
  if (e == 104u) { h.add0 = 1u << 22; h.add1 = 0u - (1u << 22); return h; }  // F2 = {1, m22}
  if (e == 103u) { h.add0 = 1u << 23; return h; }                           // F2 = 01: carries iff T2 = 1
  const uint32_t k = kept_bits(e), d = 23u - k;
  const bool ta = (k == 3u) && !ssr;
  h.add0 = (ta ? 2u : 3u) << (d - 2u);
  h.add1 = (ta ? 2u : 1u) << (d - 2u);
  h.mask = 0xFFFFFFFFu << d;
  return h;
}

// The source LSB that selects the addend is bit 16 (BF16) or bit 13 (FP16) of the pattern.
template <int SRCK>
__device__ __forceinline__ uint32_t hr16_lsb(uint32_t ybits) {
  static_assert(SRCK != kSrcF32, "16-bit sources only");
  return (ybits >> (SRCK == kSrcBF16 ? 16 : 13)) & 1u;
}
// Rounding a 16-bit source's scaled pattern ybits: (ybits + add) & mask with the addend of its exponent and
// source LSB and the mask of its exponent.  The add works on the whole pattern: the magnitude plus the addend
// stays within [0, 2^31) (the one negative addend, -2^22, belongs to exponent 104), the masks keep the sign
// bit, and Inf / NaN patterns get a zero addend.  The kernels use the form below, which leaves the mask to
// the lookup table.
//
// Sum without the per-exponent mask, for a lookup in the truncating table (trunc_table_pattern()),
// which clears the bits below the kept mantissa of the exponent it sees.  That is the exponent of the sum:
// the right one unless the add carried into the next binade, where the result is the start of that binade
// exactly but the sum still holds what is left of the discarded field (and the next binade may keep one
// bit more).  Clamping the sum to the start of the next binade removes it; the saturating add keeps
// negative Inf / NaN patterns (exponent 255, zero addend) from wrapping to zero.
#ifdef HIF8_DEVICE_HOST_SHIM
__device__ __forceinline__ uint32_t uadd_sat1(uint32_t x) { return x == 0xFFFFFFFFu ? x : x + 1u; }
#else
__device__ __forceinline__ uint32_t uadd_sat1(uint32_t x) { return __builtin_elementwise_add_sat(x, 1u); }
#endif
__device__ __forceinline__ uint32_t hr16_round_sum(uint32_t ybits, uint32_t add) {
  const uint32_t sum = ybits + add;
  const uint32_t next = uadd_sat1(ybits | 0x007FFFFFu);
  return sum < next ? sum : next;
}
// Pattern whose TA code entry i (= pattern >> 19) of the truncating table holds.
__device__ __forceinline__ uint32_t trunc_table_pattern(uint32_t i) {
  return (i << 19) & hr16_exp_entry((i >> 4) & 0xFFu).mask;
}

// Per-tensor scale from an amax (Sec. 5): fl32(target / amax), with pow2 the largest power of two not
// above it; amax zero, Inf or NaN, or a quotient that is not finite and positive, gives 1.
// The division must be the correctly rounded one (the library is compiled that way).
__device__ __forceinline__ float scale_from_amax_value(float amax, float target, int pow2) {
  union { uint32_t u; float f; } a, q, s;
  a.f = amax;
  s.f = 1.0f;
  if (a.u != 0u && a.u < 0x7F800000u) {  // positive, finite, non-zero
    q.f = target / amax;
    if (q.u != 0u && q.u < 0x7F800000u) {
      s.f = q.f;
      if (pow2) {
        if ((q.u >> 23) != 0u) s.u = q.u & 0x7F800000u;
        else s.u = 1u << (31 - __clz((int)q.u));  // subnormal quotient
      }
    }
  }
  return s.f;
}

// binary32 pattern of the value of a code (Eq. (1), Eq. (2), special patterns).
__device__ __forceinline__ uint32_t decode_bits(uint32_t code) {
  const uint32_t s = (code & 0x80u) << 24;
  const uint32_t c = code & 0x7Fu;
  if (c == 0u) return s ? 0x7FC00000u : 0u;  // NaN / Zero
  if (c == kCodeInf) return s | 0x7F800000u;
  if (c < 0x08u) return s | ((c + 104u) << 23);  // 2^(c - 23)
  uint32_t mag, Se, frac;
  if (c < 0x10u) { mag = 0u; Se = 0u; frac = (c & 7u) << 20; }
  else if (c < 0x20u) { mag = 1u; Se = (c >> 3) & 1u; frac = (c & 7u) << 20; }
  else if (c < 0x40u) { mag = 2u | ((c >> 3) & 1u); Se = (c >> 4) & 1u; frac = (c & 7u) << 20; }
  else if (c < 0x60u) { mag = 4u | ((c >> 2) & 3u); Se = (c >> 4) & 1u; frac = (c & 3u) << 21; }
  else { mag = 8u | ((c >> 1) & 7u); Se = (c >> 4) & 1u; frac = (c & 1u) << 22; }
  const uint32_t e = Se ? 127u - mag : 127u + mag;
  return s | (e << 23) | frac;
}

// binary32 -> bfloat16 pattern, round to nearest even, NaN -> 0x7FC0.
__device__ __forceinline__ uint32_t narrow_bf16(uint32_t u) {
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}

}  // namespace hif8dev
