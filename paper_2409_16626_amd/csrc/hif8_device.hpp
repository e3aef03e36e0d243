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

// rounding_mode flag bits as seen by kernels
constexpr uint32_t kFlagSat = 0x10u;
constexpr uint32_t kFlagNan2Zero = 0x20u;

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
template <bool HR, bool SRC16>
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
  if (SRC16) {
    F = (ap >> (sh - 2u)) & 3u;
    T = 2u * ((ybits >> 16) & 1u) + 1u;
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
template <bool HR, bool SRC16>
__device__ __forceinline__ uint32_t encode_alu(uint32_t ybits, uint32_t mode) {
  const uint32_t a = ybits & 0x7FFFFFFFu;
  if (a > 0x7F800000u) return nan_code(mode);
  const uint32_t c = pack_mag(round_mag<HR, SRC16>(a, ybits), overflow_code(mode));
  return c ? (c | ((ybits >> 24) & 0x80u)) : 0u;
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
