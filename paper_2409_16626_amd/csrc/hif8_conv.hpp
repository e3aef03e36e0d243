// Conversion kernels of libhif8 (HiF8, arXiv 2409.16626) for gfx950, templated on the kind of
// the high-precision tensor (binary32, bfloat16, binary16), and their host launchers.
//
// All kernels are HBM-streaming scans: every lane moves 16 bytes per load, U independent
// loads are in flight per lane, nothing is read twice.  There is no contraction, hence no MFMA.
//
//   encode, TA   : the TA code of a non-NaN binary32 value depends only on its top 13 bits
//                  (sign, exponent, 3 kept + 1 rounding mantissa bit), so the hot loop is one
//                  shift and one byte lookup in an 8 KiB table staged in LDS.  The table
//                  itself is produced on the device, once, by the integer encoder.
//   encode, HR   : table-driven rounding to the grid (hr_round_bits), then the same byte lookup.
//                  Simplified SR in every binade is the same kernel with another threshold clamp.
//                  On 16-bit sources HR proper is a single lookup in a 16 KiB table indexed by the
//                  source LSB and the top 13 bits of the scaled pattern (IMPL_HR16).
//   encode, TE   : differs from TA only at exact ties, which need the low 19 bits to be zero;
//                  a second 8 KiB table holds the TE code of those patterns.
//   encode, SR   : standard SR (comparison mode): a hashed threshold per element is added below the
//                  kept mantissa bits, the sum truncated, then the same byte lookup.
//   decode       : 256-entry binary32 table staged in LDS, one multiply by 1/scale.
//   fake-quant   : encode and decode fused; the value never leaves registers.
//   amax         : unsigned max of magnitude patterns; DPP reduction inside a wavefront,
//                  LDS across wavefronts, one atomic max per workgroup.
#pragma once

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <cstring>

#include "hif8.h"
#include "hif8_conv_api.hpp"
#include "hif8_device.hpp"
#include "hif8_host.hpp"
#include "hif8_stream.hpp"

namespace hif8conv {

using namespace hif8dev;
using namespace hif8host;

enum : int { IMPL_TA_LUT = 0, IMPL_TA_ALU = 1, IMPL_HR = 2, IMPL_TE = 3, IMPL_SR = 4, IMPL_HR16 = 5 };

template <int IMPL>
constexpr uint32_t lut_bytes() {
  return (IMPL == IMPL_TE || IMPL == IMPL_HR16) ? 16384u : IMPL == IMPL_TA_ALU ? 16u : 8192u;
}
template <int SRCK>
constexpr int vec_elems() { return SRCK == kSrcF32 ? 4 : 8; }  // elements per 16-byte source vector
template <int SRCK>
constexpr int vec_shift() { return SRCK == kSrcF32 ? 2 : 3; }

// ------------------------------------------------------------------------------------
// small device helpers
// ------------------------------------------------------------------------------------
// Per-exponent parameters of the HR / simplified-SR path (add-and-mask forms: SR14 for binary32 sources, SR2
// for 16-bit sources) in LDS, 4 KiB either way.
//   binary32 sources: 256 entries of 16 bytes {C, -mult, mask, lo | hi << 16}, one ds_read_b128 per element.
//     (Measured alternatives: 32-byte entries -- two reads, and entries 32 bytes apart share banks across
//     exponents: 2.8 TB/s on the wide-range C2 tensor; one dword array per parameter -- conflict-free but five
//     reads per element, and the LDS takes about four cycles per wavefront instruction: 5.3 TB/s; 16-byte
//     entries: 6.1-6.2 TB/s.)
//   16-bit sources: two 256-entry dword arrays add0[], add1[] -- twice as many elements per byte of
//     tensor, and with 16-byte entries {add0, add1, mask} lanes whose exponents are 16 apart collide: 5.3 TB/s
//     on a narrow tensor but 3.9 TB/s on a wide-range one; three arrays gave 5.2-5.4 TB/s on both.  The addend
//     is read from the array the source LSB selects (one read, no select); add1[] starts 32 banks after add0[]
//     so that lanes with the same exponent and different LSBs do not collide.  The mask is not applied at
//     all: the sum is looked up in the truncating encode table (one LDS read per element fewer).
//   standard SR: 256 entries of 16 bytes {offset, width, mask, factor} (sr_exp_entry()).
constexpr uint32_t kHr16Add1 = 256u + 32u;  // dword offset of add1[] in HrLds::w (16-bit sources)
template <int IMPL>
constexpr bool uses_exp_table() { return IMPL == IMPL_HR || IMPL == IMPL_SR; }
template <bool ON>
struct HrLds {
  __attribute__((aligned(16))) uint32_t w[ON ? 4 * 256 : 4];
};

struct EncCtx {
  const uint8_t* lut;  // staged table(s) in LDS
  const uint32_t* hrt; // staged per-exponent parameters in LDS (IMPL_HR, IMPL_SR): HrLds::w
  uint32_t mode;
  uint64_t seed;       // IMPL_SR
  SrKey sr_key;        // IMPL_SR: key pair of the 2^32-element block sr_hi (set by keyed())
  uint32_t sr_hi;
};

// Context for encoding elements of the 2^32-element block that holds element `elem` (standard SR draws its
// thresholds from the low index word and a per-block key pair; other methods ignore it).  The key is
// computed only when the block differs from the one the context was last keyed for.
template <int IMPL>
__device__ __forceinline__ EncCtx keyed(const EncCtx& c, uint64_t elem) {
  if constexpr (IMPL != IMPL_SR) return c;
  const uint32_t hi = (uint32_t)(elem >> 32);
  if (hi == c.sr_hi) return c;
  EncCtx k = c;
  k.sr_key = sr_key(c.seed, hi);
  k.sr_hi = hi;
  return k;
}
// A context keyed for the block of element `elem0` (kernel prologue).
template <int IMPL>
__device__ __forceinline__ EncCtx make_ctx(const uint8_t* lut, const uint32_t* hrt, uint32_t mode, uint64_t seed,
                                           uint64_t elem0 = 0) {
  EncCtx c{lut, hrt, mode, seed, SrKey{0u, 0u}, (uint32_t)(elem0 >> 32)};
  if constexpr (IMPL == IMPL_SR) c.sr_key = sr_key(seed, c.sr_hi);
  return c;
}

// Encode tables of one (NaN option, saturation) pair lie together: TA, TE's ties, truncating (8 KiB each).
// HR on 16-bit sources looks its sums up in the truncating table, everything else in the TA table (TE in
// the first two).
template <int IMPL, int SRCK>
constexpr bool uses_trunc_lut() { return IMPL == IMPL_HR && SRCK != kSrcF32; }
// T = uint8_t: the code tables; T = uint16_t: the value tables of the same layout (upper half of the
// binary32 pattern of each entry's value).
template <int IMPL, int SRCK, typename T = uint8_t>
__device__ __forceinline__ void stage_enc_lut(T* lut, const T* __restrict__ g_lut, uint32_t mode) {
  if (lut_bytes<IMPL>() < 8192u) return;
  // IMPL_HR16 is handed the direct tables [NaN -> 0][sat][source LSB][pattern >> 19] instead
  const uint32_t off = IMPL == IMPL_HR16 ? ((mode & kFlagNan2Zero) ? 32768u : 0u) + ((mode & kFlagSat) ? 16384u : 0u)
                                         : ((mode & kFlagNan2Zero) ? 49152u : 0u) + ((mode & kFlagSat) ? 24576u : 0u) +
                                               (uses_trunc_lut<IMPL, SRCK>() ? 16384u : 0u);
  const uint4* g = reinterpret_cast<const uint4*>(g_lut + off);
  uint4* l = reinterpret_cast<uint4*>(lut);
  for (uint32_t i = threadIdx.x; i < lut_bytes<IMPL>() * (uint32_t)sizeof(T) / 16u; i += blockDim.x) l[i] = g[i];
}
template <int IMPL, int SRCK>
__device__ __forceinline__ void stage_exp_table(uint32_t* w, uint32_t mode) {
  if constexpr (!uses_exp_table<IMPL>()) return;
  const bool ssr = (mode & 0xFu) == kRmSSR;
  for (uint32_t i = threadIdx.x; i < 256u; i += blockDim.x) {
    if constexpr (IMPL == IMPL_SR) {
      const SrExp h = sr_exp_entry(i);
      reinterpret_cast<uint4*>(w)[i] = make_uint4(h.off, h.width, h.mask, __float_as_uint(h.fmul));
    } else if constexpr (SRCK == kSrcF32) {
      const HrExp h = hr_exp_entry(i, ssr);
      reinterpret_cast<uint4*>(w)[i] = make_uint4(h.C, (uint32_t)h.negmult, h.mask, h.lo | (h.hi << 16));
    } else {
      const HrExp16 h = hr16_exp_entry(i, ssr);
      w[i] = h.add0; w[kHr16Add1 + i] = h.add1;  // the mask is folded into the truncating encode table
    }
  }
}
__device__ __forceinline__ void stage_dec_lut(uint32_t* lut, const uint32_t* __restrict__ g_dec) {
  for (uint32_t i = threadIdx.x; i < 256u; i += blockDim.x) lut[i] = g_dec[i];
}

// One element: scaled pattern -> index into the staged encode table (every implementation but the ALU one
// ends in one table lookup).  `elem` is the element's index in the tensor (it selects the threshold of
// standard SR and is unused otherwise); c must be keyed() for elem's block.
// NaN: ybits is always the result of the scale multiply, which returns a quiet NaN (bit 22 set) for any NaN
// input, so the pattern indexes a NaN entry of the table (which holds the code of the NaN option in
// effect); the HR and SR forms pass NaN patterns through unchanged.
template <int IMPL, int SRCK>
__device__ __forceinline__ uint32_t table_index(uint32_t ybits, const EncCtx& c, uint64_t elem) {
  static_assert(IMPL != IMPL_TA_ALU, "the ALU form has no table");
  if constexpr (IMPL == IMPL_TA_LUT) {
    return ybits >> 19;
  } else if constexpr (IMPL == IMPL_SR) {
    // standard SR: add the hashed threshold bits below the kept part, truncate
    const uint4 q = reinterpret_cast<const uint4*>(c.hrt)[(ybits >> 23) & 0xFFu];
    SrExp p;
    p.off = q.x; p.width = q.y; p.mask = q.z; p.fmul = __uint_as_float(q.w);
    return sr_round_bits(ybits, sr_hash((uint32_t)elem, c.sr_key), p) >> 19;
  } else if constexpr (IMPL == IMPL_HR16) {
    // HR proper on a 16-bit source: kept mantissa, the two fraction bits (bit 19 upwards: where three bits
    // are kept Eq. (3) asks for TA, which looks at bit 19 only) and the source LSB decide, so the code comes
    // straight from a table indexed by the LSB and the top 13 bits
    static_assert(SRCK != kSrcF32, "16-bit sources only");
    return (ybits >> 19) | (hr16_lsb<SRCK>(ybits) << 13);
  } else if constexpr (IMPL == IMPL_TE) {
    // a tie needs every bit below the rounding bit to be zero; otherwise TE rounds as TA
    return (ybits >> 19) + ((ybits & 0x7FFFFu) ? 0u : 8192u);
  } else {
    // HR / SSR: rounding to the grid, then the entry of the (now representable) pattern
    uint32_t r;
    if constexpr (SRCK == kSrcF32) {
      const uint4 q = reinterpret_cast<const uint4*>(c.hrt)[(ybits >> 23) & 0xFFu];
      HrExp p;
      p.C = q.x; p.negmult = (int32_t)q.y; p.mask = q.z; p.lo = q.w & 0xFFFFu; p.hi = q.w >> 16;
      r = hr_round_bits<SRCK>(ybits, p);
    } else {
      const uint32_t* t = c.hrt + ((ybits >> 23) & 0xFFu);
      r = hr16_round_sum(ybits, t[hr16_lsb<SRCK>(ybits) * kHr16Add1]);  // no mask: truncating table
    }
    return r >> 19;
  }
}

// One element: scaled pattern -> code.
template <int IMPL, int SRCK>
__device__ __forceinline__ uint32_t encode_one(uint32_t ybits, const EncCtx& c, uint64_t elem) {
  if constexpr (IMPL == IMPL_TA_ALU) return encode_alu<false, SRCK>(ybits, c.mode);
  else return c.lut[table_index<IMPL, SRCK>(ybits, c, elem)];
}

__device__ __forceinline__ uint32_t scaled_bits(uint32_t xbits, float scale) {
  return __float_as_uint(__fmul_rn(__uint_as_float(xbits), scale));
}

// binary32 pattern of the low / high 16-bit half of a dword holding two 16-bit floats
template <int SRCK>
__device__ __forceinline__ uint32_t widen_lo(uint32_t w) {
  if constexpr (SRCK == kSrcBF16) return w << 16;
  else return __float_as_uint((float)__builtin_bit_cast(_Float16, (uint16_t)(w & 0xFFFFu)));
}
template <int SRCK>
__device__ __forceinline__ uint32_t widen_hi(uint32_t w) {
  if constexpr (SRCK == kSrcBF16) return w & 0xFFFF0000u;
  else return __float_as_uint((float)__builtin_bit_cast(_Float16, (uint16_t)(w >> 16)));
}

// element i of a tensor as a binary32 pattern
template <int SRCK>
__device__ __forceinline__ uint32_t load_bits(const void* src, size_t i) {
  if constexpr (SRCK == kSrcF32) return __float_as_uint(reinterpret_cast<const float*>(src)[i]);
  else return widen_lo<SRCK>(reinterpret_cast<const uint16_t*>(src)[i]);
}

// True when the VE elements starting at e0 do not all lie in one 2^32-element block (standard SR only; it can
// happen only when the call's index base is not a multiple of the vector width).
template <int IMPL, int VE>
__device__ __forceinline__ bool straddles_block(uint64_t e0) {
  if constexpr (IMPL != IMPL_SR) return false;
  return (uint32_t)e0 > 0xFFFFFFFFu - (uint32_t)(VE - 1);
}

template <int IMPL>
__device__ __forceinline__ uint32_t encode4_f32(const uint4& v, float scale, const EncCtx& c0_, uint64_t e0) {
  const uint32_t y[4] = {scaled_bits(v.x, scale), scaled_bits(v.y, scale), scaled_bits(v.z, scale), scaled_bits(v.w, scale)};
  uint32_t r = 0;
  if (straddles_block<IMPL, 4>(e0)) {
#pragma unroll
    for (int j = 0; j < 4; ++j) r |= encode_one<IMPL, kSrcF32>(y[j], keyed<IMPL>(c0_, e0 + j), e0 + j) << (8 * j);
    return r;
  }
  const EncCtx c = keyed<IMPL>(c0_, e0);
#pragma unroll
  for (int j = 0; j < 4; ++j) r |= encode_one<IMPL, kSrcF32>(y[j], c, e0 + j) << (8 * j);
  return r;
}

// two 16-bit floats in one dword -> two codes in the low 16 bits
template <int IMPL, int SRCK>
__device__ __forceinline__ uint32_t encode2_16(uint32_t w, float scale, const EncCtx& c, uint64_t e0) {
  const uint32_t c0 = encode_one<IMPL, SRCK>(scaled_bits(widen_lo<SRCK>(w), scale), c, e0);
  const uint32_t c1 = encode_one<IMPL, SRCK>(scaled_bits(widen_hi<SRCK>(w), scale), c, e0 + 1);
  return c0 | (c1 << 8);
}
template <int IMPL, int SRCK>
__device__ __forceinline__ uint2 encode8_16(const uint4& v, float scale, const EncCtx& c0_, uint64_t e0) {
  uint2 o;
  if (straddles_block<IMPL, 8>(e0)) {
    const uint32_t w[4] = {v.x, v.y, v.z, v.w};
    uint32_t q[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const uint32_t c0 = encode_one<IMPL, SRCK>(scaled_bits(widen_lo<SRCK>(w[j]), scale), keyed<IMPL>(c0_, e0 + 2 * j), e0 + 2 * j);
      const uint32_t c1 = encode_one<IMPL, SRCK>(scaled_bits(widen_hi<SRCK>(w[j]), scale), keyed<IMPL>(c0_, e0 + 2 * j + 1), e0 + 2 * j + 1);
      q[j] = c0 | (c1 << 8);
    }
    o.x = q[0] | (q[1] << 16);
    o.y = q[2] | (q[3] << 16);
    return o;
  }
  const EncCtx c = keyed<IMPL>(c0_, e0);
  o.x = encode2_16<IMPL, SRCK>(v.x, scale, c, e0) | (encode2_16<IMPL, SRCK>(v.y, scale, c, e0 + 2) << 16);
  o.y = encode2_16<IMPL, SRCK>(v.z, scale, c, e0 + 4) | (encode2_16<IMPL, SRCK>(v.w, scale, c, e0 + 6) << 16);
  return o;
}

__device__ __forceinline__ uint32_t descale_bits(uint32_t code, const uint32_t* dec, float inv) {
  return __float_as_uint(__fmul_rn(__uint_as_float(dec[code & 0xFFu]), inv));
}

// binary32 pattern(s) -> 16-bit float pattern(s), round to nearest even (hardware conversions:
// v_cvt_pk_bf16_f32 / v_cvt_f16_f32); NaN -> 0x7FC0 / 0x7E00 for the quiet NaN decode produces
typedef float f32x2_t __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));
template <int DSTK>
__device__ __forceinline__ uint32_t narrow2(uint32_t b0, uint32_t b1) {
  const f32x2_t f = {__uint_as_float(b0), __uint_as_float(b1)};
  if constexpr (DSTK == kSrcBF16) return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, bf16x2_t));
  else return __builtin_bit_cast(uint32_t, __builtin_convertvector(f, f16x2_t));
}
template <int DSTK>
__device__ __forceinline__ uint32_t narrow1(uint32_t b) {
  if constexpr (DSTK == kSrcBF16) return narrow_bf16(b);
  else return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)__uint_as_float(b));
}
template <int DSTK>
__device__ __forceinline__ uint32_t descale2_16(uint32_t c0, uint32_t c1, const uint32_t* dec, float inv) {
  return narrow2<DSTK>(descale_bits(c0, dec, inv), descale_bits(c1, dec, inv));
}
template <int DSTK>
__device__ __forceinline__ uint4 descale8_16(const uint2& w, const uint32_t* dec, float inv) {
  uint4 o;
  o.x = descale2_16<DSTK>(w.x, w.x >> 8, dec, inv);
  o.y = descale2_16<DSTK>(w.x >> 16, w.x >> 24, dec, inv);
  o.z = descale2_16<DSTK>(w.y, w.y >> 8, dec, inv);
  o.w = descale2_16<DSTK>(w.y >> 16, w.y >> 24, dec, inv);
  return o;
}
__device__ __forceinline__ uint4 descale4_f32(uint32_t w, const uint32_t* dec, float inv) {
  uint4 o;
  o.x = descale_bits(w, dec, inv);
  o.y = descale_bits(w >> 8, dec, inv);
  o.z = descale_bits(w >> 16, dec, inv);
  o.w = descale_bits(w >> 24, dec, inv);
  return o;
}

// running magnitude maximum of one 16-byte vector: binary32 -> magnitude pattern; 16-bit
// floats -> two 15-bit magnitudes, one per 16-bit half (folded by fold_amax at the end; the
// magnitude patterns of bfloat16 and of binary16 both order like the values)
typedef uint16_t u16x2_t __attribute__((ext_vector_type(2)));
template <int SRCK>
__device__ __forceinline__ uint32_t vec_amax(uint32_t m, const uint4& v) {
  if constexpr (SRCK == kSrcF32) {
    return umax(m, umax(umax(v.x & 0x7FFFFFFFu, v.y & 0x7FFFFFFFu),
                        umax(v.z & 0x7FFFFFFFu, v.w & 0x7FFFFFFFu)));
  } else {
    u16x2_t mm = __builtin_bit_cast(u16x2_t, m);
    mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2_t, v.x & 0x7FFF7FFFu));
    mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2_t, v.y & 0x7FFF7FFFu));
    mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2_t, v.z & 0x7FFF7FFFu));
    mm = __builtin_elementwise_max(mm, __builtin_bit_cast(u16x2_t, v.w & 0x7FFF7FFFu));
    return __builtin_bit_cast(uint32_t, mm);
  }
}
// running maximum -> binary32 magnitude pattern
template <int SRCK>
__device__ __forceinline__ uint32_t fold_amax(uint32_t m) {
  if constexpr (SRCK == kSrcF32) return m;
  else return widen_lo<SRCK>(umax(m & 0xFFFFu, m >> 16));
}

// ------------------------------------------------------------------------------------
// Where a cast kernel takes its scale pair {scale, fl32(1/scale)} from:
//   by value            scale, inv (host-validated)
//   d_scale2            two floats in device memory, written earlier on the stream
//   parts               the per-workgroup maxima that k_amax_parts left for this tensor: every workgroup of the
//                       cast reduces them (a few hundred words, L2-resident) and derives amax, scale and 1/scale
//                       itself, so that per-tensor scaling needs two launches, no clearing launch and no atomics;
//                       workgroup 0 publishes amax and the pair to out_amax / out_scale2.
// ------------------------------------------------------------------------------------
struct ScaleArg {
  float scale, inv;
  const float* d_scale2;
  const uint32_t* parts;
  uint32_t nparts;
  float target;
  int pow2;
  float* out_amax;
  float* out_scale2;
};
inline ScaleArg scale_by_value(float scale, float inv) { return ScaleArg{scale, inv, nullptr, nullptr, 0u, 0.0f, 0, nullptr, nullptr}; }
inline ScaleArg scale_on_device(const float* d_scale2) { return ScaleArg{1.0f, 1.0f, d_scale2, nullptr, 0u, 0.0f, 0, nullptr, nullptr}; }


// Scale pair of the plain forms (uniform over the grid: scalar loads).
__device__ __forceinline__ float plain_scale(const ScaleArg& a) { return a.d_scale2 ? a.d_scale2[0] : a.scale; }
__device__ __forceinline__ float plain_inv(const ScaleArg& a) { return a.d_scale2 ? a.d_scale2[1] : a.inv; }

// The parts form.  First half (before the workgroup barrier of the kernel prologue): wavefront maxima of the
// partial maxima into LDS.  Second half (after that barrier): every lane folds them and derives the pair;
// workgroup 0 publishes amax and the pair.
struct ScaleLds {
  uint32_t wave_m[16];
};
__device__ __forceinline__ void parts_before_barrier(const ScaleArg& a, ScaleLds& l) {
  uint32_t m = 0;
  for (uint32_t i = threadIdx.x; i < a.nparts; i += blockDim.x) m = umax(m, a.parts[i]);
  m = wave_max_u32(m);
  if ((threadIdx.x & 63u) == 0u) l.wave_m[threadIdx.x >> 6] = m;
}
__device__ __forceinline__ void parts_after_barrier(const ScaleArg& a, const ScaleLds& l, float& scale, float& inv) {
  const uint32_t nw = (blockDim.x + 63u) >> 6;
  uint32_t r = l.wave_m[0];
  for (uint32_t w = 1; w < nw; ++w) r = umax(r, l.wave_m[w]);
  const float amax = __uint_as_float(r);
  scale = scale_from_amax_value(amax, a.target, a.pow2);
  inv = 1.0f / scale;
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    *a.out_amax = amax;
    a.out_scale2[0] = scale;
    a.out_scale2[1] = inv;
  }
}

// Index of the element a kernel's position `local` has in the threshold stream of standard SR; other rounding
// methods never look at it, so their kernels carry no base.
template <int IMPL>
__device__ __forceinline__ uint64_t stream_index(const SrArg& sr, uint64_t local) {
  if constexpr (IMPL == IMPL_SR) return sr.base + local;
  else return local;
}

// ------------------------------------------------------------------------------------
// streaming kernels.  The ragged tail (n modulo the vector width) is done element-wise by
// workgroup 0.
// ------------------------------------------------------------------------------------
// PARTS: the scale comes from the partial maxima of k_amax<.., PARTS> (ScaleArg::parts); otherwise by value or
// from d_scale2.
template <int U, int IMPL, int SRCK, bool PARTS>
__global__ void __launch_bounds__(1024)
k_encode(const void* __restrict__ src, uint8_t* __restrict__ dst, size_t n, ScaleArg sa,
         uint32_t* __restrict__ amax_acc, uint32_t mode, SrArg sr, const uint8_t* __restrict__ g_lut, Walk walk) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[lut_bytes<IMPL>()];
  __shared__ HrLds<uses_exp_table<IMPL>()> hrt;
  __shared__ ScaleLds sl;
  const EncCtx ctx = make_ctx<IMPL>(lut, hrt.w, mode, sr.seed, stream_index<IMPL>(sr, 0));
  float scale = 1.0f, inv = 1.0f;
  if constexpr (!PARTS) scale = plain_scale(sa);
  const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(src);
  constexpr int VE = vec_elems<SRCK>();
  const size_t nvec = n >> vec_shift<SRCK>();
  uint32_t m = 0;  // amax of the unscaled input, only tracked when amax_acc != nullptr
  tile_loop<U, uint4>(
      nvec, walk, [&](size_t idx) { return ld_stream(src4 + idx); },
      [&](size_t idx, const uint4& v) {
        if (amax_acc) m = vec_amax<SRCK>(m, v);
        if constexpr (SRCK == kSrcF32)
          st_stream(reinterpret_cast<uint32_t*>(dst) + idx, encode4_f32<IMPL>(v, scale, ctx, stream_index<IMPL>(sr, idx * VE)));
        else
          st_stream(reinterpret_cast<uint2*>(dst) + idx, encode8_16<IMPL, SRCK>(v, scale, ctx, stream_index<IMPL>(sr, idx * VE)));
      },
      [&]() {
        if (IMPL != IMPL_TA_ALU) {
          stage_enc_lut<IMPL, SRCK>(lut, g_lut, mode);
          stage_exp_table<IMPL, SRCK>(hrt.w, mode);
        }
        if constexpr (PARTS) parts_before_barrier(sa, sl);
        if (IMPL != IMPL_TA_ALU || PARTS) __syncthreads();
        if constexpr (PARTS) parts_after_barrier(sa, sl, scale, inv);
      });
  const size_t t = nvec * VE + threadIdx.x;
  m = fold_amax<SRCK>(m);
  if (blockIdx.x == 0 && t < n) {
    const uint32_t xb = load_bits<SRCK>(src, t);
    m = umax(m, xb & 0x7FFFFFFFu);
    const uint64_t e = stream_index<IMPL>(sr, t);
    dst[t] = (uint8_t)encode_one<IMPL, SRCK>(scaled_bits(xb, scale), keyed<IMPL>(ctx, e), e);
  }
  if (amax_acc) block_max_to_global(m, amax_acc);
}

template <int U, int DSTK>
__global__ void __launch_bounds__(1024)
k_decode(const uint8_t* __restrict__ src, void* __restrict__ dst, size_t n, float inv_arg,
         const float* __restrict__ d_scale2, const uint32_t* __restrict__ g_dec, Walk walk) {
  __shared__ uint32_t dec[256];
  const float inv = d_scale2 ? d_scale2[1] : inv_arg;  // fl32(1/scale)
  constexpr int VE = vec_elems<DSTK>();
  const size_t nvec = n >> vec_shift<DSTK>();
  uint4* __restrict__ dst4 = reinterpret_cast<uint4*>(dst);
  auto prologue = [&]() {
    stage_dec_lut(dec, g_dec);
    __syncthreads();
  };
  if constexpr (DSTK == kSrcF32) {
    const uint32_t* __restrict__ s4 = reinterpret_cast<const uint32_t*>(src);
    tile_loop<U, uint32_t>(
        nvec, walk, [&](size_t idx) { return ld_stream(s4 + idx); },
        [&](size_t idx, uint32_t w) { st_stream(dst4 + idx, descale4_f32(w, dec, inv)); }, prologue);
  } else {
    const uint2* __restrict__ s8 = reinterpret_cast<const uint2*>(src);
    tile_loop<U, uint2>(
        nvec, walk, [&](size_t idx) { return ld_stream(s8 + idx); },
        [&](size_t idx, const uint2& w) { st_stream(dst4 + idx, descale8_16<DSTK>(w, dec, inv)); }, prologue);
  }
  const size_t t = nvec * VE + threadIdx.x;
  if (blockIdx.x == 0 && t < n) {
    const uint32_t b = descale_bits(src[t], dec, inv);
    if constexpr (DSTK == kSrcF32) reinterpret_cast<uint32_t*>(dst)[t] = b;
    else reinterpret_cast<uint16_t*>(dst)[t] = (uint16_t)narrow1<DSTK>(b);
  }
}

// fake-quant: src and dst may alias (each lane reads its own vectors before it writes them)
template <int U, int IMPL, bool CODES, int SRCK, bool PARTS>
__global__ void __launch_bounds__(1024)
k_fake_quant(const void* src, void* dst, uint8_t* codes, size_t n, ScaleArg sa, uint32_t* amax_acc, uint32_t mode,
             SrArg sr, const uint8_t* __restrict__ g_lut, const uint32_t* __restrict__ g_dec, Walk walk) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[lut_bytes<IMPL>()];
  __shared__ HrLds<uses_exp_table<IMPL>()> hrt;
  __shared__ uint32_t dec[256];
  __shared__ ScaleLds sl;
  const EncCtx ctx = make_ctx<IMPL>(lut, hrt.w, mode, sr.seed, stream_index<IMPL>(sr, 0));
  float scale = 1.0f, inv = 1.0f;
  if constexpr (!PARTS) {
    scale = plain_scale(sa);
    inv = plain_inv(sa);
  }
  auto prologue = [&]() {
    stage_enc_lut<IMPL, SRCK>(lut, g_lut, mode);
    stage_exp_table<IMPL, SRCK>(hrt.w, mode);
    stage_dec_lut(dec, g_dec);
    if constexpr (PARTS) parts_before_barrier(sa, sl);
    __syncthreads();
    if constexpr (PARTS) parts_after_barrier(sa, sl, scale, inv);
  };
  const uint4* src4 = reinterpret_cast<const uint4*>(src);
  uint4* dst4 = reinterpret_cast<uint4*>(dst);
  constexpr int VE = vec_elems<SRCK>();
  const size_t nvec = n >> vec_shift<SRCK>();
  uint32_t m = 0;
  tile_loop<U, uint4>(
      nvec, walk, [&](size_t idx) { return ld_stream(src4 + idx); },
      [&](size_t idx, const uint4& v) {
        if (amax_acc) m = vec_amax<SRCK>(m, v);
        if constexpr (SRCK == kSrcF32) {
          const uint32_t w = encode4_f32<IMPL>(v, scale, ctx, stream_index<IMPL>(sr, idx * VE));
          st_stream(dst4 + idx, descale4_f32(w, dec, inv));
          if (CODES) st_stream(reinterpret_cast<uint32_t*>(codes) + idx, w);
        } else {
          const uint2 w = encode8_16<IMPL, SRCK>(v, scale, ctx, stream_index<IMPL>(sr, idx * VE));
          st_stream(dst4 + idx, descale8_16<SRCK>(w, dec, inv));
          if (CODES) st_stream(reinterpret_cast<uint2*>(codes) + idx, w);
        }
      },
      prologue);
  const size_t t = nvec * VE + threadIdx.x;
  m = fold_amax<SRCK>(m);
  if (blockIdx.x == 0 && t < n) {
    const uint32_t xb = load_bits<SRCK>(src, t);
    m = umax(m, xb & 0x7FFFFFFFu);
    const uint64_t e = stream_index<IMPL>(sr, t);
    const uint32_t c = encode_one<IMPL, SRCK>(scaled_bits(xb, scale), keyed<IMPL>(ctx, e), e);
    const uint32_t b = descale_bits(c, dec, inv);
    if constexpr (SRCK == kSrcF32) reinterpret_cast<uint32_t*>(dst)[t] = b;
    else reinterpret_cast<uint16_t*>(dst)[t] = (uint16_t)narrow1<SRCK>(b);
    if (CODES) codes[t] = (uint8_t)c;
  }
  if (amax_acc) block_max_to_global(m, amax_acc);
}

// ------------------------------------------------------------------------------------
// element-per-lane kernels for pointers that do not meet the fast path's alignment
// (integer encoder, any rounding method)
// ------------------------------------------------------------------------------------
template <int SRCK>
__global__ void __launch_bounds__(256)
k_encode_elem(const void* src, uint8_t* dst, size_t n, float scale_arg, const float* d_scale2,
              uint32_t* amax_acc, uint32_t mode, SrArg sr) {
  const float scale = d_scale2 ? d_scale2[0] : scale_arg;
  uint32_t m = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x) {
    const uint32_t xb = load_bits<SRCK>(src, i);
    m = umax(m, xb & 0x7FFFFFFFu);
    dst[i] = (uint8_t)encode_any<SRCK>(scaled_bits(xb, scale), mode, sr_threshold(sr.seed, sr.base + i));
  }
  if (amax_acc) block_max_to_global(m, amax_acc);
}

template <int DSTK>
__global__ void __launch_bounds__(256)
k_decode_elem(const uint8_t* src, void* dst, size_t n, float inv_arg, const float* d_scale2) {
  const float inv = d_scale2 ? d_scale2[1] : inv_arg;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x) {
    const uint32_t b = __float_as_uint(__fmul_rn(__uint_as_float(decode_bits(src[i])), inv));
    if constexpr (DSTK == kSrcF32) reinterpret_cast<uint32_t*>(dst)[i] = b;
    else reinterpret_cast<uint16_t*>(dst)[i] = (uint16_t)narrow1<DSTK>(b);
  }
}

template <int SRCK>
__global__ void __launch_bounds__(256)
k_fake_quant_elem(const void* src, void* dst, uint8_t* codes, size_t n, float scale_arg,
                  float inv_arg, const float* d_scale2, uint32_t* amax_acc, uint32_t mode,
                  SrArg sr) {
  const float scale = d_scale2 ? d_scale2[0] : scale_arg;
  const float inv = d_scale2 ? d_scale2[1] : inv_arg;
  uint32_t m = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x) {
    const uint32_t xb = load_bits<SRCK>(src, i);
    m = umax(m, xb & 0x7FFFFFFFu);
    const uint32_t c = encode_any<SRCK>(scaled_bits(xb, scale), mode, sr_threshold(sr.seed, sr.base + i));
    const uint32_t b = __float_as_uint(__fmul_rn(__uint_as_float(decode_bits(c)), inv));
    if constexpr (SRCK == kSrcF32) reinterpret_cast<uint32_t*>(dst)[i] = b;
    else reinterpret_cast<uint16_t*>(dst)[i] = (uint16_t)narrow1<SRCK>(b);
    if (codes) codes[i] = (uint8_t)c;
  }
  if (amax_acc) block_max_to_global(m, amax_acc);
}

// ------------------------------------------------------------------------------------
// amax (magnitude patterns as binary32 bits)
// ------------------------------------------------------------------------------------
// PARTS = false: one atomic max per workgroup into *out (which the host cleared on the stream before).
// PARTS = true : out[blockIdx.x] = maximum of this workgroup's share, no atomics and nothing to clear; the
//                cast that follows reduces the array (ScaleArg::parts).
template <int U, int SRCK, bool NT, bool PARTS>
__global__ void __launch_bounds__(1024)
k_amax(const void* __restrict__ src, size_t n, uint32_t* __restrict__ out, Walk walk) {
  const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(src);
  const size_t nvec = n >> vec_shift<SRCK>();
  uint32_t m = 0;
  tile_loop<U, uint4>(
      nvec, walk, [&](size_t idx) { return NT ? ld_stream(src4 + idx) : src4[idx]; },
      [&](size_t, const uint4& v) { m = vec_amax<SRCK>(m, v); }, []() {});
  m = fold_amax<SRCK>(m);
  const size_t t = nvec * vec_elems<SRCK>() + threadIdx.x;
  if (blockIdx.x == 0 && t < n) m = umax(m, load_bits<SRCK>(src, t) & 0x7FFFFFFFu);
  if constexpr (PARTS) {
    const uint32_t r = block_max_thread0(m);
    if (threadIdx.x == 0) out[blockIdx.x] = r;
  } else {
    block_max_to_global(m, out);
  }
}

template <int SRCK>
__global__ void __launch_bounds__(256)
k_amax_elem(const void* __restrict__ src, size_t n, uint32_t* __restrict__ out) {
  uint32_t m = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n;
       i += (size_t)gridDim.x * blockDim.x)
    m = umax(m, load_bits<SRCK>(src, i) & 0x7FFFFFFFu);
  block_max_to_global(m, out);
}

// ------------------------------------------------------------------------------------
// multi-tensor cast: many tensors per launch, so that a list of small tensors is not bound by
// launch gaps.  All tensors share one global tile index space; items[i].first_tile is the
// prefix sum of tile counts.  A tile is kMultiBlock * kMultiUnroll vector units of one tensor.
// ------------------------------------------------------------------------------------
// Tiles per workgroup of the multi-tensor cast.  Two keep the most workgroups in flight, which is what the plain
// TA cast wants; with the amax accumulation (one atomic per workgroup and tensor) or a larger table to stage per
// workgroup (every implementation but TA), four measured 3-16 % faster on the 225-tensor LLM weight list.
template <int IMPL, bool ACC>
__host__ __device__ constexpr uint32_t multi_tpw_encode() { return (ACC || IMPL != IMPL_TA_LUT) ? 4u : 2u; }
constexpr uint32_t kMultiTpwAmax = 8;

// largest i with items[i].first_tile <= tile (zero-size items are skipped by construction)
__device__ __forceinline__ uint32_t multi_find_item(const hif8_cast_item* __restrict__ items,
                                                    uint32_t count, uint64_t tile) {
  uint32_t lo = 0, hi = count;
  while (hi - lo > 1u) {
    const uint32_t mid = (lo + hi) >> 1;
    if (items[mid].first_tile <= tile) lo = mid; else hi = mid;
  }
  return lo;
}

template <int SRCK>
__device__ __forceinline__ uint64_t multi_item_tiles(uint64_t n) {
  const uint64_t nvec = n >> vec_shift<SRCK>();
  const uint64_t t = (nvec + kMultiTileVec - 1) / kMultiTileVec;
  return (t == 0 && n != 0) ? 1 : t;
}

// amax of the tiles [first, first + TPW) below tile_end: one atomic max per tensor touched.
// NT: non-temporal loads (the tensors are not read again soon); otherwise ordinary loads, which leave the
// data in the last-level cache for the cast of the same tiles that follows.
template <int SRCK, bool NT, uint32_t TPW>
__device__ __forceinline__ void multi_amax_tiles(const hif8_cast_item* __restrict__ items, uint32_t count,
                                                 uint64_t first, uint64_t tile_end, uint32_t* __restrict__ amax_out) {
  uint32_t m = 0;     // vector part, in the packed form of vec_amax
  uint32_t mt = 0;    // ragged-tail part, binary32 magnitude pattern
  uint32_t cur = 0xFFFFFFFFu;
  for (uint32_t i = 0; i < TPW; ++i) {
    const uint64_t tile = first + i;
    if (tile >= tile_end) break;
    const uint32_t it = multi_find_item(items, count, tile);
    if (it != cur) {
      if (cur != 0xFFFFFFFFu) {
        block_max_to_global(umax(fold_amax<SRCK>(m), mt), amax_out + cur);
        __syncthreads();
      }
      cur = it;
      m = 0;
      mt = 0;
    }
    const uint64_t n = items[it].n;
    const uint64_t nvec = n >> vec_shift<SRCK>();
    const uint64_t local = tile - items[it].first_tile;
    const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(items[it].src);
    const uint64_t v0 = local * kMultiTileVec + threadIdx.x;
    if (nvec != 0) {
      // unconditional loads, so that all are in flight together: an index past the end reads the last vector
      // again, which leaves the maximum as it is
      uint4 v[kMultiUnroll];
#pragma unroll
      for (int j = 0; j < kMultiUnroll; ++j) {
        const uint64_t idx = v0 + (uint64_t)j * kMultiBlock;
        const uint4* q = src4 + (idx < nvec ? idx : nvec - 1);
        v[j] = NT ? ld_stream(q) : *q;
      }
#pragma unroll
      for (int j = 0; j < kMultiUnroll; ++j) m = vec_amax<SRCK>(m, v[j]);
    }
    // ragged tail of the tensor, done with its last tile
    if (local + 1 == multi_item_tiles<SRCK>(n)) {
      const uint64_t t = nvec * vec_elems<SRCK>() + threadIdx.x;
      if (t < n) mt = umax(mt, load_bits<SRCK>(items[it].src, t) & 0x7FFFFFFFu);
    }
  }
  if (cur != 0xFFFFFFFFu) block_max_to_global(umax(fold_amax<SRCK>(m), mt), amax_out + cur);
}

// Cast of the tiles [first, first + multi_tpw_encode()) below tile_end, each tensor with the scale d_scale2[2 * item]
// (written earlier on the stream).  ACC: also accumulate the amax of every tensor's source into amax_acc[item]
// (delayed scaling: the scales in use come from earlier iterations, the accumulators feed the next update).
// The encode tables must be staged (and a barrier passed) before.
template <int IMPL, int SRCK, bool ACC>
__device__ __forceinline__ void multi_encode_tiles(const hif8_cast_item* __restrict__ items, uint32_t count,
                                                   uint64_t first, uint64_t tile_end, const float* __restrict__ d_scale2,
                                                   uint32_t* __restrict__ amax_acc, const EncCtx& ctx) {
  constexpr int VE = vec_elems<SRCK>();
  uint32_t m = 0, mt = 0, cur = 0xFFFFFFFFu;  // ACC: as in multi_amax_tiles
  for (uint32_t i = 0; i < multi_tpw_encode<IMPL, ACC>(); ++i) {
    const uint64_t tile = first + i;
    if (tile >= tile_end) break;
    const uint32_t it = multi_find_item(items, count, tile);
    if (ACC && it != cur) {
      if (cur != 0xFFFFFFFFu) {
        block_max_to_global(umax(fold_amax<SRCK>(m), mt), amax_acc + cur);
        __syncthreads();
      }
      cur = it;
      m = 0;
      mt = 0;
    }
    const uint64_t n = items[it].n;
    const uint64_t nvec = n >> vec_shift<SRCK>();
    const uint64_t local = tile - items[it].first_tile;
    const float scale = d_scale2[2 * it];
    const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(items[it].src);
    uint8_t* __restrict__ dst = items[it].dst;
    const uint64_t v0 = local * kMultiTileVec + threadIdx.x;
    if (nvec != 0) {
      uint4 v[kMultiUnroll];
#pragma unroll
      for (int j = 0; j < kMultiUnroll; ++j) {
        const uint64_t idx = v0 + (uint64_t)j * kMultiBlock;
        if (idx < nvec) v[j] = ld_stream(src4 + idx);
        else if (ACC) v[j] = make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int j = 0; j < kMultiUnroll; ++j) {
        const uint64_t idx = v0 + (uint64_t)j * kMultiBlock;
        if (ACC) m = vec_amax<SRCK>(m, v[j]);
        if (idx < nvec) {
          if constexpr (SRCK == kSrcF32)
            st_stream(reinterpret_cast<uint32_t*>(dst) + idx, encode4_f32<IMPL>(v[j], scale, ctx, idx * VE));
          else
            st_stream(reinterpret_cast<uint2*>(dst) + idx, encode8_16<IMPL, SRCK>(v[j], scale, ctx, idx * VE));
        }
      }
    }
    if (local + 1 == multi_item_tiles<SRCK>(n)) {
      const uint64_t t = nvec * VE + threadIdx.x;
      if (t < n) {
        const uint32_t xb = load_bits<SRCK>(items[it].src, t);
        if (ACC) mt = umax(mt, xb & 0x7FFFFFFFu);
        dst[t] = (uint8_t)encode_one<IMPL, SRCK>(scaled_bits(xb, scale), keyed<IMPL>(ctx, t), t);
      }
    }
  }
  if (ACC && cur != 0xFFFFFFFFu) block_max_to_global(umax(fold_amax<SRCK>(m), mt), amax_acc + cur);
}

template <int SRCK>
__global__ void __launch_bounds__(kMultiBlock)
k_multi_amax(const hif8_cast_item* __restrict__ items, uint32_t count, uint64_t total_tiles,
             uint32_t* __restrict__ amax_out) {
  multi_amax_tiles<SRCK, true, kMultiTpwAmax>(items, count, (uint64_t)blockIdx.x * kMultiTpwAmax, total_tiles, amax_out);
}

template <int IMPL, int SRCK, bool ACC>
__global__ void __launch_bounds__(kMultiBlock)
k_multi_encode(const hif8_cast_item* __restrict__ items, uint32_t count, uint64_t total_tiles,
               const float* __restrict__ d_scale2, uint32_t* __restrict__ amax_acc, uint32_t mode, uint64_t seed,
               const uint8_t* __restrict__ g_lut) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[lut_bytes<IMPL>()];
  __shared__ HrLds<uses_exp_table<IMPL>()> hrt;
  const EncCtx ctx = make_ctx<IMPL>(lut, hrt.w, mode, seed);
  stage_enc_lut<IMPL, SRCK>(lut, g_lut, mode);
  stage_exp_table<IMPL, SRCK>(hrt.w, mode);
  __syncthreads();
  multi_encode_tiles<IMPL, SRCK, ACC>(items, count, (uint64_t)blockIdx.x * multi_tpw_encode<IMPL, ACC>(), total_tiles, d_scale2,
                                      amax_acc, ctx);
}

// One stage of the group-wise multi-tensor cast: am_wgs workgroups gather the amax of the tensors am[] of one
// group while enc_wgs workgroups cast the tensors enc[] of the group before it -- whose amax the previous stage
// gathered, so that their source now sits in the last-level cache.  One launch per group.  The tensors of a stage
// travel by value in the kernel arguments (at most kStageItems per role), each with its first position in the
// role's index space, so a workgroup finds its tensor with a few scalar compares.
//   cast: a workgroup owns kStageVec consecutive 16-byte vectors of one tensor, requests all of them at once,
//         and the last workgroup of a tensor also does its ragged tail;
//   amax: few, long-lived workgroups (at most one per compute unit) walk the chunks of kStageVecAmax vectors of
//         all tensors of the group with a stride, and end with one atomic max per tensor they touched.  (One
//         short-lived workgroup per chunk was measured first: a thousand workgroups that start together all
//         find the accumulator at zero, and their atomics on one address, served one after the other at about
//         7 ns each, then cost as much as the reads.)
// The amax workgroups come first in index order: the dispatcher hands workgroups out in that order, so they
// hold one slot of every compute unit for the whole stage and the short-lived casting workgroups stream
// through the other slots.
constexpr int kStageItems = 16;
constexpr int kStageBlock = 512;
constexpr int kStageU = 4;       // cast: 16-byte loads per lane
constexpr int kStageUAmax = 8;   // amax: 16-byte loads per lane
constexpr uint32_t kStageVec = kStageBlock * kStageU;
constexpr uint32_t kStageVecAmax = kStageBlock * kStageUAmax;
struct StageItem {
  const void* src;
  uint8_t* dst;
  uint64_t n;
  uint32_t wg_first;  // cast: first workgroup of the role that works on this tensor; amax: its first chunk
  uint32_t index;     // position in the caller's list (its amax / scale pair entries)
};
struct StageArgs {
  StageItem enc[kStageItems];
  StageItem am[kStageItems];
  uint32_t n_enc, n_am;
  uint32_t enc_wgs, am_wgs;
  uint32_t am_chunks;  // chunks of all tensors of am[]
};
template <int SRCK>
__host__ __device__ inline uint32_t stage_item_wgs(uint64_t n, uint32_t vec_per_wg) {
  const uint64_t nvec = n >> vec_shift<SRCK>();
  const uint64_t w = (nvec + vec_per_wg - 1) / vec_per_wg;
  return (uint32_t)((w == 0 && n != 0) ? 1 : w);
}

// entry of `items` whose workgroup range holds w (wg_first ascending, items[0].wg_first == 0)
__device__ __forceinline__ int stage_find(const StageItem* items, uint32_t n_items, uint32_t w) {
  int j = 0;
#pragma unroll
  for (int k = 1; k < kStageItems; ++k)
    if ((uint32_t)k < n_items && items[k].wg_first <= w) j = k;
  return j;
}

template <int IMPL, int SRCK>
__global__ void __launch_bounds__(kStageBlock)
k_group_stage(const StageArgs sg, uint32_t* __restrict__ amax, float* __restrict__ d_scale2, float target, int pow2,
              uint32_t mode, uint64_t seed, const uint8_t* __restrict__ g_lut) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[lut_bytes<IMPL>()];
  __shared__ HrLds<uses_exp_table<IMPL>()> hrt;
  constexpr int VE = vec_elems<SRCK>();
  const bool is_amax = blockIdx.x < sg.am_wgs;
  const uint32_t w = is_amax ? blockIdx.x : blockIdx.x - sg.am_wgs;  // index within the role
  if (!is_amax) {
    const int j = stage_find(sg.enc, sg.n_enc, w);
    const StageItem it = sg.enc[j];
    const uint64_t nvec = it.n >> vec_shift<SRCK>();
    const uint32_t local = w - it.wg_first;
    const uint64_t v0 = (uint64_t)local * kStageVec + threadIdx.x;
    const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(it.src);
    const bool full = (uint64_t)(local + 1) * kStageVec <= nvec;  // whole chunk inside the tensor: no guards
    uint4 v[kStageU];
    if (nvec != 0) {  // (a tensor shorter than one vector has only its ragged tail)
#pragma unroll
      for (int u = 0; u < kStageU; ++u) {
        const uint64_t idx = v0 + (uint64_t)u * kStageBlock;
        v[u] = ld_stream(src4 + ((full || idx < nvec) ? idx : nvec - 1));  // past the end: the last vector again, not stored
      }
    }
    const EncCtx ctx = make_ctx<IMPL>(lut, hrt.w, mode, seed);
    stage_enc_lut<IMPL, SRCK>(lut, g_lut, mode);
    stage_exp_table<IMPL, SRCK>(hrt.w, mode);
    const float scale = scale_from_amax_value(__uint_as_float(amax[it.index]), target, pow2);
    if (local == 0 && threadIdx.x == 0) {
      d_scale2[2 * it.index] = scale;
      d_scale2[2 * it.index + 1] = 1.0f / scale;
    }
    __syncthreads();
#pragma unroll
    for (int u = 0; u < kStageU; ++u) {
      const uint64_t idx = v0 + (uint64_t)u * kStageBlock;
      if constexpr (SRCK == kSrcF32) {
        const uint32_t c = encode4_f32<IMPL>(v[u], scale, ctx, idx * VE);
        if (full) st_stream(reinterpret_cast<uint32_t*>(it.dst) + idx, c);
        else if (idx < nvec) st_stream(reinterpret_cast<uint32_t*>(it.dst) + idx, c);
      } else {
        const uint2 c = encode8_16<IMPL, SRCK>(v[u], scale, ctx, idx * VE);
        if (full) st_stream(reinterpret_cast<uint2*>(it.dst) + idx, c);
        else if (idx < nvec) st_stream(reinterpret_cast<uint2*>(it.dst) + idx, c);
      }
    }
    if (local + 1 == stage_item_wgs<SRCK>(it.n, kStageVec)) {  // ragged tail of the tensor
      const uint64_t t = nvec * VE + threadIdx.x;
      if (t < it.n)
        it.dst[t] = (uint8_t)encode_one<IMPL, SRCK>(scaled_bits(load_bits<SRCK>(it.src, t), scale), keyed<IMPL>(ctx, t), t);
    }
  } else {
    uint32_t m = 0, mt = 0;  // vector part (packed form of vec_amax) and ragged-tail part of the current tensor
    int cur = -1;
    for (uint32_t c = w; c < sg.am_chunks; c += sg.am_wgs) {
      const int j = stage_find(sg.am, sg.n_am, c);
      if (j != cur) {
        if (cur >= 0) {
          block_max_to_global(umax(fold_amax<SRCK>(m), mt), amax + sg.am[cur].index);
          __syncthreads();
        }
        cur = j;
        m = 0;
        mt = 0;
      }
      const StageItem it = sg.am[j];
      const uint64_t nvec = it.n >> vec_shift<SRCK>();
      const uint32_t local = c - it.wg_first;
      const uint64_t v0 = (uint64_t)local * kStageVecAmax + threadIdx.x;
      const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(it.src);
      if (nvec != 0) {
        // unconditional loads (so that all are in flight together): an index past the end reads the last
        // vector again, which leaves the maximum as it is.  Ordinary loads: the cast of the next stage
        // re-reads the data from the last-level cache.
        uint4 v[kStageUAmax];
#pragma unroll
        for (int u = 0; u < kStageUAmax; ++u) {
          const uint64_t idx = v0 + (uint64_t)u * kStageBlock;
          v[u] = src4[idx < nvec ? idx : nvec - 1];
        }
#pragma unroll
        for (int u = 0; u < kStageUAmax; ++u) m = vec_amax<SRCK>(m, v[u]);
      }
      if (local + 1 == stage_item_wgs<SRCK>(it.n, kStageVecAmax)) {
        const uint64_t t = nvec * VE + threadIdx.x;
        if (t < it.n) mt = umax(mt, load_bits<SRCK>(it.src, t) & 0x7FFFFFFFu);
      }
    }
    if (cur >= 0) block_max_to_global(umax(fold_amax<SRCK>(m), mt), amax + sg.am[cur].index);
  }
}

// ====================================================================================
// host side
// ====================================================================================
// global table a kernel of implementation IMPL stages from
template <int IMPL>
inline const uint8_t* enc_table_for(const DevTables& tb) { return IMPL == IMPL_HR16 ? tb.hr16_lut : tb.enc_lut; }

template <int SRCK>
inline int impl_for(uint32_t mode) {
  switch (mode & HIF8_RM_MASK) {
    case HIF8_RM_HR: return SRCK != kSrcF32 ? IMPL_HR16 : IMPL_HR;
    case HIF8_RM_SSR: return IMPL_HR;
    case HIF8_RM_TE: return IMPL_TE;
    case HIF8_RM_SR: return IMPL_SR;
    default: return tune_ta_impl() ? IMPL_TA_ALU : IMPL_TA_LUT;
  }
}

// Calls f(integral_constant IMPL, integral_constant U).  The comparison modes TE and SR are
// built for one unroll factor only.
template <int SRCK, typename F>
inline void dispatch_impl(int impl, int unroll, F&& f) {
  using std::integral_constant;
  switch (impl) {
    case IMPL_HR16:
      if constexpr (SRCK != kSrcF32) dispatch_unroll(unroll, [&](auto u) { f(integral_constant<int, IMPL_HR16>{}, u); });
      break;
    case IMPL_TA_ALU: dispatch_unroll(unroll, [&](auto u) { f(integral_constant<int, IMPL_TA_ALU>{}, u); }); break;
    case IMPL_HR: dispatch_unroll(unroll, [&](auto u) { f(integral_constant<int, IMPL_HR>{}, u); }); break;
    case IMPL_TE: f(integral_constant<int, IMPL_TE>{}, integral_constant<int, 2>{}); break;
    case IMPL_SR: f(integral_constant<int, IMPL_SR>{}, integral_constant<int, 2>{}); break;
    default: dispatch_unroll(unroll, [&](auto u) { f(integral_constant<int, IMPL_TA_LUT>{}, u); }); break;
  }
}

// The fast (16-byte vector) form of the cast; the caller has validated the arguments and the alignment.
template <int SRCK>
void launch_encode_fast(const void* src, uint8_t* dst, size_t n, const ScaleArg& sa, uint32_t* amax_acc, uint32_t mode,
                        const SrArg& sr, int cus, const DevTables& tb, hipStream_t st) {
  const size_t nvec = n >> vec_shift<SRCK>();
  const int impl = impl_for<SRCK>(mode);
  // TE and standard SR stage larger tables and are built for one unroll factor: they keep the 512-lane shape
  const bool one_unroll = impl == IMPL_TE || impl == IMPL_SR;
  Shape shape = shape_for((SRCK != kSrcF32 || one_unroll) ? FAM_ENC16 : (impl == IMPL_HR ? FAM_ENC32_HR : FAM_ENC32_TA));
  if (one_unroll) shape.unroll = 2;
  Walk walk;
  const dim3 grid(grid_for(nvec, cus, shape, &walk)), block(shape.block);
  dispatch_impl<SRCK>(impl, shape.unroll, [&](auto impl_c, auto u_c) {
    constexpr int U = decltype(u_c)::value, IMPL = decltype(impl_c)::value;
    if (sa.parts)
      hipLaunchKernelGGL((k_encode<U, IMPL, SRCK, true>), grid, block, 0, st, src, dst, n, sa, amax_acc, mode, sr,
                         enc_table_for<IMPL>(tb), walk);
    else
      hipLaunchKernelGGL((k_encode<U, IMPL, SRCK, false>), grid, block, 0, st, src, dst, n, sa, amax_acc, mode, sr,
                         enc_table_for<IMPL>(tb), walk);
  });
}

template <int SRCK>
void launch_fake_quant_fast(const void* src, void* dst, uint8_t* codes, size_t n, const ScaleArg& sa, uint32_t* amax_acc,
                            uint32_t mode, const SrArg& sr, int cus, const DevTables& tb, hipStream_t st) {
  const size_t nvec = n >> vec_shift<SRCK>();
  const int impl = impl_for<SRCK>(mode);
  Shape shape = shape_for(FAM_FQ);
  if (impl == IMPL_TE || impl == IMPL_SR) shape.unroll = 2;
  Walk walk;
  const dim3 grid(grid_for(nvec, cus, shape, &walk)), block(shape.block);
  dispatch_impl<SRCK>(impl, shape.unroll, [&](auto impl_c, auto u_c) {
    constexpr int U = decltype(u_c)::value, IMPL = decltype(impl_c)::value;
    auto go = [&](auto codes_c, auto parts_c) {
      hipLaunchKernelGGL((k_fake_quant<U, IMPL, decltype(codes_c)::value, SRCK, decltype(parts_c)::value>), grid, block, 0, st,
                         src, dst, codes, n, sa, amax_acc, mode, sr, enc_table_for<IMPL>(tb), tb.dec_lut, walk);
    };
    using std::true_type;
    using std::false_type;
    if (codes) { if (sa.parts) go(true_type{}, true_type{}); else go(true_type{}, false_type{}); }
    else { if (sa.parts) go(false_type{}, true_type{}); else go(false_type{}, false_type{}); }
  });
}

template <int SRCK>
inline bool encode_fast_ok(const void* src, const uint8_t* dst) {
  return aligned_to(src, 16) && aligned_to(dst, SRCK == kSrcF32 ? 4 : 8);
}
template <int SRCK>
inline bool fake_quant_fast_ok(const void* src, const void* dst, const uint8_t* codes) {
  return aligned_to(src, 16) && aligned_to(dst, 16) && (!codes || aligned_to(codes, SRCK == kSrcF32 ? 4 : 8));
}

template <int SRCK>
hif8_status conv_encode(const void* src, uint8_t* dst, size_t n, float scale, const float* d_scale2,
                        float* d_amax_acc, uint32_t mode, const SrArg* sr_or_null, hipStream_t st) {
  uint32_t* amax_acc = reinterpret_cast<uint32_t*>(d_amax_acc);
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  float inv = 1.0f;
  if (!d_scale2 && !valid_scale(scale, &inv)) return HIF8_ERR_SCALE;
  if (n == 0) return HIF8_OK;
  if (!src || !dst) return HIF8_ERR_NULL;
  int cus = 0;
  DevTables tb;
  hif8_status s = ensure_init(&cus, &tb);
  if (s != HIF8_OK) return s;
  const SrArg sr = sr_or_null ? *sr_or_null : SrArg{sr_seed(), 0};
  if (!encode_fast_ok<SRCK>(src, dst)) {
    hipLaunchKernelGGL(k_encode_elem<SRCK>, dim3(grid_elem(n, cus)), dim3(256), 0, st, src, dst, n,
                       scale, d_scale2, amax_acc, mode, sr);
    return finish_launch();
  }
  launch_encode_fast<SRCK>(src, dst, n, d_scale2 ? scale_on_device(d_scale2) : scale_by_value(scale, inv), amax_acc, mode,
                           sr, cus, tb, st);
  return finish_launch();
}

template <int DSTK>
hif8_status conv_decode(const uint8_t* src, void* dst, size_t n, float scale, const float* d_scale2,
                        hipStream_t st) {
  float inv = 1.0f;
  if (!d_scale2 && !valid_scale(scale, &inv)) return HIF8_ERR_SCALE;
  if (n == 0) return HIF8_OK;
  if (!src || !dst) return HIF8_ERR_NULL;
  int cus = 0;
  DevTables tb;
  hif8_status s = ensure_init(&cus, &tb);
  if (s != HIF8_OK) return s;
  const bool fast = aligned_to(src, DSTK == kSrcF32 ? 4 : 8) && aligned_to(dst, 16);
  if (!fast) {
    hipLaunchKernelGGL(k_decode_elem<DSTK>, dim3(grid_elem(n, cus)), dim3(256), 0, st, src, dst, n,
                       inv, d_scale2);
    return finish_launch();
  }
  const size_t nvec = n >> vec_shift<DSTK>();
  const Shape shape = shape_for(FAM_DEC);
  Walk walk;
  const dim3 grid(grid_for(nvec, cus, shape, &walk)), block(shape.block);
  dispatch_unroll(shape.unroll, [&](auto u_c) {
    hipLaunchKernelGGL((k_decode<decltype(u_c)::value, DSTK>), grid, block, 0, st, src, dst, n, inv, d_scale2,
                       tb.dec_lut, walk);
  });
  return finish_launch();
}

template <int SRCK>
hif8_status conv_fake_quant(const void* src, void* dst, uint8_t* codes, size_t n, float scale,
                            const float* d_scale2, float* d_amax_acc, uint32_t mode, const SrArg* sr_or_null,
                            hipStream_t st) {
  uint32_t* amax_acc = reinterpret_cast<uint32_t*>(d_amax_acc);
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  float inv = 1.0f;
  if (!d_scale2 && !valid_scale(scale, &inv)) return HIF8_ERR_SCALE;
  if (n == 0) return HIF8_OK;
  if (!src || !dst) return HIF8_ERR_NULL;
  int cus = 0;
  DevTables tb;
  hif8_status s = ensure_init(&cus, &tb);
  if (s != HIF8_OK) return s;
  const SrArg sr = sr_or_null ? *sr_or_null : SrArg{sr_seed(), 0};
  if (!fake_quant_fast_ok<SRCK>(src, dst, codes)) {
    hipLaunchKernelGGL(k_fake_quant_elem<SRCK>, dim3(grid_elem(n, cus)), dim3(256), 0, st, src, dst,
                       codes, n, scale, inv, d_scale2, amax_acc, mode, sr);
    return finish_launch();
  }
  launch_fake_quant_fast<SRCK>(src, dst, codes, n, d_scale2 ? scale_on_device(d_scale2) : scale_by_value(scale, inv),
                               amax_acc, mode, sr, cus, tb, st);
  return finish_launch();
}

// amax over the fast path: PARTS = false accumulates into *out (cleared by the caller), PARTS = true writes
// one partial maximum per workgroup to out[0 .. return value) (at most kMaxParts).
// cached: ordinary loads, which leave the tensor in the last-level cache for a pass that follows.
template <int SRCK, bool PARTS>
uint32_t launch_amax_fast(const void* src, size_t n, uint32_t* out, bool cached, int cus, hipStream_t st) {
  const size_t nvec = n >> vec_shift<SRCK>();
  const Shape shape = shape_for(PARTS ? FAM_AMAX_PARTS : FAM_AMAX);
  Walk walk;
  const unsigned g = grid_for(nvec, cus, shape, &walk, PARTS ? kMaxParts : 0u);
  const dim3 grid(g), block(shape.block);
  dispatch_unroll(shape.unroll, [&](auto u_c) {
    constexpr int U = decltype(u_c)::value;
    if (cached) hipLaunchKernelGGL((k_amax<U, SRCK, false, PARTS>), grid, block, 0, st, src, n, out, walk);
    else hipLaunchKernelGGL((k_amax<U, SRCK, true, PARTS>), grid, block, 0, st, src, n, out, walk);
  });
  return g;
}

template <int SRCK>
hif8_status conv_amax(const void* src, size_t n, float* d_amax, hipStream_t st) {
  if (!d_amax || (!src && n != 0)) return HIF8_ERR_NULL;
  int cus = 0;
  hif8_status s = ensure_init(&cus, nullptr);
  if (s != HIF8_OK) return s;
  uint32_t* out = reinterpret_cast<uint32_t*>(d_amax);
  s = launch_fill_u32(out, 0u, 1u, st);
  if (s != HIF8_OK) return s;
  if (n == 0) return HIF8_OK;
  if (!aligned_to(src, 16)) {
    hipLaunchKernelGGL(k_amax_elem<SRCK>, dim3(grid_elem(n, cus)), dim3(256), 0, st, src, n, out);
    return finish_launch();
  }
  // amax is normally followed by a cast of the same tensor: ordinary (cached) loads leave a tensor
  // that fits the 256 MB last-level cache there for the second pass; larger ones are streamed
  const size_t bytes = n * (SRCK == kSrcF32 ? 4 : 2);
  const int nt_knob = tune_amax_nt();
  const bool nt = nt_knob < 0 ? bytes > ((size_t)192 << 20) : nt_knob != 0;
  launch_amax_fast<SRCK, false>(src, n, out, !nt, cus, st);
  return finish_launch();
}

// Per-tensor scaling in one call (Sec. 5: amax, scale factor, cast): pass 1 leaves one partial maximum per
// workgroup in `parts` (ordinary loads, so a tensor that fits the last-level cache stays there), pass 2 is the
// cast -- codes only when dst is null, else the fused round trip with optional codes -- whose workgroups reduce
// the partial maxima and derive the scale themselves.  Two launches; no clearing launch, no atomics, no
// separate scale launch.  Inputs that miss the fast path's alignment take the separate calls.
template <int SRCK>
hif8_status conv_quantize_tensor(const void* src, void* dst, uint8_t* codes, size_t n, float target, int pow2,
                                 uint32_t mode, float* d_amax, float* d_scale2, uint32_t* parts, const SrArg* sr_or_null,
                                 hipStream_t st) {
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  if (!(target > 0.0f) || std::isinf(target)) return HIF8_ERR_ARG;
  if (!d_amax || !d_scale2 || !parts) return HIF8_ERR_NULL;
  if (n != 0 && (!src || (!dst && !codes))) return HIF8_ERR_NULL;
  int cus = 0;
  DevTables tb;
  hif8_status s = ensure_init(&cus, &tb);
  if (s != HIF8_OK) return s;
  const bool fast = n != 0 && (dst ? fake_quant_fast_ok<SRCK>(src, dst, codes) : encode_fast_ok<SRCK>(src, codes));
  if (!fast) {
    s = conv_amax<SRCK>(src, n, d_amax, st);
    if (s != HIF8_OK) return s;
    s = launch_scale_from_amax(d_amax, d_scale2, 1u, target, pow2, st);
    if (s != HIF8_OK || n == 0) return s;
    return dst ? conv_fake_quant<SRCK>(src, dst, codes, n, 1.0f, d_scale2, nullptr, mode, sr_or_null, st)
               : conv_encode<SRCK>(src, codes, n, 1.0f, d_scale2, nullptr, mode, sr_or_null, st);
  }
  const SrArg sr = sr_or_null ? *sr_or_null : SrArg{sr_seed(), 0};
  const uint32_t nparts = launch_amax_fast<SRCK, true>(src, n, parts, true, cus, st);
  const ScaleArg sa{1.0f, 1.0f, nullptr, parts, nparts, target, pow2, d_amax, d_scale2};
  if (dst) launch_fake_quant_fast<SRCK>(src, dst, codes, n, sa, nullptr, mode, sr, cus, tb, st);
  else launch_encode_fast<SRCK>(src, codes, n, sa, nullptr, mode, sr, cus, tb, st);
  return finish_launch();
}

// Calls go(integral_constant IMPL) for the implementation a multi-tensor cast under `mode` uses.
template <int SRCK, typename F>
inline void dispatch_multi_impl(uint32_t mode, F&& go) {
  using std::integral_constant;
  switch (impl_for<SRCK>(mode)) {
    case IMPL_HR16:
      if constexpr (SRCK != kSrcF32) go(integral_constant<int, IMPL_HR16>{});
      break;
    case IMPL_HR: go(integral_constant<int, IMPL_HR>{}); break;
    case IMPL_TE: go(integral_constant<int, IMPL_TE>{}); break;
    case IMPL_SR: go(integral_constant<int, IMPL_SR>{}); break;
    default: go(integral_constant<int, IMPL_TA_LUT>{}); break;
  }
}

template <int SRCK, bool ACC>
void launch_multi_encode(const hif8_cast_item* d_items, uint32_t cnt, uint64_t total_tiles, const float* d_scale2,
                         uint32_t* amax_acc, uint32_t mode, uint64_t seed, const DevTables& tb, hipStream_t st) {
  const dim3 blk(kMultiBlock);
  dispatch_multi_impl<SRCK>(mode, [&](auto impl_c) {
    constexpr int IMPL = decltype(impl_c)::value;
    constexpr uint32_t tpw = multi_tpw_encode<IMPL, ACC>();
    const dim3 g2((unsigned)((total_tiles + tpw - 1) / tpw));
    hipLaunchKernelGGL((k_multi_encode<IMPL, SRCK, ACC>), g2, blk, 0, st, d_items, cnt, total_tiles, d_scale2, amax_acc, mode,
                       seed, enc_table_for<IMPL>(tb));
  });
}

// Multi-tensor cast with the scales already on the device (delayed scaling): one launch.
template <int SRCK>
hif8_status conv_multi_encode_ds(const hif8_cast_item* d_items, size_t count, uint64_t total_tiles,
                                 const float* d_scale2, float* d_amax_acc, uint32_t mode, hipStream_t st) {
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  if (count == 0) return HIF8_OK;
  if (!d_items || !d_scale2) return HIF8_ERR_NULL;
  if (count > 0xFFFFFFu) return HIF8_ERR_ARG;
  DevTables tb;
  hif8_status s = ensure_init(nullptr, &tb);
  if (s != HIF8_OK) return s;
  if (total_tiles == 0) return HIF8_OK;
  uint32_t* acc = reinterpret_cast<uint32_t*>(d_amax_acc);
  if (acc) launch_multi_encode<SRCK, true>(d_items, (uint32_t)count, total_tiles, d_scale2, acc, mode, sr_seed(), tb, st);
  else launch_multi_encode<SRCK, false>(d_items, (uint32_t)count, total_tiles, d_scale2, nullptr, mode, sr_seed(), tb, st);
  return finish_launch();
}

// Multi-tensor cast with fresh per-tensor scales.  With the planned items also at hand on the host the list is cut
// into groups of whole tensors of at most `group_bytes` of source each (a larger tensor is a group of its own), and
// the stages [amax of group g+1 | cast of group g] are enqueued back to back, one launch each: the cast of a group
// then finds its source in the 256 MB last-level cache instead of reading it from HBM a second time.  Without the
// host copy: amax of every tensor, then the scales, then the cast of every tensor (four launches).
template <int SRCK>
hif8_status conv_multi_cast(const hif8_cast_item* host_items_or_null, const hif8_cast_item* d_items, size_t count,
                            uint64_t total_tiles, float* d_amax, float* d_scale2, float target, int pow2, uint32_t mode,
                            hipStream_t st) {
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  if (!(target > 0.0f) || std::isinf(target)) return HIF8_ERR_ARG;
  if (count == 0) return HIF8_OK;
  if (!d_items || !d_amax || !d_scale2) return HIF8_ERR_NULL;
  if (count > 0xFFFFFFu) return HIF8_ERR_ARG;
  if (host_items_or_null) {  // the host copy must be the planned array: tile counts consistent with total_tiles
    uint64_t tiles = 0;
    for (size_t i = 0; i < count; ++i) {
      if (host_items_or_null[i].first_tile != tiles) return HIF8_ERR_ARG;
      tiles += plan_item_tiles(host_items_or_null[i].n, SRCK != kSrcF32);
    }
    if (tiles != total_tiles) return HIF8_ERR_ARG;
  }
  DevTables tb;
  int cus = 0;
  hif8_status s = ensure_init(&cus, &tb);
  if (s != HIF8_OK) return s;
  const uint64_t seed = sr_seed();
  const uint32_t cnt = (uint32_t)count;
  uint32_t* am = reinterpret_cast<uint32_t*>(d_amax);
  s = launch_fill_u32(am, 0u, cnt, st);
  if (s != HIF8_OK) return s;
  if (!host_items_or_null) {
    if (total_tiles != 0) {
      const unsigned g1 = (unsigned)((total_tiles + kMultiTpwAmax - 1) / kMultiTpwAmax);
      hipLaunchKernelGGL(k_multi_amax<SRCK>, dim3(g1), dim3(kMultiBlock), 0, st, d_items, cnt, total_tiles, am);
    }
    s = launch_scale_from_amax(d_amax, d_scale2, cnt, target, pow2, st);
    if (s != HIF8_OK) return s;
    if (total_tiles != 0) launch_multi_encode<SRCK, false>(d_items, cnt, total_tiles, d_scale2, nullptr, mode, seed, tb, st);
    return finish_launch();
  }
  // tensors without elements own no tile, hence no workgroup that would write their pair: with every amax
  // still zero, one small launch sets every pair to {1, 1}; the stages overwrite those of the other tensors
  bool any_empty = false;
  for (size_t k = 0; k < count; ++k) any_empty = any_empty || host_items_or_null[k].n == 0;
  if (any_empty) {
    s = launch_scale_from_amax(d_amax, d_scale2, cnt, target, pow2, st);
    if (s != HIF8_OK) return s;
  }
  // group-wise stages: stage k gathers the amax of group k and casts group k - 1.  A group is a run of whole
  // tensors (empty ones skipped): at least one, more while they fit group_bytes and kStageItems.
  const uint64_t group_bytes = multi_group_bytes();
  const uint64_t esize = SRCK == kSrcF32 ? 4 : 2;
  StageArgs sg;
  std::memset(&sg, 0, sizeof(sg));
  const bool overlap = multi_stage_overlap();
  const uint32_t am_cap = (uint32_t)cus * (uint32_t)shape_for(FAM_MULTI_STAGE).wg_per_cu;
  size_t i = 0;
  for (;;) {
    // the group gathered by the previous stage is cast by this one
    sg.n_enc = sg.n_am;
    sg.enc_wgs = 0;
    for (uint32_t k = 0; k < sg.n_enc; ++k) {
      sg.enc[k] = sg.am[k];
      sg.enc[k].wg_first = sg.enc_wgs;
      sg.enc_wgs += stage_item_wgs<SRCK>(sg.enc[k].n, kStageVec);
    }
    sg.n_am = 0;
    sg.am_chunks = 0;
    uint64_t bytes = 0;
    while (i < count && sg.n_am < (uint32_t)kStageItems) {
      const hif8_cast_item& h = host_items_or_null[i];
      if (h.n == 0) { ++i; continue; }
      if (sg.n_am != 0 && bytes + h.n * esize > group_bytes) break;
      const uint32_t chunks = stage_item_wgs<SRCK>(h.n, kStageVecAmax);
      if (stage_item_wgs<SRCK>(h.n, kStageVec) > 0x3FFFFFFFu) return HIF8_ERR_ARG;
      if (sg.n_am != 0 && (uint64_t)sg.am_chunks + chunks > 0x3FFFFFFFu) break;
      sg.am[sg.n_am] = StageItem{h.src, h.dst, h.n, sg.am_chunks, (uint32_t)i};
      sg.am_chunks += chunks;
      sg.n_am += 1;
      bytes += h.n * esize;
      ++i;
    }
    sg.am_wgs = sg.am_chunks < am_cap ? sg.am_chunks : am_cap;
    if (sg.n_enc == 0 && sg.n_am == 0) break;  // nothing left to gather, nothing left to cast
    if ((uint64_t)sg.enc_wgs + sg.am_wgs > 0x7FFFFFFFull) return HIF8_ERR_ARG;
    auto launch = [&](const StageArgs& a) {
      if (a.enc_wgs + a.am_wgs == 0) return;
      dispatch_multi_impl<SRCK>(mode, [&](auto impl_c) {
        constexpr int IMPL = decltype(impl_c)::value;
        hipLaunchKernelGGL((k_group_stage<IMPL, SRCK>), dim3(a.enc_wgs + a.am_wgs), dim3(kStageBlock), 0, st, a, am,
                           d_scale2, target, pow2, mode, seed, enc_table_for<IMPL>(tb));
      });
    };
    if (!overlap) {  // the cast of a group, then the amax of the next, as two launches
      StageArgs a = sg;
      a.n_am = 0; a.am_wgs = 0; a.am_chunks = 0;
      launch(a);
      a = sg;
      a.n_enc = 0; a.enc_wgs = 0;
      launch(a);
    } else {
      launch(sg);
    }
  }
  return finish_launch();
}

}  // namespace hif8conv

// explicit instantiation of every host entry point for one kind
#define HIF8_INSTANTIATE_CONV(K)                                                                         \
  namespace hif8conv {                                                                                   \
  template hif8_status conv_encode<K>(const void*, uint8_t*, size_t, float, const float*, float*,        \
                                      uint32_t, const SrArg*, hipStream_t);                              \
  template hif8_status conv_decode<K>(const uint8_t*, void*, size_t, float, const float*, hipStream_t);  \
  template hif8_status conv_fake_quant<K>(const void*, void*, uint8_t*, size_t, float, const float*,     \
                                          float*, uint32_t, const SrArg*, hipStream_t);                  \
  template hif8_status conv_amax<K>(const void*, size_t, float*, hipStream_t);                           \
  template hif8_status conv_quantize_tensor<K>(const void*, void*, uint8_t*, size_t, float, int, uint32_t, \
                                               float*, float*, uint32_t*, const SrArg*, hipStream_t);    \
  template hif8_status conv_multi_cast<K>(const hif8_cast_item*, const hif8_cast_item*, size_t, uint64_t, \
                                          float*, float*, float, int, uint32_t, hipStream_t);            \
  template hif8_status conv_multi_encode_ds<K>(const hif8_cast_item*, size_t, uint64_t, const float*,    \
                                               float*, uint32_t, hipStream_t);                           \
  }
