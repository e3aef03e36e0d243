/*
 * HiF8 CPU oracle -- TEST INFRASTRUCTURE, NOT PRODUCT CODE.
 *
 * A plain, slow, obviously-correct implementation of the HiFloat8 conversion
 * path of "Ascend HiFloat8 Format for Deep Learning" (arXiv 2409.16626),
 * written from the paper only.  It shares no code, tables or helpers with the
 * HIP library and must only be used by tests, the smoke check and the CPU
 * baseline leg of the benchmark.
 *
 *   decode : the definition written out -- Table 1 (fields), Table 2 (dot
 *            prefix code), Table 3 (Em / Ei / E / mantissa width), Eq. (1)
 *            normal numbers, Eq. (2) denormal numbers, and the special
 *            patterns of Sec. 2.1 / Table 4.
 *   encode : nearest representable value found by brute-force search over
 *            every finite HiF8 magnitude, in fp64, with the tie / stochastic
 *            rules of Sec. 3.1 (rounding half away from zero, "TA") and
 *            Sec. 3.2 (simplified stochastic rounding SR14 / SR2 and hybrid
 *            rounding, Eq. (3)).
 *
 * Readings taken where the paper is silent or ambiguous:
 *   - Em bit order: Se is the first (most significant) bit, magnitude bits
 *     follow (the only order that reproduces the Table 4 patterns).
 *   - Rounding in the denormal range, at the underflow edge and at the
 *     overflow edge is the same "nearest in linear value, ties away from zero"
 *     as everywhere else: the neighbour below the smallest denormal is 0 and
 *     the neighbour above the largest normal is the value 1.5*2^15 that the
 *     Infinity patterns would have under Eq. (1); landing there is overflow.
 *   - Overflow and +-Inf inputs give the Infinity pattern, or with the
 *     saturation option the largest finite value 2^15 (PARITY UNPINNED for
 *     the +-Inf input case: the paper names the option but not this case).
 *   - NaN gives the NaN pattern, or with the NaN-to-zero option the zero
 *     pattern.  Results of magnitude zero are the single zero pattern 0x00
 *     whatever the sign (Sec. 2.1: one zero pattern only).
 *   - SR carry rule is F >= T (Sec. 3.2) except that F = 0 with T = 0 does
 *     not carry, so exactly representable inputs stay put (PARITY UNPINNED:
 *     deliberate deviation from the literal text on a measure-zero set).
 *   - SR14: T = the 14 LSBs of the FP32 pattern being converted, F = the top
 *     14 bits of the discarded fraction; SR2: T = 2*LSB_of_BF16 + 1 (the only
 *     order that yields the stated thresholds 0.25 and 0.75), F = the top 2
 *     bits of the discarded fraction.  The figure that draws the bit
 *     positions is missing from the paper text available to this build, so
 *     the positions follow the prose (PARITY UNPINNED beyond the prose).
 *   - Below the smallest denormal SR works on the fixed-point fraction of one
 *     step 2^-22 (lo = 0, hi = 2^-22)  (PARITY UNPINNED).
 *   - E in Eq. (3) is the binary exponent of the value being rounded, i.e.
 *     after the high-precision scale multiply and before rounding.
 *   - The scale multiply is one IEEE binary32 round-to-nearest-even multiply;
 *     the inverse scale used by decode / fake-quant is fl32(1/scale).
 *   - amax is the maximum of the magnitude bit patterns compared as unsigned
 *     integers (so Inf dominates finite values and any NaN dominates Inf).
 *   - scale from amax: fl32(target / amax); with pow2 the largest power of
 *     two not above it; amax zero, Inf or NaN gives scale 1.
 *   - Comparison modes (not adopted by the format; kept so that the paper's TA/TE/SR/HR
 *     comparisons can be repeated):
 *     TE  "even" means the neighbour that is an even multiple of the local step
 *         hi - lo (IEEE-style).  In the denormal range the steps are powers of
 *         two, so lo = 1 * step is odd and a tie goes up; at the underflow edge
 *         lo = 0 is even and the tie 2^-23 goes to zero; at the overflow edge
 *         lo = 2^15 = 2 * step is even and the tie 1.25 * 2^15 stays finite.
 *         (PARITY UNPINNED outside the normal bands.)
 *     SSR the simplified SR rule of HR applied in every binade, also |E| < 4.
 *     SR  carry iff T < F with T = t32 / 2^32, t32 a 32-bit threshold drawn per
 *         element from a counter-based generator (below); strict "<" makes the
 *         carry probability exactly F for a discrete uniform T and keeps
 *         representable inputs fixed (the paper writes F >= T for a real-valued T).
 *         Sec. 3.2 asks for one uniform random number per element and names no source,
 *         so the generator is this build's choice.  Threshold of element i under the
 *         64-bit seed s: a key pair (k1, k2) = the two halves of the splitmix64 finaliser
 *         of s + 0x9E3779B97F4A7C15 * (hi32(i) + 1), i.e. a non-linear function of the whole
 *         seed that is constant over 2^32 consecutive elements; then the 32-bit finaliser
 *         of MurmurHash3 over lo32(i) ^ k1 with k2 added between its two multiplications.
 *         Two seeds give two different functions of the index (not one sequence in another
 *         order), which the pins check.
 *   - FP16 sources use SR2 with the FP16 LSB (bit 13 of the binary32 pattern
 *     being converted, so that, as for BF16, a scaled product is handled too).
 *
 * Arithmetic is fp64 throughout except where the method itself fixes binary32
 * (the scale multiply and the descale multiply).  Every fp64 quantity used in
 * a comparison is exact: inputs are binary32, HiF8 values have at most 4
 * significant bits.
 *
 * Build: gcc -O2 -fopenmp -ffp-contract=off -shared -fPIC hif8_oracle.c -lm
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

/* rounding_mode bit-field understood by the oracle (same numeric values as the
 * public header of the HIP library, typed in again here on purpose). */
#define ORM_TA 0u
#define ORM_HR 1u
#define ORM_TE 2u  /* rounding half to even: described in Sec. 3.1, not adopted by the format */
#define ORM_SSR 3u /* simplified SR (SR14 / SR2) in every binade, Sec. 3.2                   */
#define ORM_SR 4u  /* standard SR, Sec. 3.2, threshold from a counter-based generator        */
#define ORM_MASK 0xFu

/* source kinds: which simplified SR applies (Sec. 3.2: SR14 for FP32, SR2 for FP16 and BF16)
 * and where the source format's LSB sits in the binary32 pattern being converted */
#define OSRC_F32 0
#define OSRC_BF16 1 /* LSB = bit 16 */
#define OSRC_F16 2  /* LSB = bit 13 */
#define OFLAG_SAT 0x10u
#define OFLAG_NAN2ZERO 0x20u

/* debug switch: literal "F >= T" even when F = T = 0 (see header). */
static int g_literal_sr_zero = 0;
void hif8o_set_literal_sr_zero(int on) { g_literal_sr_zero = on; }

/* ------------------------------------------------------------------------
 * Decode: Sec. 2.1, Tables 1-3, Eq. (1), Eq. (2), special values.
 * Returns the real value of a code as fp64 (exact); NaN and +-Inf as such.
 * Optional outputs describe the parse (for the tests that count fields).
 *   kind: 0 zero, 1 NaN, 2 Inf, 3 denormal, 4 normal
 * ---------------------------------------------------------------------- */
double hif8o_decode_fields(uint8_t code, int *kind, int *D_out, int *E_out,
                           int *mant_width, int *mant) {
  int bits[8]; /* bits[0] is the MSB (sign) ... bits[7] the LSB */
  for (int i = 0; i < 8; ++i) bits[i] = (code >> (7 - i)) & 1;
  int pos = 0;
  int S = bits[pos++]; /* sign field: 1 bit, 1 = negative */

  /* dot field: prefix code of Table 2 */
  int D = -1; /* -1 = DML */
  if (bits[pos] == 1 && bits[pos + 1] == 1) { D = 4; pos += 2; }
  else if (bits[pos] == 1 && bits[pos + 1] == 0) { D = 3; pos += 2; }
  else if (bits[pos] == 0 && bits[pos + 1] == 1) { D = 2; pos += 2; }
  else if (bits[pos + 2] == 1) { D = 1; pos += 3; }          /* 001  */
  else if (bits[pos + 3] == 1) { D = 0; pos += 4; }          /* 0001 */
  else { D = -1; pos += 4; }                                 /* 0000 */

  double sign = S ? -1.0 : 1.0;

  if (D < 0) {
    /* denormal: the 3 remaining bits are a biased exponent, Eq. (2) */
    int M = 0;
    for (; pos < 8; ++pos) M = (M << 1) | bits[pos];
    if (D_out) *D_out = -1;
    if (mant_width) *mant_width = 3;
    if (mant) *mant = M;
    if (M == 0) { /* the two M = 0 patterns: Zero (S=0) and NaN (S=1) */
      if (E_out) *E_out = 0;
      if (S) { if (kind) *kind = 1; return NAN; }
      if (kind) *kind = 0;
      return 0.0;
    }
    if (E_out) *E_out = M - 23;
    if (kind) *kind = 3;
    return sign * ldexp(1.0, M - 23);
  }

  /* exponent field: D bits of Em = {Se, Mag[2:end]}, hidden leading 1 */
  int E = 0;
  if (D > 0) {
    int Se = bits[pos++];
    int mag = 1; /* the unstored MSB of the magnitude */
    for (int i = 1; i < D; ++i) mag = (mag << 1) | bits[pos++];
    E = Se ? -mag : mag;
  }
  /* mantissa field: whatever is left (Table 1: 5-D, 4-D or 3-D bits) */
  int W = 8 - pos;
  int M = 0;
  for (; pos < 8; ++pos) M = (M << 1) | bits[pos];

  if (D_out) *D_out = D;
  if (E_out) *E_out = E;
  if (mant_width) *mant_width = W;
  if (mant) *mant = M;

  double v = ldexp(1.0 + (double)M / (double)(1 << W), E); /* Eq. (1) */
  /* the two patterns of largest magnitude 1.5 * 2^15 are the Infinities */
  if (v == 1.5 * 32768.0) {
    if (kind) *kind = 2;
    return sign * INFINITY;
  }
  if (kind) *kind = 4;
  return sign * v;
}

double hif8o_decode_value(uint8_t code) {
  return hif8o_decode_fields(code, 0, 0, 0, 0, 0);
}

/* ------------------------------------------------------------------------
 * The set of finite non-negative magnitudes, ascending, built by decoding.
 * ---------------------------------------------------------------------- */
static double g_val[128];
static uint8_t g_code[128];
static int g_nval = 0;
static uint8_t g_code_inf = 0; /* positive Infinity pattern  */
static uint8_t g_code_max = 0; /* largest positive finite    */
static const double V_OVERFLOW = 1.5 * 32768.0; /* Eq. (1) value of the Inf slot */

static void build_value_table(void) {
  if (g_nval) return;
  double v[128];
  uint8_t c[128];
  int n = 0;
  uint8_t cinf = 0;
  for (int code = 0; code < 128; ++code) { /* S = 0 half */
    double x = hif8o_decode_value((uint8_t)code);
    if (isnan(x)) continue;
    if (isinf(x)) { cinf = (uint8_t)code; continue; }
    v[n] = x; c[n] = (uint8_t)code; ++n;
  }
  /* insertion sort by value */
  for (int i = 1; i < n; ++i) {
    double xv = v[i]; uint8_t xc = c[i];
    int j = i - 1;
    while (j >= 0 && v[j] > xv) { v[j + 1] = v[j]; c[j + 1] = c[j]; --j; }
    v[j + 1] = xv; c[j + 1] = xc;
  }
  memcpy(g_val, v, sizeof(double) * n);
  memcpy(g_code, c, n);
  g_code_inf = cinf;
  g_code_max = c[n - 1];
#ifdef _OPENMP
#pragma omp flush
#endif
  g_nval = n;
}

int hif8o_value_table(double *vals, uint8_t *codes) {
  build_value_table();
  for (int i = 0; i < g_nval; ++i) { vals[i] = g_val[i]; codes[i] = g_code[i]; }
  return g_nval;
}

static uint32_t f32_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }
static float bits_f32(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }

/* ------------------------------------------------------------------------
 * Encode one binary32 value y (already scaled).  src_bf16 selects which
 * simplified SR the hybrid mode uses (SR2 for 16-bit sources, SR14 for FP32).
 * ---------------------------------------------------------------------- */
/* counter-based threshold generator for standard SR (see header) */
uint32_t hif8o_sr_threshold(uint64_t seed, uint64_t index) {
  /* key pair of the 2^32-element block that holds `index`: splitmix64's output function */
  uint64_t z = seed + 0x9E3779B97F4A7C15ull * ((index >> 32) + 1ull);
  z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
  z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
  z = z ^ (z >> 31);
  const uint32_t k1 = (uint32_t)z, k2 = (uint32_t)(z >> 32);
  /* MurmurHash3's 32-bit finaliser over the low index word, keyed at its input and in its middle */
  uint32_t x = (uint32_t)index ^ k1;
  x ^= x >> 16; x *= 0x85EBCA6Bu; x += k2;
  x ^= x >> 13; x *= 0xC2B2AE35u; x ^= x >> 16;
  return x;
}
static uint64_t g_sr_seed = 0;
void hif8o_set_sr_seed(uint64_t seed) { g_sr_seed = seed; }
/* index of the first element of the arrays passed to the array functions (so that a slice of a
 * large tensor can be checked with the thresholds its elements have inside that tensor) */
static uint64_t g_sr_index_base = 0;
void hif8o_set_sr_index_base(uint64_t base) { g_sr_index_base = base; }

uint8_t hif8o_encode_one_t(float y, uint32_t mode, int src_kind, uint32_t t32);
uint8_t hif8o_encode_one(float y, uint32_t mode, int src_kind) {
  return hif8o_encode_one_t(y, mode, src_kind, 0u);
}

/* t32: the 32-bit threshold of this element (used by ORM_SR only) */
uint8_t hif8o_encode_one_t(float y, uint32_t mode, int src_kind, uint32_t t32) {
  build_value_table();
  const uint32_t rm = mode & ORM_MASK;
  const int sat = (mode & OFLAG_SAT) != 0;
  const int nan2zero = (mode & OFLAG_NAN2ZERO) != 0;

  if (isnan(y)) return nan2zero ? 0x00 : 0x80;

  const uint8_t sign = signbit(y) ? 0x80 : 0x00;
  const uint8_t overflow_code = (uint8_t)((sat ? g_code_max : g_code_inf) | sign);
  if (isinf(y)) return overflow_code;

  const double a = fabs((double)y);
  if (a >= V_OVERFLOW) return overflow_code;
  if (a == 0.0) return 0x00;

  /* bracketing pair lo <= a < hi by linear scan */
  int i = 0;
  while (i + 1 < g_nval && g_val[i + 1] <= a) ++i;
  const double lo = g_val[i];
  const double hi = (i + 1 < g_nval) ? g_val[i + 1] : V_OVERFLOW;

  int up;
  int use_sr = (rm == ORM_SSR);
  if (rm == ORM_HR) {
    int ex;
    (void)frexp(a, &ex);       /* a = f * 2^ex, f in [0.5, 1) */
    const int E = ex - 1;      /* floor(log2 a) */
    use_sr = (E <= -4 || E >= 4); /* Eq. (3) */
  }
  if (rm == ORM_TE) {
    /* Sec. 3.1, TE: nearest, exact half goes to the even multiple of the step */
    const double mid = 0.5 * (lo + hi);
    if (a != mid) up = (a > mid);
    else up = (fmod(lo / (hi - lo), 2.0) != 0.0); /* lo = n * step, n odd -> go up */
  } else if (rm == ORM_SR) {
    /* Sec. 3.2, standard SR: carry iff T < F, T = t32 / 2^32 */
    const double frac = (a - lo) / (hi - lo);
    up = ((double)t32 / 4294967296.0 < frac);
  } else if (!use_sr) {
    /* Sec. 3.1, TA: nearest, exact half goes away from zero */
    const double mid = 0.5 * (lo + hi);
    up = (a >= mid);
  } else {
    /* Sec. 3.2, simplified SR: carry iff F >= T */
    const uint32_t ybits = f32_bits(y);
    const double frac = (a - lo) / (hi - lo); /* in [0, 1), exact */
    uint32_t F, T;
    if (src_kind == OSRC_BF16 || src_kind == OSRC_F16) {
      const int lsb_pos = (src_kind == OSRC_BF16) ? 16 : 13;
      F = (uint32_t)floor(frac * 4.0);
      T = 2u * ((ybits >> lsb_pos) & 1u) + 1u;
    } else {
      F = (uint32_t)floor(frac * 16384.0);
      T = ybits & 0x3FFFu;
    }
    up = (F >= T);
    if (F == 0 && T == 0 && !g_literal_sr_zero) up = 0;
  }

  if (!up) {
    if (lo == 0.0) return 0x00;
    return (uint8_t)(g_code[i] | sign);
  }
  if (i + 1 >= g_nval) return overflow_code; /* rounded up into the Inf slot */
  return (uint8_t)(g_code[i + 1] | sign);
}

/* ------------------------------------------------------------------------
 * Helpers for the 16-bit brain float container.
 * ---------------------------------------------------------------------- */
static float bf16_to_f32(uint16_t h) { return bits_f32((uint32_t)h << 16); }

/* binary32 -> bfloat16, round to nearest even; NaN -> canonical quiet NaN */
static uint16_t f32_to_bf16_rne(float f) {
  if (isnan(f)) return 0x7FC0;
  /* work on the value, not on a bit trick: find the two neighbouring
   * bfloat16 values and pick the nearer, ties to the even pattern */
  uint32_t u = f32_bits(f);
  uint32_t lo = u & 0xFFFF0000u;          /* truncation toward zero */
  if (lo == u) return (uint16_t)(u >> 16);
  uint32_t hi = lo + 0x10000u;            /* next pattern away from zero (may be Inf) */
  double x = fabs((double)f);
  double dlo = fabs((double)bits_f32(lo));
  double dhi_v;
  if (((hi >> 23) & 0xFF) == 0xFF) {
    /* the neighbour above the largest finite bfloat16 acts as 2^128 */
    dhi_v = ldexp(1.0, 128);
  } else {
    dhi_v = fabs((double)bits_f32(hi));
  }
  double d0 = x - dlo, d1 = dhi_v - x;
  if (d0 < d1) return (uint16_t)(lo >> 16);
  if (d1 < d0) return (uint16_t)(hi >> 16);
  return (uint16_t)((((lo >> 16) & 1u) == 0 ? lo : hi) >> 16);
}

/* array form of the narrowing, exported so that it can be pinned on its own */
void hif8o_narrow_bf16(const float *src, uint16_t *dst, size_t n) {
  for (size_t i = 0; i < n; ++i) dst[i] = f32_to_bf16_rne(src[i]);
}

/* descaled binary32 value of a code: fl32(value * inv_scale); specials fixed:
 * NaN -> 0x7FC00000, Inf -> +-0x7F800000, zero -> +0.0 */
static float decode_descaled(uint8_t code, float inv_scale) {
  double v = hif8o_decode_value(code);
  if (isnan(v)) return bits_f32(0x7FC00000u);
  if (isinf(v)) return v > 0 ? bits_f32(0x7F800000u) : bits_f32(0xFF800000u);
  volatile float fv = (float)v; /* exact: at most 4 significant bits */
  volatile float r = fv * inv_scale;
  if (isnan(r)) return bits_f32(0x7FC00000u);
  return r;
}

/* ------------------------------------------------------------------------
 * Helpers for IEEE binary16 (1 sign, 5 exponent, 10 mantissa bits).
 * ---------------------------------------------------------------------- */
static float f16_to_f32(uint16_t h) {
  const int s = h >> 15, e = (h >> 10) & 0x1F, m = h & 0x3FF;
  double v;
  if (e == 0x1F) {
    if (m) return bits_f32(0x7FC00000u | ((uint32_t)s << 31) | ((uint32_t)m << 13));
    v = INFINITY;
  } else if (e == 0) {
    v = ldexp((double)m, -24);                 /* subnormal: m * 2^-24 */
  } else {
    v = ldexp(1.0 + (double)m / 1024.0, e - 15);
  }
  return (float)(s ? -v : v);                  /* every binary16 value is exact in binary32 */
}

/* binary32 -> binary16, round to nearest even; NaN -> 0x7E00 */
static uint16_t f32_to_f16_rne(float f) {
  if (isnan(f)) return 0x7E00;
  const uint16_t s = signbit(f) ? 0x8000 : 0;
  double x = fabs((double)f);
  if (isinf(f)) return (uint16_t)(s | 0x7C00);
  if (x == 0.0) return s;
  int ex;
  (void)frexp(x, &ex);
  int E = ex - 1;                              /* floor(log2 x) */
  if (E < -14) E = -14;                        /* subnormal range shares the quantum 2^-24 */
  const double q = ldexp(1.0, E - 10);         /* spacing of binary16 values near x */
  const double r = rint(x / q) * q;            /* default rounding mode: nearest even; exact in fp64 */
  if (r >= 65536.0) return (uint16_t)(s | 0x7C00); /* rounds past the largest finite 65504 */
  if (r < ldexp(1.0, -14)) return (uint16_t)(s | (uint16_t)(r / ldexp(1.0, -24)));
  (void)frexp(r, &ex);
  const int Er = ex - 1;
  const double frac = r / ldexp(1.0, Er) - 1.0; /* in [0, 1) */
  return (uint16_t)(s | ((Er + 15) << 10) | (uint16_t)(frac * 1024.0));
}

void hif8o_widen_f16(const uint16_t *src, float *dst, size_t n) {
  for (size_t i = 0; i < n; ++i) dst[i] = f16_to_f32(src[i]);
}
void hif8o_narrow_f16(const float *src, uint16_t *dst, size_t n) {
  for (size_t i = 0; i < n; ++i) dst[i] = f32_to_f16_rne(src[i]);
}

/* ------------------------------------------------------------------------
 * Array entry points (what the tests and the CPU baseline call).
 * ---------------------------------------------------------------------- */
static int g_threads_used = 1;
int hif8o_threads_used(void) { return g_threads_used; }

static void note_threads(void) {
#ifdef _OPENMP
  g_threads_used = omp_get_max_threads();
#else
  g_threads_used = 1;
#endif
}

void hif8o_encode_f32(const float *src, uint8_t *dst, size_t n, float scale, uint32_t mode) {
  build_value_table(); note_threads();
#pragma omp parallel for schedule(static)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
    volatile float y = src[i] * scale;
    dst[i] = hif8o_encode_one_t(y, mode, OSRC_F32, hif8o_sr_threshold(g_sr_seed, g_sr_index_base + (uint64_t)i));
  }
}

void hif8o_encode_bf16(const uint16_t *src, uint8_t *dst, size_t n, float scale, uint32_t mode) {
  build_value_table(); note_threads();
#pragma omp parallel for schedule(static)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
    volatile float y = bf16_to_f32(src[i]) * scale;
    dst[i] = hif8o_encode_one_t(y, mode, OSRC_BF16, hif8o_sr_threshold(g_sr_seed, g_sr_index_base + (uint64_t)i));
  }
}

void hif8o_encode_f16(const uint16_t *src, uint8_t *dst, size_t n, float scale, uint32_t mode) {
  build_value_table(); note_threads();
#pragma omp parallel for schedule(static)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
    volatile float y = f16_to_f32(src[i]) * scale;
    dst[i] = hif8o_encode_one_t(y, mode, OSRC_F16, hif8o_sr_threshold(g_sr_seed, g_sr_index_base + (uint64_t)i));
  }
}

void hif8o_decode_f32(const uint8_t *src, float *dst, size_t n, float scale) {
  note_threads();
  volatile float inv = 1.0f / scale;
#pragma omp parallel for schedule(static)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) dst[i] = decode_descaled(src[i], inv);
}

void hif8o_decode_bf16(const uint8_t *src, uint16_t *dst, size_t n, float scale) {
  note_threads();
  volatile float inv = 1.0f / scale;
#pragma omp parallel for schedule(static)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i)
    dst[i] = f32_to_bf16_rne(decode_descaled(src[i], inv));
}

void hif8o_fake_quant_f32(const float *src, float *dst, uint8_t *codes_or_null, size_t n,
                          float scale, uint32_t mode) {
  build_value_table(); note_threads();
  volatile float inv = 1.0f / scale;
#pragma omp parallel for schedule(static)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
    volatile float y = src[i] * scale;
    uint8_t c = hif8o_encode_one_t(y, mode, OSRC_F32, hif8o_sr_threshold(g_sr_seed, g_sr_index_base + (uint64_t)i));
    if (codes_or_null) codes_or_null[i] = c;
    dst[i] = decode_descaled(c, inv);
  }
}

void hif8o_fake_quant_bf16(const uint16_t *src, uint16_t *dst, uint8_t *codes_or_null, size_t n,
                           float scale, uint32_t mode) {
  build_value_table(); note_threads();
  volatile float inv = 1.0f / scale;
#pragma omp parallel for schedule(static)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
    volatile float y = bf16_to_f32(src[i]) * scale;
    uint8_t c = hif8o_encode_one_t(y, mode, OSRC_BF16, hif8o_sr_threshold(g_sr_seed, g_sr_index_base + (uint64_t)i));
    if (codes_or_null) codes_or_null[i] = c;
    dst[i] = f32_to_bf16_rne(decode_descaled(c, inv));
  }
}

void hif8o_fake_quant_f16(const uint16_t *src, uint16_t *dst, uint8_t *codes_or_null, size_t n,
                          float scale, uint32_t mode) {
  build_value_table(); note_threads();
  volatile float inv = 1.0f / scale;
#pragma omp parallel for schedule(static)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
    volatile float y = f16_to_f32(src[i]) * scale;
    uint8_t c = hif8o_encode_one_t(y, mode, OSRC_F16, hif8o_sr_threshold(g_sr_seed, g_sr_index_base + (uint64_t)i));
    if (codes_or_null) codes_or_null[i] = c;
    dst[i] = f32_to_f16_rne(decode_descaled(c, inv));
  }
}

void hif8o_decode_f16(const uint8_t *src, uint16_t *dst, size_t n, float scale) {
  note_threads();
  volatile float inv = 1.0f / scale;
#pragma omp parallel for schedule(static)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i)
    dst[i] = f32_to_f16_rne(decode_descaled(src[i], inv));
}

float hif8o_amax_f16(const uint16_t *src, size_t n) {
  uint32_t m = 0;                     /* magnitude patterns of binary16 order like the values */
#pragma omp parallel for schedule(static) reduction(max : m)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
    uint32_t a = src[i] & 0x7FFFu;
    if (a > m) m = a;
  }
  return f16_to_f32((uint16_t)m);
}

/* amax: maximum magnitude pattern, compared as unsigned integers */
float hif8o_amax_f32(const float *src, size_t n) {
  uint32_t m = 0;
#pragma omp parallel for schedule(static) reduction(max : m)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
    uint32_t a = f32_bits(src[i]) & 0x7FFFFFFFu;
    if (a > m) m = a;
  }
  return bits_f32(m);
}

float hif8o_amax_bf16(const uint16_t *src, size_t n) {
  uint32_t m = 0;
#pragma omp parallel for schedule(static) reduction(max : m)
  for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
    uint32_t a = ((uint32_t)src[i] << 16) & 0x7FFFFFFFu;
    if (a > m) m = a;
  }
  return bits_f32(m);
}

/* per-tensor scale from amax (Sec. 5, per-tensor scaling: power-of-two scale
 * factors; the update rule itself is left open by the paper) */
float hif8o_scale_from_amax(float amax, float target, int pow2) {
  if (isnan(amax) || isinf(amax) || amax <= 0.0f) return 1.0f;
  volatile float s = target / amax;
  if (isnan(s) || isinf(s) || s <= 0.0f) return 1.0f;
  if (pow2) {
    int ex;
    (void)frexp((double)s, &ex); /* s = f * 2^ex, f in [0.5,1) -> floor pow2 = 2^(ex-1) */
    double p = ldexp(1.0, ex - 1);
    volatile float pf = (float)p; /* exact unless s is subnormal-small; then keep s */
    if (pf > 0.0f) return pf;
  }
  return s;
}

/* ------------------------------------------------------------------------
 * Scale sweep (the cast-and-score step of Algorithm 1, applied to one tensor):
 * for each exponent e = e_lo .. e_lo + count - 1 the tensor is scaled by 2^e,
 * cast to HiF8, restored by 2^-e, and the squared error against the original is
 * summed:  err[k] = sum_i ( x_i - value(Q(fl32(x_i * 2^e))) * 2^-e )^2.
 * Sums are fp64 (each term is exact in fp64: the difference of two binary32
 * values that is itself a binary32-sized quantity, squared).  IEEE semantics for
 * non-finite terms: a cast that overflows to Infinity makes the sum +Inf, a NaN
 * element makes it NaN.  Algorithm 1 scores the MSE of the layer output; this is
 * the same score taken on the tensor itself (MSE = err / n).
 * src_kind: OSRC_F32 (x points to float), OSRC_BF16 / OSRC_F16 (uint16_t patterns).
 * ---------------------------------------------------------------------- */
static float load_as_f32(const void *x, size_t i, int src_kind) {
  if (src_kind == OSRC_F32) return ((const float *)x)[i];
  if (src_kind == OSRC_BF16) return bf16_to_f32(((const uint16_t *)x)[i]);
  return f16_to_f32(((const uint16_t *)x)[i]);
}

void hif8o_scale_sweep(const void *x, size_t n, int src_kind, int e_lo, int count,
                       uint32_t mode, double *err_out) {
  build_value_table(); note_threads();
  for (int k = 0; k < count; ++k) {
    const float s = (float)ldexp(1.0, e_lo + k);
    volatile float inv = 1.0f / s;
    double acc = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : acc)
    for (ptrdiff_t i = 0; i < (ptrdiff_t)n; ++i) {
      const float xi = load_as_f32(x, (size_t)i, src_kind);
      volatile float y = xi * s;
      const uint8_t c = hif8o_encode_one_t(y, mode, src_kind, hif8o_sr_threshold(g_sr_seed, g_sr_index_base + (uint64_t)i));
      const double q = (double)decode_descaled(c, inv);
      const double d = (double)xi - q;
      acc += d * d;
    }
    err_out[k] = acc;
  }
}

/* ------------------------------------------------------------------------
 * Per-channel scaling (Sec. 4.2 suggests per-channel scaling for weights as a
 * further method): a row-major [rows, cols] matrix with one amax / scale per
 * row (axis = 0: the channel index is the row) or per column (axis = 1).
 * ---------------------------------------------------------------------- */
void hif8o_amax_axis(const void *x, size_t rows, size_t cols, int src_kind, int axis, float *amax_out) {
  const size_t nch = axis == 0 ? rows : cols;
  for (size_t c = 0; c < nch; ++c) {
    uint32_t m = 0;
    const size_t len = axis == 0 ? cols : rows;
    for (size_t j = 0; j < len; ++j) {
      const size_t idx = axis == 0 ? c * cols + j : j * cols + c;
      uint32_t a = f32_bits(load_as_f32(x, idx, src_kind)) & 0x7FFFFFFFu;
      if (a > m) m = a;
    }
    amax_out[c] = bits_f32(m);
  }
}

/* codes[r, c] = code(Q(fl32(x[r, c] * scale[channel]))); standard-SR thresholds are indexed
 * by the flat element index r * cols + c */
void hif8o_encode_axis(const void *x, uint8_t *dst, size_t rows, size_t cols, int src_kind, int axis,
                       const float *scale, uint32_t mode) {
  build_value_table(); note_threads();
#pragma omp parallel for schedule(static)
  for (ptrdiff_t r = 0; r < (ptrdiff_t)rows; ++r) {
    for (size_t c = 0; c < cols; ++c) {
      const size_t idx = (size_t)r * cols + c;
      volatile float y = load_as_f32(x, idx, src_kind) * scale[axis == 0 ? (size_t)r : c];
      dst[idx] = hif8o_encode_one_t(y, mode, src_kind, hif8o_sr_threshold(g_sr_seed, g_sr_index_base + (uint64_t)idx));
    }
  }
}

/* dst[r, c] = narrow(fl32(value(codes[r, c]) * fl32(1 / scale[channel]))) */
void hif8o_decode_axis(const uint8_t *codes, void *dst, size_t rows, size_t cols, int dst_kind, int axis,
                       const float *scale) {
  for (size_t r = 0; r < rows; ++r) {
    for (size_t c = 0; c < cols; ++c) {
      const size_t idx = r * cols + c;
      volatile float inv = 1.0f / scale[axis == 0 ? r : c];
      const float v = decode_descaled(codes[idx], inv);
      if (dst_kind == OSRC_F32) ((float *)dst)[idx] = v;
      else if (dst_kind == OSRC_BF16) ((uint16_t *)dst)[idx] = f32_to_bf16_rne(v);
      else ((uint16_t *)dst)[idx] = f32_to_f16_rne(v);
    }
  }
}
