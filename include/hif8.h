/*
 * hif8.h -- C ABI of libhif8: HiFloat8 (HiF8) conversion kernels for AMD MI355X (gfx950).
 *
 * The format and the rounding methods are those of "Ascend HiFloat8 Format for
 * Deep Learning" (arXiv 2409.16626):
 *   Sec. 2.1, Tables 1-3   field layout: sign | dot (prefix code) | exponent Em | mantissa
 *   Eq. (1), Eq. (2)       value of normal / denormal codes; Zero, NaN, +-Inf patterns
 *   Sec. 3.1               rounding half away from zero (TA)
 *   Sec. 3.2, Eq. (3)      hybrid rounding (HR): TA if |E| < 4, else simplified stochastic
 *                          rounding (SR14 for FP32 sources, SR2 for 16-bit sources)
 *   Sec. 3.1, Sec. 3.2     the methods the paper compares these with: rounding half to even
 *                          (TE), simplified SR in every binade, standard SR
 *   Sec. 3 (options)       saturation on overflow, NaN to zero
 *   Sec. 5 (PTS)           per-tensor amax, scale factor, scale before / descale after
 *
 * General conventions (apply to every entry point unless stated otherwise)
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates nothing and frees nothing.  The only state it keeps is a set of
 *     small read-only lookup tables in static device memory, written once per
 *     device by hif8_init().
 *   - Calls only enqueue work on `stream` and return; they never synchronise
 *     (exception: the first call on a device, see hif8_init) and never read
 *     results back to the host.
 *   - Element counts are size_t; kernels index with 64 bits.
 *   - bfloat16 (_bf16 entry points) and IEEE binary16 (_f16 entry points) tensors are
 *     passed as raw uint16_t bit patterns.
 *   - Any pointer alignment and any n are accepted.  The fast path needs the
 *     source 16-byte aligned and the destination(s) aligned to their per-lane
 *     store width (4 B for u8 codes of an FP32 source, 8 B for u8 codes of a
 *     16-bit source, 16 B for FP32 / BF16 / FP16 outputs); otherwise a slower
 *     element-per-lane kernel computes the same result.
 *   - n == 0 is valid and enqueues nothing (hif8_amax_* still writes 0); data pointers
 *     may then be NULL.  Mode and scale are validated first in every case.
 *   - Return value: HIF8_OK, or a negative hif8_status.  On error nothing has
 *     been enqueued.
 *   - Semantics, with fl32() = IEEE binary32 round-to-nearest-even and Q() the
 *     HiF8 rounding selected by `mode`:
 *         encode      dst[i] = code( Q( fl32( widen(src[i]) * scale ) ) )
 *         decode      dst[i] = narrow( fl32( value(src[i]) * fl32(1/scale) ) )
 *         fake_quant  dst[i] = decode(encode(src[i])) with the same scale
 *     narrow() to BF16 / FP16 is round-to-nearest-even.  value(NaN code) is the quiet
 *     NaN 0x7FC00000 (BF16 0x7FC0, FP16 0x7E00), value(Inf codes) is +-Inf, value(0x00) is
 *     +0.0.  scale = 1 gives the paper's plain cast.
 *   - `scale` must be finite and > 0, and 1/scale must be finite and > 0,
 *     else HIF8_ERR_SCALE.
 */
#ifndef HIF8_H_
#define HIF8_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* opaque HIP stream handle (hipStream_t); 0 / NULL is the default stream */
typedef void* hif8_stream_t;

typedef int hif8_status;
enum {
  HIF8_OK = 0,
  HIF8_ERR_NULL = -1,  /* a required pointer is NULL                      */
  HIF8_ERR_MODE = -2,  /* unknown rounding method or unknown flag bits    */
  HIF8_ERR_SCALE = -3, /* scale (or 1/scale) not finite and positive      */
  HIF8_ERR_HIP = -4,   /* a HIP call failed; see hif8_last_hip_error()    */
  HIF8_ERR_ARG = -5    /* any other invalid argument                      */
};

/* rounding_mode bit-field */
#define HIF8_RM_TA 0u            /* Sec. 3.1: round half away from zero                          */
#define HIF8_RM_HR 1u            /* Eq. (3): TA if |E| < 4, else SR14 (FP32 src) / SR2 (16-bit)  */
/* Comparison modes: described by the paper, not adopted by the format. */
#define HIF8_RM_TE 2u            /* Sec. 3.1: round half to even (a tie goes to the neighbour that
                                    is an even multiple of the local step; 0 counts as even)     */
#define HIF8_RM_SSR 3u           /* Sec. 3.2: simplified SR (SR14 / SR2) in every binade         */
#define HIF8_RM_SR 4u            /* Sec. 3.2: standard SR; element i carries iff t_i / 2^32 is
                                    below its discarded fraction, t_i = hif8_sr_threshold(seed, i)
                                    with the seed set by hif8_set_sr_seed                        */
#define HIF8_RM_MASK 0xFu        /* values 5..15 reserved                                        */
#define HIF8_FLAG_SAT 0x10u      /* overflow and +-Inf input -> +-2^15 instead of +-Inf        */
#define HIF8_FLAG_NAN2ZERO 0x20u /* NaN input -> 0x00 instead of 0x80                          */

/* Largest finite HiF8 magnitude (Table 4: max positive normal = 2^15). */
#define HIF8_MAX_FINITE 32768.0f

/* Library version, major*10000 + minor*100 + patch. */
int hif8_version(void);

/* Raw hipError_t of the most recent failing HIP call on this thread (0 if none). */
int hif8_last_hip_error(void);

/*
 * Writes the read-only lookup tables (FP32 pattern -> code for TA, code -> value)
 * into static device memory of the CURRENT device and waits for that to finish.
 * Idempotent and thread-safe.  Every other entry point calls it lazily on first
 * use of a device (that one call synchronises `stream`); callers that must not
 * synchronise later -- e.g. under HIP graph capture -- call hif8_init() once per
 * device beforehand.
 */
hif8_status hif8_init(void);

/*
 * Threshold generator of HIF8_RM_SR.  Sec. 3.2 asks for one uniform random number per element and
 * names no source; a counter-based hash supplies it here, so results are reproducible and
 * independent of the launch shape.  The 32-bit threshold of the element with index i in the
 * threshold stream of a 64-bit seed:
 *     z  = seed + 0x9E3779B97F4A7C15 * (hi32(i) + 1)                         (mod 2^64)
 *     z  = (z ^ z >> 30) * 0xBF58476D1CE4E5B9;  z = (z ^ z >> 27) * 0x94D049BB133111EB;  z ^= z >> 31
 *     k1 = lo32(z), k2 = hi32(z)           (splitmix64's output function; constant over 2^32 elements)
 *     x  = lo32(i) ^ k1;  x ^= x >> 16;  x *= 0x85EBCA6B;  x += k2;  x ^= x >> 13;  x *= 0xC2B2AE35;
 *     t  = x ^ x >> 16                     (MurmurHash3's 32-bit finaliser, keyed at its input and middle)
 * The whole seed enters non-linearly: two seeds give two different functions of the index, not one
 * sequence in another order.
 *   hif8_set_sr_seed    process-wide default seed (default 0); a call without a seed argument uses
 *                       the value in effect when it is enqueued, with index base 0
 *   hif8_sr_threshold   host-side evaluation of t
 *   *_sr entry points   (below) take the seed and the index base of the call explicitly:
 *                       element j of the call draws t(seed, index_base + j).  Casting the tensors
 *                       of one training step with one seed and consecutive index ranges (or one
 *                       seed per tensor) keeps their thresholds independent; a slice of a tensor
 *                       cast with its offset as index base gets the thresholds it has inside the
 *                       whole tensor.
 */
hif8_status hif8_set_sr_seed(uint64_t seed);
uint64_t hif8_get_sr_seed(void);
uint32_t hif8_sr_threshold(uint64_t seed, uint64_t index);

/*
 * Per-tensor amax (Sec. 5, per-tensor scaling): *d_amax = max_i |src[i]|.
 * The maximum is taken over the magnitude bit patterns as unsigned integers, so
 * Inf dominates finite values and any NaN dominates Inf (the result is then a NaN).
 * For FP16 sources the payload of a NaN result is unspecified.
 * d_amax: one device float, overwritten (the call clears it on the stream first).
 */
hif8_status hif8_amax_f32(const float* src, size_t n, float* d_amax, hif8_stream_t stream);
hif8_status hif8_amax_bf16(const uint16_t* src, size_t n, float* d_amax, hif8_stream_t stream);
hif8_status hif8_amax_f16(const uint16_t* src, size_t n, float* d_amax, hif8_stream_t stream);

/*
 * Scale factor from a device-resident amax, without a host round trip
 * (Sec. 5, per-tensor scaling: each GEMM input is multiplied by its own factor so that
 * it sits well inside the HiF8 range; power-of-two factors add no rounding error).
 *   d_scale2[0] = scale = fl32(target / amax), or with pow2 != 0 the largest power
 *                 of two not above it; amax zero, Inf or NaN (or a quotient that
 *                 is not finite and positive) gives scale = 1.
 *   d_scale2[1] = fl32(1 / scale).
 * d_amax: one device float (input).  d_scale2: two device floats (output).
 */
hif8_status hif8_scale_from_amax(const float* d_amax, float* d_scale2, float target, int pow2,
                                 hif8_stream_t stream);

/*
 * Encode (Sec. 3; Tables 1-3): n source values -> n packed u8 HiF8 codes.
 * src and dst must not overlap.
 */
hif8_status hif8_encode_f32(const float* src, uint8_t* dst, size_t n, float scale,
                            uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_encode_bf16(const uint16_t* src, uint8_t* dst, size_t n, float scale,
                             uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_encode_f16(const uint16_t* src, uint8_t* dst, size_t n, float scale,
                            uint32_t rounding_mode, hif8_stream_t stream);

/*
 * Decode (Eq. (1), Eq. (2), special patterns): n u8 codes -> n values, descaled.
 * src and dst must not overlap.
 */
hif8_status hif8_decode_f32(const uint8_t* src, float* dst, size_t n, float scale,
                            hif8_stream_t stream);
hif8_status hif8_decode_bf16(const uint8_t* src, uint16_t* dst, size_t n, float scale,
                             hif8_stream_t stream);
hif8_status hif8_decode_f16(const uint8_t* src, uint16_t* dst, size_t n, float scale,
                            hif8_stream_t stream);

/*
 * Fake quantisation (Sec. 4: the paper's simulated HiF8 -- every tensor value is
 * replaced by the HiF8-representable value it rounds to, kept in the source data type):
 * encode and decode fused in registers.
 * dst may equal src (in place).  codes_or_null, if not NULL, also receives the
 * n u8 codes and must not overlap src or dst.
 */
hif8_status hif8_fake_quant_f32(const float* src, float* dst, uint8_t* codes_or_null, size_t n,
                                float scale, uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_fake_quant_bf16(const uint16_t* src, uint16_t* dst, uint8_t* codes_or_null,
                                 size_t n, float scale, uint32_t rounding_mode,
                                 hif8_stream_t stream);
hif8_status hif8_fake_quant_f16(const uint16_t* src, uint16_t* dst, uint8_t* codes_or_null,
                                size_t n, float scale, uint32_t rounding_mode,
                                hif8_stream_t stream);

/*
 * Device-state ("_ds") variants: identical to the calls above except that
 *   - the scale pair is read by the kernel from d_scale2 = {scale, fl32(1/scale)} in device
 *     memory, as written by hif8_scale_from_amax on the same stream (not validated: the host
 *     never sees the values);
 *   - encode and fake_quant take d_amax_accum_or_null: if not NULL, the same pass also
 *     accumulates max_i |src[i]| of the UNSCALED input into that device float with an atomic
 *     max on its bit pattern (same ordering as hif8_amax_*).  This is the delayed scaling of
 *     Sec. 5 (amax gathered every few iterations feeds the scale of later ones) at no extra
 *     memory pass.  The call does not clear the accumulator: the caller starts a window by
 *     writing 0 to it (hif8_amax_* with n = 0 does that on the stream).
 */
hif8_status hif8_encode_f32_ds(const float* src, uint8_t* dst, size_t n, const float* d_scale2,
                               float* d_amax_accum_or_null, uint32_t rounding_mode,
                               hif8_stream_t stream);
hif8_status hif8_encode_bf16_ds(const uint16_t* src, uint8_t* dst, size_t n,
                                const float* d_scale2, float* d_amax_accum_or_null,
                                uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_encode_f16_ds(const uint16_t* src, uint8_t* dst, size_t n,
                               const float* d_scale2, float* d_amax_accum_or_null,
                               uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_decode_f32_ds(const uint8_t* src, float* dst, size_t n, const float* d_scale2,
                               hif8_stream_t stream);
hif8_status hif8_decode_bf16_ds(const uint8_t* src, uint16_t* dst, size_t n,
                                const float* d_scale2, hif8_stream_t stream);
hif8_status hif8_decode_f16_ds(const uint8_t* src, uint16_t* dst, size_t n,
                               const float* d_scale2, hif8_stream_t stream);
hif8_status hif8_fake_quant_f32_ds(const float* src, float* dst, uint8_t* codes_or_null, size_t n,
                                   const float* d_scale2, float* d_amax_accum_or_null,
                                   uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_fake_quant_bf16_ds(const uint16_t* src, uint16_t* dst, uint8_t* codes_or_null,
                                    size_t n, const float* d_scale2, float* d_amax_accum_or_null,
                                    uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_fake_quant_f16_ds(const uint16_t* src, uint16_t* dst, uint8_t* codes_or_null,
                                   size_t n, const float* d_scale2, float* d_amax_accum_or_null,
                                   uint32_t rounding_mode, hif8_stream_t stream);

/*
 * Casts with an explicit threshold stream for HIF8_RM_SR (Sec. 3.2: one random number per element):
 * hif8_encode_* / hif8_fake_quant_* with the seed and the index base of this call as arguments
 * instead of the process-wide seed (see hif8_set_sr_seed).  Any rounding_mode is accepted; only
 * HIF8_RM_SR looks at the two values.  index_base + n must not exceed 2^64.
 */
hif8_status hif8_encode_f32_sr(const float* src, uint8_t* dst, size_t n, float scale,
                               uint32_t rounding_mode, uint64_t seed, uint64_t index_base,
                               hif8_stream_t stream);
hif8_status hif8_encode_bf16_sr(const uint16_t* src, uint8_t* dst, size_t n, float scale,
                                uint32_t rounding_mode, uint64_t seed, uint64_t index_base,
                                hif8_stream_t stream);
hif8_status hif8_encode_f16_sr(const uint16_t* src, uint8_t* dst, size_t n, float scale,
                               uint32_t rounding_mode, uint64_t seed, uint64_t index_base,
                               hif8_stream_t stream);
hif8_status hif8_fake_quant_f32_sr(const float* src, float* dst, uint8_t* codes_or_null, size_t n,
                                   float scale, uint32_t rounding_mode, uint64_t seed,
                                   uint64_t index_base, hif8_stream_t stream);
hif8_status hif8_fake_quant_bf16_sr(const uint16_t* src, uint16_t* dst, uint8_t* codes_or_null,
                                    size_t n, float scale, uint32_t rounding_mode, uint64_t seed,
                                    uint64_t index_base, hif8_stream_t stream);
hif8_status hif8_fake_quant_f16_sr(const uint16_t* src, uint16_t* dst, uint8_t* codes_or_null,
                                   size_t n, float scale, uint32_t rounding_mode, uint64_t seed,
                                   uint64_t index_base, hif8_stream_t stream);

/*
 * Per-tensor scaling in one call (Sec. 5, per-tensor scaling: amax of the tensor, scale factor
 * from it, scale and cast):
 *     d_amax[0]   = max_i |src[i]|                         as hif8_amax_*
 *     d_scale2[0] = scale, d_scale2[1] = fl32(1 / scale)   as hif8_scale_from_amax(d_amax, target, pow2)
 *     codes[i]    = code(Q(fl32(widen(src[i]) * scale)))   as hif8_encode_*_ds          (if codes != NULL)
 *     dst[i]      = decode(codes[i]) descaled              as hif8_fake_quant_*_ds      (if dst != NULL)
 * i.e. exactly what the three separate calls produce, in two launches instead of four: the first
 * pass leaves one partial maximum per workgroup in `workspace`, and every workgroup of the cast
 * reduces those and derives the scale itself (no clearing launch, no atomics, no scale launch).
 * The first pass reads with ordinary loads, so a tensor that fits the 256 MB last-level cache is
 * still there when the cast reads it again.
 * At least one of dst, codes must be given; dst may equal src.  d_amax: one device float,
 * d_scale2: two device floats, both written.  workspace: device scratch of at least
 * hif8_quantize_workspace_bytes() bytes (4 KiB), 4-byte aligned, caller-owned; its contents need
 * not be kept between calls, and calls that share it must not overlap in time.  n == 0 writes
 * amax 0 and the pair {1, 1}.  Inputs that miss the fast path's alignment (see the general
 * conventions) are handed to the separate calls.  Errors: HIF8_ERR_MODE, HIF8_ERR_ARG (target not
 * finite and positive, workspace too small or misaligned), HIF8_ERR_NULL.
 */
size_t hif8_quantize_workspace_bytes(void);
hif8_status hif8_quantize_tensor_f32(const float* src, float* dst_or_null, uint8_t* codes_or_null,
                                     size_t n, float target, int pow2, uint32_t rounding_mode,
                                     float* d_amax, float* d_scale2, void* workspace,
                                     size_t workspace_bytes, hif8_stream_t stream);
hif8_status hif8_quantize_tensor_bf16(const uint16_t* src, uint16_t* dst_or_null,
                                      uint8_t* codes_or_null, size_t n, float target, int pow2,
                                      uint32_t rounding_mode, float* d_amax, float* d_scale2,
                                      void* workspace, size_t workspace_bytes, hif8_stream_t stream);
hif8_status hif8_quantize_tensor_f16(const uint16_t* src, uint16_t* dst_or_null,
                                     uint8_t* codes_or_null, size_t n, float target, int pow2,
                                     uint32_t rounding_mode, float* d_amax, float* d_scale2,
                                     void* workspace, size_t workspace_bytes, hif8_stream_t stream);

/*
 * hif8_quantize_tensor_* for callers that cannot provide (or allocate) a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid allocation.  Same results as
 * hif8_quantize_tensor_{f32,bf16,f16} (src_kind selects which); the partial maxima live in a 4 KiB
 * array in static device memory of the library instead (one copy per GPU, held until the process
 * ends).  The call allocates nothing and frees nothing.  Every call on a GPU shares that GPU's
 * array: calls that overlap in time on one GPU (two streams, two threads) race and give wrong
 * results -- serialise them, or use the workspace form.  n above HIF8_STATIC_MAX_ELEMENTS (2^32) is
 * refused with HIF8_ERR_ARG, as is an unknown src_kind; other errors as hif8_quantize_tensor_*.
 * src, dst_or_null: tensors of the kind src_kind names.
 */
#define HIF8_KIND_F32 0
#define HIF8_KIND_BF16 1
#define HIF8_KIND_F16 2
#define HIF8_STATIC_MAX_ELEMENTS ((size_t)1 << 32)
hif8_status hif8_quantize_tensor_static(const void* src, void* dst_or_null, uint8_t* codes_or_null,
                                        size_t n, int src_kind, float target, int pow2,
                                        uint32_t rounding_mode, float* d_amax, float* d_scale2,
                                        hif8_stream_t stream);

/*
 * Multi-tensor cast: per-tensor amax, scale and encode for a whole list of tensors in a few
 * launches instead of four per tensor -- the per-tensor scaling recipe of Sec. 5 applied to every
 * weight (or activation) tensor of a model at once.
 *
 *   hif8_cast_item   one tensor: src (device, 16-byte aligned; all items of a list have the
 *                    same type), dst (device, n u8 codes, 8-byte aligned for BF16 / FP16
 *                    sources, 4-byte for FP32), n elements,
 *                    first_tile (filled by hif8_multi_plan).
 *   hif8_multi_plan  HOST-side helper: validates a HOST array of items, fills first_tile and
 *                    returns the total tile count.  The caller then copies the array to
 *                    device memory (it may be reused for any number of casts).
 *   hif8_multi_cast_{bf16,f16,f32}
 *                    d_items: the planned array in DEVICE memory; host_items_or_null: the same
 *                    planned array in HOST memory (read during the call only, for the sizes);
 *                    d_amax: count device floats (output, amax per tensor); d_scale2: 2*count
 *                    device floats (output, {scale, 1/scale} per tensor, as
 *                    hif8_scale_from_amax); target, pow2 as in hif8_scale_from_amax.  Results
 *                    equal the per-tensor sequence hif8_amax_* -> hif8_scale_from_amax ->
 *                    hif8_encode_*_ds.  With the host copy the list is cut into groups of whole
 *                    tensors of about 192 MiB of source (at most 16 tensors), and one launch per group
 *                    gathers the amax of that group while it casts the previous one, whose source was
 *                    read a moment before: the two passes overlap and no launch has to wait for
 *                    the whole list.  Without it (NULL): amax of all tensors, scales, cast of all
 *                    tensors (four launches).  HIF8_ERR_ARG if the host copy does not match
 *                    total_tiles.
 *   hif8_multi_encode_{bf16,f16,f32}_ds
 *                    the cast alone, in ONE launch, with scales that are already on the device
 *                    (delayed scaling, Sec. 5: scales from earlier iterations): d_scale2: 2*count
 *                    device floats (input, {scale, 1/scale} per tensor); d_amax_accum_or_null:
 *                    count device floats, or null; when given, the amax of every tensor's source
 *                    is accumulated into its entry (max with what the entry holds; the call does
 *                    not clear it), as the *_ds casts do for one tensor.  Results equal
 *                    hif8_encode_*_ds per tensor.
 * Misaligned items make hif8_multi_plan return HIF8_ERR_ARG (use the per-tensor calls).
 */
typedef struct hif8_cast_item {
  const void* src;
  uint8_t* dst;
  uint64_t n;
  uint64_t first_tile;
} hif8_cast_item;

hif8_status hif8_multi_plan(hif8_cast_item* host_items, size_t count, int src_is_16bit,
                            uint64_t* total_tiles_out);
hif8_status hif8_multi_cast_bf16(const hif8_cast_item* host_items_or_null, const hif8_cast_item* d_items,
                                 size_t count, uint64_t total_tiles,
                                 float* d_amax, float* d_scale2, float target, int pow2,
                                 uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_multi_cast_f32(const hif8_cast_item* host_items_or_null, const hif8_cast_item* d_items,
                                 size_t count, uint64_t total_tiles,
                                float* d_amax, float* d_scale2, float target, int pow2,
                                uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_multi_encode_bf16_ds(const hif8_cast_item* d_items, size_t count, uint64_t total_tiles,
                                      const float* d_scale2, float* d_amax_accum_or_null,
                                      uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_multi_encode_f32_ds(const hif8_cast_item* d_items, size_t count, uint64_t total_tiles,
                                     const float* d_scale2, float* d_amax_accum_or_null,
                                     uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_multi_encode_f16_ds(const hif8_cast_item* d_items, size_t count, uint64_t total_tiles,
                                     const float* d_scale2, float* d_amax_accum_or_null,
                                     uint32_t rounding_mode, hif8_stream_t stream);
hif8_status hif8_multi_cast_f16(const hif8_cast_item* host_items_or_null, const hif8_cast_item* d_items,
                                 size_t count, uint64_t total_tiles,
                                float* d_amax, float* d_scale2, float target, int pow2,
                                uint32_t rounding_mode, hif8_stream_t stream);

/*
 * Scale sweep: the cast-and-score step of Algorithm 1 (HiF8 calibration with per-tensor
 * scaling: try a run of power-of-two scale factors, keep the one with the smallest error)
 * applied to one tensor, in one pass over it.  For k = 0 .. count-1, e = e_lo + k:
 *     d_err[k] = sum_i ( x_i - value(Q(fl32(x_i * 2^e))) * 2^-e )^2          (MSE = d_err[k] / n)
 * Differences, squares and sums are fp64; a cast that overflows to Infinity makes the sum +Inf,
 * a NaN element makes it NaN (HIF8_FLAG_SAT keeps overflow finite).  Partial sums are combined
 * with fp64 atomics, so the last bits depend on the order (relative spread ~1e-15).
 * Algorithm 1 proper scores the layer output; hif8_calibrate_layer does that with the GEMM.
 * count in [1, 16]; |e| <= 126.  d_err: count device doubles, overwritten.  n == 0 gives zeros.
 */
hif8_status hif8_scale_sweep_f32(const float* src, size_t n, int e_lo, int count,
                                 uint32_t rounding_mode, double* d_err, hif8_stream_t stream);
hif8_status hif8_scale_sweep_bf16(const uint16_t* src, size_t n, int e_lo, int count,
                                  uint32_t rounding_mode, double* d_err, hif8_stream_t stream);
hif8_status hif8_scale_sweep_f16(const uint16_t* src, size_t n, int e_lo, int count,
                                 uint32_t rounding_mode, double* d_err, hif8_stream_t stream);

/*
 * Per-channel scaling of a row-major [rows, cols] matrix (Sec. 4.2 names per-tensor scaling
 * for activations with per-channel scaling for weights as a further method).  axis = 0: one
 * scale per row; axis = 1: one scale per column.  nch = rows or cols accordingly.
 *   hif8_amax_axis_*        d_amax[ch] = max |x| over the channel (nch device floats, overwritten;
 *                           same ordering of Inf / NaN as hif8_amax_*)
 *   hif8_scale_from_amax_n  hif8_scale_from_amax for `count` consecutive amax values:
 *                           d_scale2[2 ch] = scale, d_scale2[2 ch + 1] = fl32(1 / scale)
 *   hif8_encode_axis_*      dst[r, c] = code(Q(fl32(x[r, c] * scale[ch])))  (standard-SR thresholds
 *                           are indexed by the flat element index r * cols + c)
 *   hif8_decode_axis_*      dst[r, c] = narrow(fl32(value(src[r, c]) * fl32(1 / scale[ch])))
 * The fast paths need 16-byte aligned matrices (codes: 4 / 8 bytes as for hif8_encode_*) and
 * cols a multiple of 4 (FP32) or 8 (16-bit); anything else takes an element-per-lane path.
 * rows and cols must each be below 2^31.
 */
hif8_status hif8_scale_from_amax_n(const float* d_amax, float* d_scale2, size_t count, float target,
                                   int pow2, hif8_stream_t stream);
hif8_status hif8_amax_axis_f32(const float* src, size_t rows, size_t cols, int axis, float* d_amax,
                               hif8_stream_t stream);
hif8_status hif8_amax_axis_bf16(const uint16_t* src, size_t rows, size_t cols, int axis,
                                float* d_amax, hif8_stream_t stream);
hif8_status hif8_amax_axis_f16(const uint16_t* src, size_t rows, size_t cols, int axis,
                               float* d_amax, hif8_stream_t stream);
hif8_status hif8_encode_axis_f32(const float* src, uint8_t* dst, size_t rows, size_t cols, int axis,
                                 const float* d_scale2, uint32_t rounding_mode,
                                 hif8_stream_t stream);
hif8_status hif8_encode_axis_bf16(const uint16_t* src, uint8_t* dst, size_t rows, size_t cols,
                                  int axis, const float* d_scale2, uint32_t rounding_mode,
                                  hif8_stream_t stream);
hif8_status hif8_encode_axis_f16(const uint16_t* src, uint8_t* dst, size_t rows, size_t cols,
                                 int axis, const float* d_scale2, uint32_t rounding_mode,
                                 hif8_stream_t stream);
hif8_status hif8_decode_axis_f32(const uint8_t* src, float* dst, size_t rows, size_t cols, int axis,
                                 const float* d_scale2, hif8_stream_t stream);
hif8_status hif8_decode_axis_bf16(const uint8_t* src, uint16_t* dst, size_t rows, size_t cols,
                                  int axis, const float* d_scale2, hif8_stream_t stream);
hif8_status hif8_decode_axis_f16(const uint8_t* src, uint16_t* dst, size_t rows, size_t cols,
                                 int axis, const float* d_scale2, hif8_stream_t stream);

/*
 * Per-row scaling (channels along axis 0, the layout of a weight matrix [out channels, in]; Sec. 4.2
 * names per-channel scaling of weights as a further method) in one call and, where a row fits the
 * registers of a workgroup, one pass over the source:
 *     d_amax[r]  = max_c |src[r, c]|                      (rows device floats, always written)
 *     d_scale2[2 r], [2 r + 1] = scale, fl32(1 / scale)    as hif8_scale_from_amax(d_amax[r], target, pow2)
 *     dst[r, c]  = code(Q(fl32(src[r, c] * scale)))
 * i.e. exactly what hif8_amax_axis_* (axis 0), hif8_scale_from_amax_n and hif8_encode_axis_* (axis 0)
 * produce in three launches and two reads of the source.  The single-pass form needs the fast-path
 * alignment of hif8_encode_axis_* and at most 16,384 (FP32) or 32,768 (16-bit) columns; other inputs
 * are handed to the three separate launches.  All pointers are device pointers owned by the caller;
 * rows == 0 is a no-op; HIF8_ERR_NULL for a null d_amax or d_scale2 (or null data with rows * cols > 0),
 * HIF8_ERR_MODE / HIF8_ERR_ARG as for the separate calls.
 */
hif8_status hif8_quantize_rows_f32(const float* src, uint8_t* dst, size_t rows, size_t cols, float target,
                                   int pow2, uint32_t rounding_mode, float* d_amax, float* d_scale2,
                                   hif8_stream_t stream);
hif8_status hif8_quantize_rows_bf16(const uint16_t* src, uint8_t* dst, size_t rows, size_t cols, float target,
                                    int pow2, uint32_t rounding_mode, float* d_amax, float* d_scale2,
                                    hif8_stream_t stream);
hif8_status hif8_quantize_rows_f16(const uint16_t* src, uint8_t* dst, size_t rows, size_t cols, float target,
                                   int pow2, uint32_t rounding_mode, float* d_amax, float* d_scale2,
                                   hif8_stream_t stream);

/*
 * Per-tensor scaling state for training (Sec. 5.1, PTS): one scale per GEMM input tensor, all 1
 * at the start; every `interval` iterations (the paper uses 10) the amax of each tensor is
 * gathered and its scale becomes the largest power of two s with amax * s <= target; in every
 * iteration the current scale multiplies the tensor before the cast and the GEMM output is
 * descaled.  The paper leaves the update rule open ("a certain algorithm") apart from the
 * power-of-two restriction; a tensor whose gathered amax is 0, Inf or NaN keeps its scale.
 *
 * The state lives in caller-owned device memory: d_amax (count floats, the accumulators that
 * the _ds casts fill through d_amax_accum_or_null, or hif8_amax_* / hif8_multi_cast_* write)
 * and d_scale2 (count {scale, 1/scale} pairs, read by the _ds casts).  Both arrays have the layout
 * that hif8_multi_encode_*_ds takes, so all tensors of the state can be cast in one launch (pass
 * d_amax as its accumulators on gathering iterations, null otherwise).  The struct itself is
 * host memory owned by the caller; the library keeps no reference to it.
 *   hif8_pts_init           scales = 1, accumulators = 0, iteration = 0 (one small launch);
 *                           target must be a power of two (HiF8's largest finite value 2^15, or
 *                           lower to leave headroom), interval >= 1
 *   hif8_pts_collects       1 if the current iteration is one that gathers amax
 *                           (iteration % interval == 0), else 0: pass the accumulators to the
 *                           casts only then
 *   hif8_pts_end_iteration  on a gathering iteration: one launch that refreshes every scale from
 *                           its accumulator and clears the accumulator; then iteration += 1.
 *                           The new scales apply from the next cast enqueued on the stream
 *                           (delayed scaling: no second pass over the tensors).
 */
typedef struct hif8_pts_state {
  float* d_amax;
  float* d_scale2;
  uint32_t count;
  uint32_t interval;
  float target;
  uint64_t iteration;
} hif8_pts_state;

hif8_status hif8_pts_init(hif8_pts_state* st, float* d_amax, float* d_scale2, size_t count,
                          uint32_t interval, float target, hif8_stream_t stream);
int hif8_pts_collects(const hif8_pts_state* st);
hif8_status hif8_pts_end_iteration(hif8_pts_state* st, hif8_stream_t stream);

/*
 * Adaptive loss scaling (Sec. 5.1, ALS): the dynamic loss scale of mixed-precision training
 * (halve on an overflow, double after `window` overflow-free iterations) with a window that
 * moves along {1, 20, 50, 100, 200, 500, 1000}: initial scale 2^32, initial window 20; three
 * scale increases since the last window change move the window one place up, three decreases
 * in a row move it one place down.  Host-only state machine (no device work): the caller
 * reports per iteration whether the gradients overflowed (e.g. hif8_amax_* returned Inf / NaN).
 * The scale stays within [1, 2^126].
 */
typedef struct hif8_als_state {
  float scale;
  int32_t window_index;
  int32_t good_steps;
  int32_t increases;
  int32_t decrease_streak;
} hif8_als_state;

void hif8_als_init(hif8_als_state* st);
int hif8_als_window(const hif8_als_state* st); /* current window length, -1 on a bad state */
hif8_status hif8_als_update(hif8_als_state* st, int found_overflow);

/*
 * Simulated HiF8 GEMM (Sec. 4 / Sec. 5: the GEMM inputs are cast to HiF8 and the product is
 * taken on the represented values; Algorithm 1 "MatMul & Restore": the product is descaled by
 * the two input scales):
 *     out[m, n] = fl32( (sum_k value(a[m, k]) * value(b[n, k])) * fl32(fl32(1/scale_a) * fl32(1/scale_b)) )
 * a_codes: [M, K] u8, b_codes: [N, K] u8, both row-major with K contiguous (b is the weight in
 * [out_features, in_features] order); out: [M, N] row-major FP32 / BF16 / FP16 (round to
 * nearest even).  Products are exact; sums are FP32 on the matrix cores (bf16 MFMA, every HiF8
 * value is exact in bfloat16), so results agree with exact arithmetic to within
 * K * 2^-23 * sum_k |a b| * descale per element, and the summation order is fixed for a given
 * shape and tile variant.  NaN / Inf codes propagate by IEEE rules.
 * The matrix-core path needs K % 16 == 0 and 16-byte aligned operands; anything else takes a
 * plain one-element-per-lane kernel.  M, N, K < 2^31.
 *   hif8_gemm_sqerr   no output matrix: *d_err += sum (out[m, n] - ref[m, n])^2 in fp64
 *                     (ref: [M, N] FP32; the caller clears *d_err) -- the "Quantization Error"
 *                     step of Algorithm 1.
 */
hif8_status hif8_gemm_f32(const uint8_t* a_codes, const uint8_t* b_codes, float* out, size_t M,
                          size_t N, size_t K, float scale_a, float scale_b, hif8_stream_t stream);
hif8_status hif8_gemm_bf16(const uint8_t* a_codes, const uint8_t* b_codes, uint16_t* out, size_t M,
                           size_t N, size_t K, float scale_a, float scale_b, hif8_stream_t stream);
hif8_status hif8_gemm_f16(const uint8_t* a_codes, const uint8_t* b_codes, uint16_t* out, size_t M,
                          size_t N, size_t K, float scale_a, float scale_b, hif8_stream_t stream);
hif8_status hif8_gemm_sqerr(const uint8_t* a_codes, const uint8_t* b_codes, const float* ref, size_t M,
                            size_t N, size_t K, float scale_a, float scale_b, double* d_err,
                            hif8_stream_t stream);

/*
 * The same GEMM on operands expanded to bfloat16 beforehand.  Every HiF8 value is exact in
 * bfloat16, so a code matrix that takes part in several products (the 10 + 10 casts and 100
 * products of Algorithm 1's search; a cast weight used by the forward and the backward GEMM of a
 * training step, Sec. 5) is expanded once and the products then run without the decoder: tiles go
 * from HBM straight into LDS and the kernel is faster than the code-operand one for
 * matrix-core-bound shapes, at 2 bytes per operand element instead of 1.
 *   hif8_expanded_ld(K)   row pitch (elements) of an expanded operand: K rounded up to a multiple of 64
 *   hif8_expand_bf16      dst[r * ld + k] = bf16 pattern of value(codes[r * K + k]) for k < K and 0 for
 *                         K <= k < ld.  codes: [rows, K] u8 device; dst: [rows, ld] u16 device, 16-byte
 *                         aligned, caller-owned; ld a multiple of 64 and >= K.  (NaN / Inf codes expand
 *                         to NaN / Inf and propagate through the product.)
 *   hif8_expand_bf16_t    the same with a transposition: dst[c * ld + r] = value(codes[r * cols + c]) for r < rows and 0
 *                         for rows <= r < ld; dst: [cols, ld], ld a multiple of 64 and >= rows.  With it the three
 *                         products of a linear layer all run on the one K-contiguous kernel (X: [M, K], W: [N, K], dY: [M, N]):
 *                         Y = X W^T from expand(X), expand(W); dX = dY W from expand(dY), expand_t(W);
 *                         dW = dY^T X from expand_t(dY), expand_t(X).
 *   hif8_gemm_expanded_*  out[m, n] = fl32( (sum_k a[m, k] * b[n, k]) * fl32(fl32(1/scale_a) * fl32(1/scale_b)) )
 *                         a: [M, ld], b: [N, ld] u16 bfloat16 patterns as written by hif8_expand_bf16
 *                         (16-byte aligned; the columns K .. ld-1 must hold zeros); out / ref / d_err as in
 *                         hif8_gemm_*.  K >= 1, ld <= 2^22; M, N < 2^31.  Same error bound as hif8_gemm_*; the summation
 *                         order differs from that kernel's, so the two agree to within that bound, and
 *                         exactly whenever every partial sum is exact in FP32.
 */
size_t hif8_expanded_ld(size_t K);
hif8_status hif8_expand_bf16(const uint8_t* codes, size_t rows, size_t K, uint16_t* dst, size_t ld,
                             hif8_stream_t stream);
hif8_status hif8_expand_bf16_t(const uint8_t* codes, size_t rows, size_t cols, uint16_t* dst, size_t ld,
                               hif8_stream_t stream);
hif8_status hif8_gemm_expanded_f32(const uint16_t* a, const uint16_t* b, float* out, size_t M, size_t N,
                                   size_t K, size_t ld, float scale_a, float scale_b,
                                   hif8_stream_t stream);
hif8_status hif8_gemm_expanded_bf16(const uint16_t* a, const uint16_t* b, uint16_t* out, size_t M,
                                    size_t N, size_t K, size_t ld, float scale_a, float scale_b,
                                    hif8_stream_t stream);
hif8_status hif8_gemm_expanded_f16(const uint16_t* a, const uint16_t* b, uint16_t* out, size_t M,
                                   size_t N, size_t K, size_t ld, float scale_a, float scale_b,
                                   hif8_stream_t stream);
hif8_status hif8_gemm_expanded_sqerr(const uint16_t* a, const uint16_t* b, const float* ref, size_t M,
                                     size_t N, size_t K, size_t ld, float scale_a, float scale_b,
                                     double* d_err, hif8_stream_t stream);

/*
 * hif8_gemm_* on code operands with a workspace: both code matrices are expanded to bfloat16 into the
 * workspace (hif8_expand_bf16) and multiplied by the expanded-operand kernel -- three launches on `stream`, and
 * for matrix-core-bound shapes about two thirds of the time of hif8_gemm_* (whose kernel expands the codes on
 * their way into LDS and is bound by that work).  Arguments, result and error bound as for hif8_gemm_* (the
 * result equals that of hif8_gemm_expanded_* on the expanded operands bit for bit); any K and any alignment of
 * the code matrices.
 * workspace: device memory, 16-byte aligned, at least hif8_gemm_workspace_bytes(M, N, K) bytes
 * (= 2 (M + N) hif8_expanded_ld(K), 0 when M, N or K is 0), caller-owned, free for other use once the
 * work enqueued here has run; a smaller workspace_bytes is HIF8_ERR_ARG.  K beyond 2^22 (the expanded-operand
 * kernel's limit) falls back to the hif8_gemm_* kernel and leaves the workspace unused.
 */
size_t hif8_gemm_workspace_bytes(size_t M, size_t N, size_t K);
hif8_status hif8_gemm_ws_f32(const uint8_t* a_codes, const uint8_t* b_codes, float* out, size_t M, size_t N,
                             size_t K, float scale_a, float scale_b, void* workspace, size_t workspace_bytes,
                             hif8_stream_t stream);
hif8_status hif8_gemm_ws_bf16(const uint8_t* a_codes, const uint8_t* b_codes, uint16_t* out, size_t M, size_t N,
                              size_t K, float scale_a, float scale_b, void* workspace, size_t workspace_bytes,
                              hif8_stream_t stream);
hif8_status hif8_gemm_ws_f16(const uint8_t* a_codes, const uint8_t* b_codes, uint16_t* out, size_t M, size_t N,
                             size_t K, float scale_a, float scale_b, void* workspace, size_t workspace_bytes,
                             hif8_stream_t stream);
hif8_status hif8_gemm_ws_sqerr(const uint8_t* a_codes, const uint8_t* b_codes, const float* ref, size_t M, size_t N,
                               size_t K, float scale_a, float scale_b, double* d_err, void* workspace,
                               size_t workspace_bytes, hif8_stream_t stream);

/*
 * Algorithm 1 (HiF8 calibration with per-tensor scaling) for ONE layer: given the layer's
 * high-precision input a [M, K], weight w [N, K] (K contiguous in both) and high-precision
 * output o_ref [M, N] (FP32), try every pair of power-of-two scales 2^Ea, 2^Ew with
 * Ea = ea_lo .. ea_lo + ea_count - 1, Ew likewise (the paper searches [-4, 5] x [-4, 5]):
 *     A_q = Q(a * 2^Ea),  W_q = Q(w * 2^Ew),  O_q = (A_q x W_q^T) * 2^-(Ea + Ew),
 *     d_err[i * ew_count + j] = sum (O_q - o_ref)^2          (fp64; MSE = d_err / (M N))
 * and, if d_best_or_null is given, write the pair with the smallest finite error to it as two
 * int32 {Ea, Ew}.  The paper casts with TA here; any rounding_mode is accepted.  The model-level
 * loop (collecting o_ref, feeding O_q through the non-linearities to the next layer) is the
 * caller's.  Enqueues ea_count + ew_count casts (each followed by its expansion to bfloat16) and
 * ea_count * ew_count error GEMMs (one batched launch) on `stream`.
 * workspace: device scratch for one code matrix and the expanded operands, at least
 * hif8_calibrate_workspace_bytes(M, N, K, ea_count, ew_count) bytes, 16-byte aligned, caller-owned.
 * Counts are limited to 64 each, exponents to [-60, 60], K to 2^22.
 */
size_t hif8_calibrate_workspace_bytes(size_t M, size_t N, size_t K, int ea_count, int ew_count);
hif8_status hif8_calibrate_layer_f32(const float* a, const float* w, const float* o_ref, size_t M,
                                     size_t N, size_t K, int ea_lo, int ea_count, int ew_lo,
                                     int ew_count, uint32_t rounding_mode, void* workspace,
                                     size_t workspace_bytes, double* d_err, int32_t* d_best_or_null,
                                     hif8_stream_t stream);
hif8_status hif8_calibrate_layer_bf16(const uint16_t* a, const uint16_t* w, const float* o_ref,
                                      size_t M, size_t N, size_t K, int ea_lo, int ea_count,
                                      int ew_lo, int ew_count, uint32_t rounding_mode,
                                      void* workspace, size_t workspace_bytes, double* d_err,
                                      int32_t* d_best_or_null, hif8_stream_t stream);
hif8_status hif8_calibrate_layer_f16(const uint16_t* a, const uint16_t* w, const float* o_ref,
                                     size_t M, size_t N, size_t K, int ea_lo, int ea_count,
                                     int ew_lo, int ew_count, uint32_t rounding_mode,
                                     void* workspace, size_t workspace_bytes, double* d_err,
                                     int32_t* d_best_or_null, hif8_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* HIF8_H_ */
