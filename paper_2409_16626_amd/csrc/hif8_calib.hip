// Calibration-side kernels of libhif8 (gfx950):
//   scale sweep       the cast-and-score step of Algorithm 1 (HiF8 calibration with per-tensor
//                     scaling) applied to one tensor: squared cast error at a run of
//                     power-of-two scales, one read of the tensor for all of them;
//   per-channel ops   amax / encode / decode of a row-major matrix with one scale per row or per
//                     column (Sec. 4.2 names per-channel weight scaling as a further method).
// They reuse the element encoders and the streaming helpers of the conversion kernels.
#include "hif8_conv.hpp"

namespace hif8calib {

using namespace hif8dev;
using namespace hif8host;
using namespace hif8conv;

constexpr int kSweepMax = 16;  // scales per call
constexpr int kSweepBlock = 256;

__device__ __forceinline__ double wave_sum_f64(double v) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
  return v;
}

// err[k] += the workgroup's sum of acc[k], k < count: wavefront sums by shuffles, across the
// wavefronts through LDS, then ONE hardware fp64 atomic per scale and workgroup (thousands of
// wavefronts adding to the same few addresses would otherwise serialise at the L2).
// Every lane of the workgroup must call it.
template <int KMAX>
__device__ __forceinline__ void block_add_f64(const double (&acc)[KMAX], int count, double* __restrict__ err) {
  __shared__ double part[kSweepBlock / 64][kSweepMax];
  const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    if (k < count) {
      const double w = wave_sum_f64(acc[k]);
      if (lane == 0u) part[wv][k] = w;
    }
  }
  __syncthreads();
  if (threadIdx.x < (uint32_t)count) {
    double t = part[0][threadIdx.x];
    for (uint32_t w = 1; w < blockDim.x / 64u; ++w) t += part[w][threadIdx.x];
    unsafeAtomicAdd(err + threadIdx.x, t);
  }
}

// err[k] += sum over this workgroup's elements of (x - value(Q(x * 2^(e_lo+k))) * 2^-(e_lo+k))^2.
// The differences and squares are taken in fp64 (exact for every finite term), lane sums are
// fp64, and each workgroup adds its total with one fp64 atomic per scale.
// NSC: number of scales fixed at compile time (straight-line code), or 0: `count` at run time.
template <int IMPL, int SRCK, int NSC>
__global__ void __launch_bounds__(kSweepBlock)
k_scale_sweep(const void* __restrict__ src, size_t n, int e_lo, int count_arg, uint32_t mode, uint64_t seed,
              const uint16_t* __restrict__ g_val, double* __restrict__ err) {
  // the sweep needs values, not codes: its table holds the upper half of the binary32 pattern of every
  // encode-table entry's value (at most four significant bits, Inf and the quiet NaN included), so that a
  // cast costs one LDS read instead of two
  __shared__ __attribute__((aligned(16))) uint16_t val[lut_bytes<IMPL>()];
  __shared__ HrLds<uses_exp_table<IMPL>()> hrt;
  const EncCtx ctx = make_ctx<IMPL>(nullptr, hrt.w, mode, seed);
  stage_enc_lut<IMPL, SRCK, uint16_t>(val, g_val, mode);
  stage_exp_table<IMPL, SRCK>(hrt.w, mode);
  __syncthreads();

  constexpr int VE = vec_elems<SRCK>();
  constexpr int KMAX = NSC ? NSC : kSweepMax;
  const int count = NSC ? NSC : count_arg;
  const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(src);
  const size_t nvec = n >> vec_shift<SRCK>();
  double acc[KMAX];
  float sc[KMAX], isc[KMAX];
#pragma unroll
  for (int k = 0; k < KMAX; ++k) {
    acc[k] = 0.0;
    sc[k] = pow2f(k < count ? e_lo + k : 0);
    isc[k] = pow2f(k < count ? -(e_lo + k) : 0);
  }

  // one element at all scales, in stages so that the table reads of the scales are in flight
  // together: casts, then descaled values, then the fp64 accumulation
  auto score = [&](uint32_t xb, uint64_t elem) {
    const EncCtx kc = keyed<IMPL>(ctx, elem);
    const double xd = (double)__uint_as_float(xb);
    if constexpr (NSC != 0) {
      uint32_t c[KMAX], q[KMAX];
#pragma unroll
      for (int k = 0; k < KMAX; ++k) c[k] = val[table_index<IMPL, SRCK>(scaled_bits(xb, sc[k]), kc, elem)];
#pragma unroll
      for (int k = 0; k < KMAX; ++k) q[k] = scaled_bits(c[k] << 16, isc[k]);
#pragma unroll
      for (int k = 0; k < KMAX; ++k) {
        const double d = xd - (double)__uint_as_float(q[k]);
        acc[k] = fma(d, d, acc[k]);
      }
    } else {
#pragma unroll
      for (int k = 0; k < KMAX; ++k) {
        if (k < count) {  // uniform across the grid
          const uint32_t c = val[table_index<IMPL, SRCK>(scaled_bits(xb, sc[k]), kc, elem)];
          const double d = xd - (double)__uint_as_float(scaled_bits(c << 16, isc[k]));
          acc[k] = fma(d, d, acc[k]);
        }
      }
    }
  };

  const size_t stride = (size_t)gridDim.x * blockDim.x;
  size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  uint4 v = make_uint4(0u, 0u, 0u, 0u);
  if (idx < nvec) v = ld_stream(src4 + idx);
  while (idx < nvec) {
    const uint4 cur = v;
    const size_t nxt = idx + stride;
    if (nxt < nvec) v = ld_stream(src4 + nxt);  // next vector in flight while this one is scored
    const uint64_t e0 = (uint64_t)idx * VE;
    if constexpr (SRCK == kSrcF32) {
      score(cur.x, e0); score(cur.y, e0 + 1); score(cur.z, e0 + 2); score(cur.w, e0 + 3);
    } else {
      score(widen_lo<SRCK>(cur.x), e0); score(widen_hi<SRCK>(cur.x), e0 + 1);
      score(widen_lo<SRCK>(cur.y), e0 + 2); score(widen_hi<SRCK>(cur.y), e0 + 3);
      score(widen_lo<SRCK>(cur.z), e0 + 4); score(widen_hi<SRCK>(cur.z), e0 + 5);
      score(widen_lo<SRCK>(cur.w), e0 + 6); score(widen_hi<SRCK>(cur.w), e0 + 7);
    }
    idx = nxt;
  }
  const size_t t = nvec * VE + threadIdx.x;  // ragged tail, workgroup 0
  if (blockIdx.x == 0 && t < n) score(load_bits<SRCK>(src, t), t);

  block_add_f64<KMAX>(acc, count, err);
}

// element-per-lane form for sources that are not 16-byte aligned
template <int SRCK>
__global__ void __launch_bounds__(kSweepBlock)
k_scale_sweep_elem(const void* __restrict__ src, size_t n, int e_lo, int count, uint32_t mode,
                   uint64_t seed, double* __restrict__ err) {
  double acc[kSweepMax];
#pragma unroll
  for (int k = 0; k < kSweepMax; ++k) acc[k] = 0.0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const uint32_t xb = load_bits<SRCK>(src, i);
    const double xd = (double)__uint_as_float(xb);
    const uint32_t t32 = sr_threshold(seed, i);
#pragma unroll
    for (int k = 0; k < kSweepMax; ++k) {
      if (k < count) {
        const float s = pow2f(e_lo + k), inv = pow2f(-(e_lo + k));
        const uint32_t c = encode_any<SRCK>(scaled_bits(xb, s), mode, t32);
        const double d = xd - (double)__fmul_rn(__uint_as_float(decode_bits(c)), inv);
        acc[k] = fma(d, d, acc[k]);
      }
    }
  }
  block_add_f64<kSweepMax>(acc, count, err);
}

// ------------------------------------------------------------------------------------
// per-channel kernels.  Row-major [rows, cols]; axis 0: one scale per row, axis 1: one per column.
// Fast paths need 16-byte aligned bases and cols a multiple of the vector width, so that no
// 16-byte vector straddles two rows; otherwise the element kernels below do the same work.
//
// axis 0: a workgroup owns one chunk of one row (block index -> row, chunk).
// axis 1: a workgroup owns a strip of 64 * VE columns and a run of rows, its wavefronts taking
//         every fourth row; each lane keeps its VE columns (and their scales) for the whole run,
//         loads stay coalesced along rows (1 KiB per wavefront and row).
// ------------------------------------------------------------------------------------
constexpr int kAxBlock = 256;
constexpr int kAxUnroll = 4;  // axis 0: 16-byte vectors per lane per chunk
constexpr int kAxWaves = kAxBlock / 64;
constexpr int kAxRowsInFlight = 4;  // axis 1: rows loaded per lane before any is used
constexpr int kAmaxColsWaves = 8;   // axis 1 amax: wavefronts per workgroup

template <int SRCK>
__global__ void __launch_bounds__(kAxBlock)
k_amax_rows(const void* __restrict__ src, uint32_t cols_vec, uint32_t chunks, uint32_t* __restrict__ out) {
  // chunks == 1: the workgroup owns the whole row and stores its maximum (the array needs no clearing);
  // otherwise the chunks of a row meet in an atomic max on the cleared array
  const uint32_t row = blockIdx.x / chunks, chunk = blockIdx.x - row * chunks;
  const uint4* __restrict__ p = reinterpret_cast<const uint4*>(src) + (size_t)row * cols_vec;
  uint32_t m = 0;
#pragma unroll
  for (int j = 0; j < kAxUnroll; ++j) {
    const uint32_t c = (chunk * kAxUnroll + j) * kAxBlock + threadIdx.x;
    if (c < cols_vec) m = vec_amax<SRCK>(m, ld_stream(p + c));
  }
  if (chunks == 1u) {
    const uint32_t r = block_max_thread0(fold_amax<SRCK>(m));
    if (threadIdx.x == 0u) out[row] = r;
  } else {
    block_max_to_global<false>(fold_amax<SRCK>(m), out + row);  // a row has few chunks: no contention to avoid
  }
}

// columns: the wavefronts of a workgroup share a strip of 64 column vectors and take every
// WAVES-th row of the workgroup's run of rows, four rows in flight per lane; their maxima are
// combined in LDS so that only one atomic per column leaves the workgroup
template <int SRCK>
__device__ __forceinline__ uint4 colmax(const uint4& m, const uint4& v) {
  uint4 o;
  if constexpr (SRCK == kSrcF32) {
    o.x = umax(m.x, v.x & 0x7FFFFFFFu); o.y = umax(m.y, v.y & 0x7FFFFFFFu);
    o.z = umax(m.z, v.z & 0x7FFFFFFFu); o.w = umax(m.w, v.w & 0x7FFFFFFFu);
  } else {
    o.x = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, m.x), __builtin_bit_cast(u16x2_t, v.x & 0x7FFF7FFFu)));
    o.y = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, m.y), __builtin_bit_cast(u16x2_t, v.y & 0x7FFF7FFFu)));
    o.z = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, m.z), __builtin_bit_cast(u16x2_t, v.z & 0x7FFF7FFFu)));
    o.w = __builtin_bit_cast(uint32_t, __builtin_elementwise_max(__builtin_bit_cast(u16x2_t, m.w), __builtin_bit_cast(u16x2_t, v.w & 0x7FFF7FFFu)));
  }
  return o;
}

template <int SRCK, int WAVES>
__global__ void __launch_bounds__(WAVES * 64)
k_amax_cols(const void* __restrict__ src, uint32_t rows, uint32_t cols_vec, uint32_t strips,
            uint32_t rows_per_wg, uint32_t* __restrict__ out) {
  constexpr int VE = vec_elems<SRCK>();
  __shared__ uint4 part[WAVES][64];
  const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
  const uint32_t rchunk = blockIdx.x / strips, strip = blockIdx.x - rchunk * strips;
  const uint32_t cv = strip * 64u + lane;
  const bool active = cv < cols_vec;
  const uint32_t r0 = rchunk * rows_per_wg;
  const uint32_t r1 = min(rows, r0 + rows_per_wg);
  const uint4* __restrict__ p = reinterpret_cast<const uint4*>(src) + cv;
  uint4 m = make_uint4(0u, 0u, 0u, 0u);  // FP32: four magnitudes; 16-bit: eight packed 15-bit magnitudes
  if (active) {
    for (uint32_t r = r0 + wv; r < r1; r += WAVES * kAxRowsInFlight) {
      uint4 v[kAxRowsInFlight];
#pragma unroll
      for (int j = 0; j < kAxRowsInFlight; ++j) {
        const uint32_t rr = r + j * WAVES;
        v[j] = rr < r1 ? ld_stream(p + (size_t)rr * cols_vec) : make_uint4(0u, 0u, 0u, 0u);
      }
#pragma unroll
      for (int j = 0; j < kAxRowsInFlight; ++j) m = colmax<SRCK>(m, v[j]);
    }
  }
  part[wv][lane] = m;
  __syncthreads();
  if (wv != 0 || !active) return;
#pragma unroll
  for (int w = 1; w < WAVES; ++w) m = colmax<SRCK>(m, part[w][lane]);  // masks are no-ops on magnitudes
  uint32_t* o = out + (size_t)cv * VE;
  auto put = [&](int j, uint32_t bits) { if (bits) atomicMax(o + j, bits); };
  if constexpr (SRCK == kSrcF32) {
    put(0, m.x); put(1, m.y); put(2, m.z); put(3, m.w);
  } else {
    put(0, widen_lo<SRCK>(m.x)); put(1, widen_hi<SRCK>(m.x)); put(2, widen_lo<SRCK>(m.y)); put(3, widen_hi<SRCK>(m.y));
    put(4, widen_lo<SRCK>(m.z)); put(5, widen_hi<SRCK>(m.z)); put(6, widen_lo<SRCK>(m.w)); put(7, widen_hi<SRCK>(m.w));
  }
}

template <int SRCK>
__global__ void __launch_bounds__(256)
k_amax_axis_elem(const void* __restrict__ src, size_t rows, size_t cols, int axis, uint32_t* __restrict__ out) {
  const size_t n = rows * cols;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const size_t r = i / cols;
    const uint32_t a = load_bits<SRCK>(src, i) & 0x7FFFFFFFu;
    if (a) atomicMax(out + (axis == 0 ? r : i - r * cols), a);
  }
}

template <int IMPL, int SRCK>
__global__ void __launch_bounds__(kAxBlock)
k_encode_rows(const void* __restrict__ src, uint8_t* __restrict__ dst, uint32_t cols_vec, uint32_t chunks,
              const float* __restrict__ d_scale2, uint32_t mode, uint64_t seed,
              const uint8_t* __restrict__ g_lut) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[lut_bytes<IMPL>()];
  __shared__ HrLds<uses_exp_table<IMPL>()> hrt;
  const EncCtx ctx = make_ctx<IMPL>(lut, hrt.w, mode, seed);
  constexpr int VE = vec_elems<SRCK>();
  const uint32_t row = blockIdx.x / chunks, chunk = blockIdx.x - row * chunks;
  const size_t rbase = (size_t)row * cols_vec;
  const uint4* __restrict__ p = reinterpret_cast<const uint4*>(src) + rbase;
  uint4 v[kAxUnroll];
#pragma unroll
  for (int j = 0; j < kAxUnroll; ++j) {
    const uint32_t c = (chunk * kAxUnroll + j) * kAxBlock + threadIdx.x;
    if (c < cols_vec) v[j] = ld_stream(p + c);
  }
  const float scale = d_scale2[2 * (size_t)row];
  stage_enc_lut<IMPL, SRCK>(lut, g_lut, mode);
  stage_exp_table<IMPL, SRCK>(hrt.w, mode);
  __syncthreads();
#pragma unroll
  for (int j = 0; j < kAxUnroll; ++j) {
    const uint32_t c = (chunk * kAxUnroll + j) * kAxBlock + threadIdx.x;
    if (c < cols_vec) {
      const size_t idx = rbase + c;
      if constexpr (SRCK == kSrcF32)
        st_stream(reinterpret_cast<uint32_t*>(dst) + idx, encode4_f32<IMPL>(v[j], scale, ctx, idx * VE));
      else
        st_stream(reinterpret_cast<uint2*>(dst) + idx, encode8_16<IMPL, SRCK>(v[j], scale, ctx, idx * VE));
    }
  }
}

// Per-row scaling in one pass: amax of the row, its scale, and the cast, with the row held in registers
// between the two (one read of the source instead of two).  A workgroup walks rows blockIdx.x, + gridDim.x, ...;
// a lane holds VPT 16-byte vectors of the row (vector j * kQrBlock + lane index), the next row is requested
// before the current one is reduced, and one barrier per row publishes the wavefront maxima (two sets of
// slots, used alternately).  Same arithmetic as hif8_amax_axis + hif8_scale_from_amax_n + hif8_encode_axis
// with axis 0: d_amax[row] and d_scale2[2 row], [2 row + 1] receive the same values.
constexpr int kQrBlock = 512;
constexpr int kQrWaves = kQrBlock / 64;

template <int IMPL, int SRCK, int VPT>
__global__ void __launch_bounds__(kQrBlock)
k_quant_rows(const void* __restrict__ src, uint8_t* __restrict__ dst, uint32_t rows, uint32_t cols_vec, float target,
             int pow2, uint32_t* __restrict__ d_amax, float* __restrict__ d_scale2, uint32_t mode, uint64_t seed,
             const uint8_t* __restrict__ g_lut) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[lut_bytes<IMPL>()];
  __shared__ HrLds<uses_exp_table<IMPL>()> hrt;
  __shared__ uint32_t part[2][kQrWaves];
  const EncCtx ctx = make_ctx<IMPL>(lut, hrt.w, mode, seed);
  constexpr int VE = vec_elems<SRCK>();
  const uint4* __restrict__ src4 = reinterpret_cast<const uint4*>(src);
  const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
  uint4 nxt[VPT];
  auto request = [&](uint32_t r) {
    const uint4* __restrict__ p = src4 + (size_t)r * cols_vec;
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
      const uint32_t c = j * kQrBlock + threadIdx.x;
      nxt[j] = c < cols_vec ? ld_stream(p + c) : make_uint4(0u, 0u, 0u, 0u);
    }
  };
  uint32_t r = blockIdx.x;  // uniform over the workgroup, as is every branch on it
  if (r < rows) request(r);
  stage_enc_lut<IMPL, SRCK>(lut, g_lut, mode);
  stage_exp_table<IMPL, SRCK>(hrt.w, mode);
  for (uint32_t it = 0; r < rows; r += gridDim.x, ++it) {
    uint4 cur[VPT];
    uint32_t m = 0;
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
      cur[j] = nxt[j];
      m = vec_amax<SRCK>(m, cur[j]);  // vectors past the row are zeros
    }
    m = wave_max_u32(fold_amax<SRCK>(m));
    if (lane == 0u) part[it & 1u][wv] = m;
    if (r + gridDim.x < rows) request(r + gridDim.x);
    __syncthreads();  // also orders the table staging before the first row's lookups
    uint32_t a = part[it & 1u][0];
#pragma unroll
    for (int w = 1; w < kQrWaves; ++w) a = umax(a, part[it & 1u][w]);
    const float scale = scale_from_amax_value(__uint_as_float(a), target, pow2);
    if (threadIdx.x == 0u) {
      d_amax[r] = a;
      d_scale2[2 * (size_t)r] = scale;
      d_scale2[2 * (size_t)r + 1] = 1.0f / scale;
    }
    const size_t rbase = (size_t)r * cols_vec;
#pragma unroll
    for (int j = 0; j < VPT; ++j) {
      const uint32_t c = j * kQrBlock + threadIdx.x;
      if (c < cols_vec) {
        const size_t idx = rbase + c;
        if constexpr (SRCK == kSrcF32)
          st_stream(reinterpret_cast<uint32_t*>(dst) + idx, encode4_f32<IMPL>(cur[j], scale, ctx, idx * VE));
        else
          st_stream(reinterpret_cast<uint2*>(dst) + idx, encode8_16<IMPL, SRCK>(cur[j], scale, ctx, idx * VE));
      }
    }
  }
}

template <int IMPL, int SRCK>
__global__ void __launch_bounds__(kAxBlock)
k_encode_cols(const void* __restrict__ src, uint8_t* __restrict__ dst, uint32_t rows, uint32_t cols_vec,
              uint32_t strips, uint32_t rows_per_wg, const float* __restrict__ d_scale2, uint32_t mode,
              uint64_t seed, const uint8_t* __restrict__ g_lut) {
  __shared__ __attribute__((aligned(16))) uint8_t lut[lut_bytes<IMPL>()];
  __shared__ HrLds<uses_exp_table<IMPL>()> hrt;
  const EncCtx ctx = make_ctx<IMPL>(lut, hrt.w, mode, seed);
  stage_enc_lut<IMPL, SRCK>(lut, g_lut, mode);
  stage_exp_table<IMPL, SRCK>(hrt.w, mode);
  __syncthreads();
  constexpr int VE = vec_elems<SRCK>();
  const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
  const uint32_t rchunk = blockIdx.x / strips, strip = blockIdx.x - rchunk * strips;
  const uint32_t cv = strip * 64u + lane;
  if (cv >= cols_vec) return;
  float sc[VE];
#pragma unroll
  for (int j = 0; j < VE; ++j) sc[j] = d_scale2[2 * ((size_t)cv * VE + j)];
  const uint32_t r0 = rchunk * rows_per_wg;
  const uint32_t r1 = min(rows, r0 + rows_per_wg);
  const uint4* __restrict__ p = reinterpret_cast<const uint4*>(src) + cv;
  auto encode_row = [&](uint32_t r, const uint4& v) {
    const size_t idx = (size_t)r * cols_vec + cv;
    const uint64_t e0 = (uint64_t)idx * VE;
    const EncCtx kc = keyed<IMPL>(ctx, e0);
    if constexpr (SRCK == kSrcF32) {
      const uint32_t c0 = encode_one<IMPL, SRCK>(scaled_bits(v.x, sc[0]), kc, e0);
      const uint32_t c1 = encode_one<IMPL, SRCK>(scaled_bits(v.y, sc[1]), kc, e0 + 1);
      const uint32_t c2 = encode_one<IMPL, SRCK>(scaled_bits(v.z, sc[2]), kc, e0 + 2);
      const uint32_t c3 = encode_one<IMPL, SRCK>(scaled_bits(v.w, sc[3]), kc, e0 + 3);
      st_stream(reinterpret_cast<uint32_t*>(dst) + idx, c0 | (c1 << 8) | (c2 << 16) | (c3 << 24));
    } else {
      const uint32_t w[4] = {v.x, v.y, v.z, v.w};
      uint32_t o[2] = {0u, 0u};
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        const uint32_t c0 = encode_one<IMPL, SRCK>(scaled_bits(widen_lo<SRCK>(w[j]), sc[2 * j]), kc, e0 + 2 * j);
        const uint32_t c1 = encode_one<IMPL, SRCK>(scaled_bits(widen_hi<SRCK>(w[j]), sc[2 * j + 1]), kc, e0 + 2 * j + 1);
        o[j >> 1] |= (c0 | (c1 << 8)) << (16 * (j & 1));
      }
      st_stream(reinterpret_cast<uint2*>(dst) + idx, make_uint2(o[0], o[1]));
    }
  };
  for (uint32_t r = r0 + wv; r < r1; r += kAxWaves * kAxRowsInFlight) {
    uint4 v[kAxRowsInFlight];
#pragma unroll
    for (int j = 0; j < kAxRowsInFlight; ++j) {
      const uint32_t rr = r + j * kAxWaves;
      if (rr < r1) v[j] = ld_stream(p + (size_t)rr * cols_vec);
    }
#pragma unroll
    for (int j = 0; j < kAxRowsInFlight; ++j) {
      const uint32_t rr = r + j * kAxWaves;
      if (rr < r1) encode_row(rr, v[j]);
    }
  }
}

template <int SRCK>
__global__ void __launch_bounds__(256)
k_encode_axis_elem(const void* __restrict__ src, uint8_t* __restrict__ dst, size_t rows, size_t cols, int axis,
                   const float* __restrict__ d_scale2, uint32_t mode, uint64_t seed) {
  const size_t n = rows * cols;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const size_t r = i / cols;
    const float scale = d_scale2[2 * (axis == 0 ? r : i - r * cols)];
    dst[i] = (uint8_t)encode_any<SRCK>(scaled_bits(load_bits<SRCK>(src, i), scale), mode, sr_threshold(seed, i));
  }
}

// decode: one lane's worth of codes (VE of them) -> one 16-byte vector of DSTK values
template <int DSTK>
__global__ void __launch_bounds__(kAxBlock)
k_decode_rows(const uint8_t* __restrict__ src, void* __restrict__ dst, uint32_t cols_vec, uint32_t chunks,
              const float* __restrict__ d_scale2, const uint32_t* __restrict__ g_dec) {
  __shared__ uint32_t dec[256];
  stage_dec_lut(dec, g_dec);
  __syncthreads();
  const uint32_t row = blockIdx.x / chunks, chunk = blockIdx.x - row * chunks;
  const size_t rbase = (size_t)row * cols_vec;
  const float inv = d_scale2[2 * (size_t)row + 1];
  uint4* __restrict__ d4 = reinterpret_cast<uint4*>(dst);
#pragma unroll
  for (int j = 0; j < kAxUnroll; ++j) {
    const uint32_t c = (chunk * kAxUnroll + j) * kAxBlock + threadIdx.x;
    if (c < cols_vec) {
      const size_t idx = rbase + c;
      if constexpr (DSTK == kSrcF32)
        st_stream(d4 + idx, descale4_f32(ld_stream(reinterpret_cast<const uint32_t*>(src) + idx), dec, inv));
      else
        st_stream(d4 + idx, descale8_16<DSTK>(ld_stream(reinterpret_cast<const uint2*>(src) + idx), dec, inv));
    }
  }
}

template <int DSTK>
__global__ void __launch_bounds__(kAxBlock)
k_decode_cols(const uint8_t* __restrict__ src, void* __restrict__ dst, uint32_t rows, uint32_t cols_vec,
              uint32_t strips, uint32_t rows_per_wg, const float* __restrict__ d_scale2,
              const uint32_t* __restrict__ g_dec) {
  __shared__ uint32_t dec[256];
  stage_dec_lut(dec, g_dec);
  __syncthreads();
  constexpr int VE = vec_elems<DSTK>();
  const uint32_t lane = threadIdx.x & 63u, wv = threadIdx.x >> 6;
  const uint32_t rchunk = blockIdx.x / strips, strip = blockIdx.x - rchunk * strips;
  const uint32_t cv = strip * 64u + lane;
  if (cv >= cols_vec) return;
  float inv[VE];
#pragma unroll
  for (int j = 0; j < VE; ++j) inv[j] = d_scale2[2 * ((size_t)cv * VE + j) + 1];
  const uint32_t r0 = rchunk * rows_per_wg;
  const uint32_t r1 = min(rows, r0 + rows_per_wg);
  uint4* __restrict__ d4 = reinterpret_cast<uint4*>(dst);
  for (uint32_t r = r0 + wv; r < r1; r += kAxWaves * kAxRowsInFlight) {
    uint2 w[kAxRowsInFlight];
#pragma unroll
    for (int j = 0; j < kAxRowsInFlight; ++j) {
      const uint32_t rr = r + j * kAxWaves;
      if (rr < r1) {
        const size_t idx = (size_t)rr * cols_vec + cv;
        if constexpr (DSTK == kSrcF32) w[j] = make_uint2(ld_stream(reinterpret_cast<const uint32_t*>(src) + idx), 0u);
        else w[j] = ld_stream(reinterpret_cast<const uint2*>(src) + idx);
      }
    }
#pragma unroll
    for (int j = 0; j < kAxRowsInFlight; ++j) {
      const uint32_t rr = r + j * kAxWaves;
      if (rr < r1) {
        const size_t idx = (size_t)rr * cols_vec + cv;
        uint4 o;
        if constexpr (DSTK == kSrcF32) {
          o.x = descale_bits(w[j].x, dec, inv[0]);
          o.y = descale_bits(w[j].x >> 8, dec, inv[1]);
          o.z = descale_bits(w[j].x >> 16, dec, inv[2]);
          o.w = descale_bits(w[j].x >> 24, dec, inv[3]);
        } else {
          o.x = narrow2<DSTK>(descale_bits(w[j].x, dec, inv[0]), descale_bits(w[j].x >> 8, dec, inv[1]));
          o.y = narrow2<DSTK>(descale_bits(w[j].x >> 16, dec, inv[2]), descale_bits(w[j].x >> 24, dec, inv[3]));
          o.z = narrow2<DSTK>(descale_bits(w[j].y, dec, inv[4]), descale_bits(w[j].y >> 8, dec, inv[5]));
          o.w = narrow2<DSTK>(descale_bits(w[j].y >> 16, dec, inv[6]), descale_bits(w[j].y >> 24, dec, inv[7]));
        }
        st_stream(d4 + idx, o);
      }
    }
  }
}

template <int DSTK>
__global__ void __launch_bounds__(256)
k_decode_axis_elem(const uint8_t* __restrict__ src, void* __restrict__ dst, size_t rows, size_t cols, int axis,
                   const float* __restrict__ d_scale2) {
  const size_t n = rows * cols;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) {
    const size_t r = i / cols;
    const float inv = d_scale2[2 * (axis == 0 ? r : i - r * cols) + 1];
    const uint32_t b = __float_as_uint(__fmul_rn(__uint_as_float(decode_bits(src[i])), inv));
    if constexpr (DSTK == kSrcF32) reinterpret_cast<uint32_t*>(dst)[i] = b;
    else reinterpret_cast<uint16_t*>(dst)[i] = (uint16_t)narrow1<DSTK>(b);
  }
}

// ====================================================================================
// host side
// ====================================================================================
template <typename F>
void dispatch_impl_only(int impl, F&& f) {
  using std::integral_constant;
  switch (impl) {
    case IMPL_HR: f(integral_constant<int, IMPL_HR>{}); break;
    case IMPL_TE: f(integral_constant<int, IMPL_TE>{}); break;
    case IMPL_SR: f(integral_constant<int, IMPL_SR>{}); break;
    default: f(integral_constant<int, IMPL_TA_LUT>{}); break;
  }
}
// the sweep and the per-channel kernels stage their tables for little data per workgroup: they keep the
// small per-exponent tables for HR whatever the source kind
inline int impl_no_alu(uint32_t mode) {
  const int i = impl_for<kSrcF32>(mode);
  return i == IMPL_TA_ALU ? IMPL_TA_LUT : i;
}

template <int SRCK>
hif8_status scale_sweep(const void* src, size_t n, int e_lo, int count, uint32_t mode, double* d_err,
                        hipStream_t st) {
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  if (count < 1 || count > kSweepMax || e_lo < -126 || e_lo + count - 1 > 126) return HIF8_ERR_ARG;
  if (!d_err || (!src && n != 0)) return HIF8_ERR_NULL;
  if (!aligned_to(d_err, 8)) return HIF8_ERR_ARG;  // fp64 atomics need naturally aligned doubles
  int cus = 0;
  DevTables tb;
  hif8_status s = ensure_init(&cus, &tb);
  if (s != HIF8_OK) return s;
  s = launch_fill_u32(reinterpret_cast<uint32_t*>(d_err), 0u, 2u * (uint32_t)count, st);
  if (s != HIF8_OK || n == 0) return s;
  const uint64_t seed = sr_seed();
  if (!aligned_to(src, 16)) {
    hipLaunchKernelGGL(k_scale_sweep_elem<SRCK>, dim3(grid_elem(n, cus)), dim3(kSweepBlock), 0, st, src, n,
                       e_lo, count, mode, seed, d_err);
    return finish_launch();
  }
  const size_t nvec = n >> vec_shift<SRCK>();
  hif8_status rc = HIF8_OK;
  dispatch_impl_only(impl_no_alu(mode), [&](auto impl_c) {
    constexpr int IMPL = decltype(impl_c)::value;
    size_t wgs = (nvec + kSweepBlock - 1) / kSweepBlock;
    const size_t cap = (size_t)cus * 8;  // grid-stride: a few workgroups per CU
    if (wgs > cap) wgs = cap;
    if (wgs == 0) wgs = 1;
    // the paper's search range (10 scales) gets straight-line code; other counts a run-time bound
    if (count == 10)
      hipLaunchKernelGGL((k_scale_sweep<IMPL, SRCK, 10>), dim3((unsigned)wgs), dim3(kSweepBlock), 0, st, src, n,
                         e_lo, count, mode, seed, tb.val_lut, d_err);
    else
      hipLaunchKernelGGL((k_scale_sweep<IMPL, SRCK, 0>), dim3((unsigned)wgs), dim3(kSweepBlock), 0, st, src, n,
                         e_lo, count, mode, seed, tb.val_lut, d_err);
  });
  return rc != HIF8_OK ? rc : finish_launch();
}

struct AxisPlan {
  bool fast;
  uint32_t cols_vec, chunks, strips, rows_per_wg, row_chunks;
};

// shapes of the per-channel launches; sizes are limited to what 32-bit row / vector counts hold
template <int KIND>
bool plan_axis(size_t rows, size_t cols, int cus, bool aligned, AxisPlan* p) {
  constexpr size_t VE = vec_elems<KIND>();
  if (rows > 0x7FFFFFFFu || cols > 0x7FFFFFFFu) return false;
  p->fast = aligned && (cols % VE) == 0;
  p->cols_vec = (uint32_t)(cols / VE);
  const uint32_t per_chunk = kAxBlock * kAxUnroll;
  p->chunks = (p->cols_vec + per_chunk - 1) / per_chunk;
  p->strips = (p->cols_vec + 63) / 64;
  // axis 1: enough row chunks to give every CU about three workgroups, at least 64 rows each (every
  // lane loads the scales of its columns once per workgroup; measured on [11008, 4096] and [32000, 4096]
  // BF16 and [8192, 8192] FP32: three per CU beat six by 5-12 %), in multiples of what the lanes keep in flight
  uint32_t want = (uint32_t)((size_t)cus * 3 / (p->strips ? p->strips : 1));
  if (want < 1) want = 1;
  uint32_t rpw = (uint32_t)((rows + want - 1) / want);
  if (rpw < 64) rpw = 64;
  rpw = (rpw + kAxWaves * kAxRowsInFlight - 1) / (kAxWaves * kAxRowsInFlight) * (kAxWaves * kAxRowsInFlight);
  p->rows_per_wg = rpw;
  p->row_chunks = (uint32_t)((rows + rpw - 1) / rpw);
  if ((uint64_t)rows * p->chunks > 0x7FFFFFFFull || (uint64_t)p->row_chunks * p->strips > 0x7FFFFFFFull) return false;
  return true;
}

template <int SRCK>
hif8_status amax_axis(const void* src, size_t rows, size_t cols, int axis, float* d_amax, hipStream_t st) {
  if (axis != 0 && axis != 1) return HIF8_ERR_ARG;
  const size_t nch = axis == 0 ? rows : cols;
  if (nch == 0) return HIF8_OK;
  if (!d_amax || (!src && rows * cols != 0)) return HIF8_ERR_NULL;
  int cus = 0;
  hif8_status s = ensure_init(&cus, nullptr);
  if (s != HIF8_OK) return s;
  AxisPlan p;
  if (!plan_axis<SRCK>(rows, cols, cus, aligned_to(src, 16), &p)) return HIF8_ERR_ARG;
  uint32_t* out = reinterpret_cast<uint32_t*>(d_amax);
  const bool stores = p.fast && axis == 0 && p.chunks == 1 && rows * cols != 0;  // k_amax_rows writes every row itself
  if (!stores) {
    s = launch_fill_u32(out, 0u, (uint32_t)nch, st);
    if (s != HIF8_OK || rows * cols == 0) return s;
  }
  if (!p.fast) {
    hipLaunchKernelGGL(k_amax_axis_elem<SRCK>, dim3(grid_elem(rows * cols, cus)), dim3(256), 0, st, src, rows, cols, axis, out);
  } else if (axis == 0) {
    hipLaunchKernelGGL(k_amax_rows<SRCK>, dim3((unsigned)(rows * p.chunks)), dim3(kAxBlock), 0, st, src, p.cols_vec, p.chunks, out);
  } else {
    // longer runs of rows than the casts use -- about one workgroup per CU -- because every
    // workgroup ends with one atomic per column (measured on [11008, 4096] BF16: 50 us with 64-row
    // runs, 25 us with 384-row runs, 50 us again with 1024-row runs that leave most CUs idle), and
    // eight wavefronts per workgroup so that a CU still has enough loads in flight (20 us; four
    // wavefronts 24 us, sixteen no better)
    const uint32_t unit = kAmaxColsWaves * kAxRowsInFlight;
    uint32_t want_chunks = (uint32_t)cus / (p.strips ? p.strips : 1u);
    if (want_chunks < 1u) want_chunks = 1u;
    uint32_t rpw = (uint32_t)((rows + want_chunks - 1) / want_chunks);
    rpw = (rpw + unit - 1) / unit * unit;
    if (rpw < 64u) rpw = 64u;
    const uint32_t row_chunks = (uint32_t)((rows + rpw - 1) / rpw);
    hipLaunchKernelGGL((k_amax_cols<SRCK, kAmaxColsWaves>), dim3(row_chunks * p.strips), dim3(kAmaxColsWaves * 64), 0,
                       st, src, (uint32_t)rows, p.cols_vec, p.strips, rpw, out);
  }
  return finish_launch();
}

template <int SRCK>
hif8_status encode_axis(const void* src, uint8_t* dst, size_t rows, size_t cols, int axis, const float* d_scale2,
                        uint32_t mode, hipStream_t st) {
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  if (axis != 0 && axis != 1) return HIF8_ERR_ARG;
  if (rows * cols == 0) return HIF8_OK;
  if (!src || !dst || !d_scale2) return HIF8_ERR_NULL;
  int cus = 0;
  DevTables tb;
  hif8_status s = ensure_init(&cus, &tb);
  if (s != HIF8_OK) return s;
  AxisPlan p;
  const bool al = aligned_to(src, 16) && aligned_to(dst, SRCK == kSrcF32 ? 4 : 8);
  if (!plan_axis<SRCK>(rows, cols, cus, al, &p)) return HIF8_ERR_ARG;
  const uint64_t seed = sr_seed();
  if (!p.fast) {
    hipLaunchKernelGGL(k_encode_axis_elem<SRCK>, dim3(grid_elem(rows * cols, cus)), dim3(256), 0, st, src, dst, rows,
                       cols, axis, d_scale2, mode, seed);
    return finish_launch();
  }
  dispatch_impl_only(impl_no_alu(mode), [&](auto impl_c) {
    constexpr int IMPL = decltype(impl_c)::value;
    if (axis == 0)
      hipLaunchKernelGGL((k_encode_rows<IMPL, SRCK>), dim3((unsigned)(rows * p.chunks)), dim3(kAxBlock), 0, st, src,
                         dst, p.cols_vec, p.chunks, d_scale2, mode, seed, tb.enc_lut);
    else
      hipLaunchKernelGGL((k_encode_cols<IMPL, SRCK>), dim3(p.row_chunks * p.strips), dim3(kAxBlock), 0, st, src, dst,
                         (uint32_t)rows, p.cols_vec, p.strips, p.rows_per_wg, d_scale2, mode, seed, tb.enc_lut);
  });
  return finish_launch();
}

// Fused per-row path when a row fits the registers of one workgroup and the fast-path alignment holds;
// otherwise the three separate launches (same results).
template <int SRCK>
hif8_status quantize_rows(const void* src, uint8_t* dst, size_t rows, size_t cols, float target, int pow2, uint32_t mode,
                          float* d_amax, float* d_scale2, hipStream_t st) {
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  if (!(target > 0.0f) || std::isinf(target)) return HIF8_ERR_ARG;
  if (rows == 0) return HIF8_OK;
  if (!d_amax || !d_scale2 || (rows * cols != 0 && (!src || !dst))) return HIF8_ERR_NULL;
  if (rows > 0x7FFFFFFFu || cols > 0x7FFFFFFFu) return HIF8_ERR_ARG;
  int cus = 0;
  DevTables tb;
  hif8_status s = ensure_init(&cus, &tb);
  if (s != HIF8_OK) return s;
  constexpr size_t VE = vec_elems<SRCK>();
  const bool al = aligned_to(src, 16) && aligned_to(dst, SRCK == kSrcF32 ? 4 : 8);
  const size_t cols_vec = cols / VE;
  if (!al || cols == 0 || (cols % VE) != 0 || cols_vec > (size_t)kQrBlock * 8) {
    s = amax_axis<SRCK>(src, rows, cols, 0, d_amax, st);
    if (s != HIF8_OK) return s;
    s = hif8host::launch_scale_from_amax(d_amax, d_scale2, (uint32_t)rows, target, pow2, st);
    if (s != HIF8_OK) return s;
    return encode_axis<SRCK>(src, dst, rows, cols, 0, d_scale2, mode, st);
  }
  const uint64_t seed = sr_seed();
  // enough workgroups to fill the chip (four of 512 lanes per CU), each walking several rows (measured flat from 3 to 8 per CU)
  size_t wgs = (size_t)cus * 4;
  if (wgs > rows) wgs = rows;
  const int vpt = cols_vec <= (size_t)kQrBlock ? 1 : cols_vec <= (size_t)kQrBlock * 2 ? 2 : cols_vec <= (size_t)kQrBlock * 4 ? 4 : 8;
  uint32_t* am = reinterpret_cast<uint32_t*>(d_amax);
  dispatch_impl_only(impl_no_alu(mode), [&](auto impl_c) {
    constexpr int IMPL = decltype(impl_c)::value;
    auto go = [&](auto vpt_c) {
      constexpr int VPT = decltype(vpt_c)::value;
      hipLaunchKernelGGL((k_quant_rows<IMPL, SRCK, VPT>), dim3((unsigned)wgs), dim3(kQrBlock), 0, st, src, dst, (uint32_t)rows,
                         (uint32_t)cols_vec, target, pow2, am, d_scale2, mode, seed, tb.enc_lut);
    };
    using std::integral_constant;
    if (vpt == 1) go(integral_constant<int, 1>{});
    else if (vpt == 2) go(integral_constant<int, 2>{});
    else if (vpt == 4) go(integral_constant<int, 4>{});
    else go(integral_constant<int, 8>{});
  });
  return finish_launch();
}

template <int DSTK>
hif8_status decode_axis(const uint8_t* src, void* dst, size_t rows, size_t cols, int axis, const float* d_scale2,
                        hipStream_t st) {
  if (axis != 0 && axis != 1) return HIF8_ERR_ARG;
  if (rows * cols == 0) return HIF8_OK;
  if (!src || !dst || !d_scale2) return HIF8_ERR_NULL;
  int cus = 0;
  DevTables tb;
  hif8_status s = ensure_init(&cus, &tb);
  if (s != HIF8_OK) return s;
  AxisPlan p;
  const bool al = aligned_to(dst, 16) && aligned_to(src, DSTK == kSrcF32 ? 4 : 8);
  if (!plan_axis<DSTK>(rows, cols, cus, al, &p)) return HIF8_ERR_ARG;
  if (!p.fast) {
    hipLaunchKernelGGL(k_decode_axis_elem<DSTK>, dim3(grid_elem(rows * cols, cus)), dim3(256), 0, st, src, dst, rows,
                       cols, axis, d_scale2);
  } else if (axis == 0) {
    hipLaunchKernelGGL(k_decode_rows<DSTK>, dim3((unsigned)(rows * p.chunks)), dim3(kAxBlock), 0, st, src, dst,
                       p.cols_vec, p.chunks, d_scale2, tb.dec_lut);
  } else {
    hipLaunchKernelGGL(k_decode_cols<DSTK>, dim3(p.row_chunks * p.strips), dim3(kAxBlock), 0, st, src, dst,
                       (uint32_t)rows, p.cols_vec, p.strips, p.rows_per_wg, d_scale2, tb.dec_lut);
  }
  return finish_launch();
}

}  // namespace hif8calib

using namespace hif8calib;
using hif8dev::kSrcBF16;
using hif8dev::kSrcF16;
using hif8dev::kSrcF32;

extern "C" {

hif8_status hif8_scale_from_amax_n(const float* d_amax, float* d_scale2, size_t count, float target, int pow2,
                                   hif8_stream_t stream) {
  if (count == 0) return HIF8_OK;
  if (!d_amax || !d_scale2) return HIF8_ERR_NULL;
  if (!(target > 0.0f) || std::isinf(target) || count > 0x7FFFFFFFu) return HIF8_ERR_ARG;
  return hif8host::launch_scale_from_amax(d_amax, d_scale2, (uint32_t)count, target, pow2, (hipStream_t)stream);
}

#define HIF8_DEFINE_CALIB(SFX, T, K)                                                                          \
  hif8_status hif8_scale_sweep_##SFX(const T* src, size_t n, int e_lo, int count, uint32_t mode,              \
                                     double* d_err, hif8_stream_t stream) {                                   \
    return scale_sweep<K>(src, n, e_lo, count, mode, d_err, (hipStream_t)stream);                             \
  }                                                                                                           \
  hif8_status hif8_amax_axis_##SFX(const T* src, size_t rows, size_t cols, int axis, float* d_amax,           \
                                   hif8_stream_t stream) {                                                    \
    return amax_axis<K>(src, rows, cols, axis, d_amax, (hipStream_t)stream);                                  \
  }                                                                                                           \
  hif8_status hif8_encode_axis_##SFX(const T* src, uint8_t* dst, size_t rows, size_t cols, int axis,          \
                                     const float* d_scale2, uint32_t mode, hif8_stream_t stream) {            \
    return encode_axis<K>(src, dst, rows, cols, axis, d_scale2, mode, (hipStream_t)stream);                   \
  }                                                                                                           \
  hif8_status hif8_decode_axis_##SFX(const uint8_t* src, T* dst, size_t rows, size_t cols, int axis,          \
                                     const float* d_scale2, hif8_stream_t stream) {                           \
    return decode_axis<K>(src, dst, rows, cols, axis, d_scale2, (hipStream_t)stream);                         \
  }                                                                                                           \
  hif8_status hif8_quantize_rows_##SFX(const T* src, uint8_t* dst, size_t rows, size_t cols, float target,    \
                                       int pow2, uint32_t mode, float* d_amax, float* d_scale2,               \
                                       hif8_stream_t stream) {                                                \
    return quantize_rows<K>(src, dst, rows, cols, target, pow2, mode, d_amax, d_scale2, (hipStream_t)stream); \
  }

HIF8_DEFINE_CALIB(f32, float, kSrcF32)
HIF8_DEFINE_CALIB(bf16, uint16_t, kSrcBF16)
HIF8_DEFINE_CALIB(f16, uint16_t, kSrcF16)
#undef HIF8_DEFINE_CALIB

}  // extern "C"
