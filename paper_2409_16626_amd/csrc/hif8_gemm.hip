// Simulated HiF8 GEMM on the matrix cores of gfx950, and Algorithm 1's per-layer scale search.
//
// The paper's experiments cast the GEMM inputs (activations, weights, activation gradients) to
// HiF8 and run the GEMM on the represented values (Sec. 4, Sec. 5); Algorithm 1 ("MatMul &
// Restore") descales the product by the two input scales.  Every HiF8 value is exact in
// bfloat16 (at most 3 mantissa bits, exponents -22..15), so the product is computed with bf16
// MFMA instructions and FP32 accumulation; the u8 codes are expanded to bf16 on their way from
// HBM into LDS (one table lookup per element, table replicated per LDS bank so that lookups of a
// wavefront never conflict), which halves the operand traffic against a bf16 GEMM.
//
//   O[M, N] = (value(A[M, K]) x value(B[N, K])^T) * descale        (both operands K-contiguous)
//
// Tiling: a workgroup of WM x WN wavefronts owns a (WM TM 32) x (WN TN 32) tile of O; each
// wavefront TM x TN blocks of v_mfma_f32_32x32x16_bf16; K advances in steps of BK through a
// double-buffered LDS tile, with the next tile's codes in flight in registers during the MFMAs.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <mutex>

#include "hif8.h"
#include "hif8_diag.h"
#include "hif8_conv_api.hpp"
#include "hif8_device.hpp"
#include "hif8_gemm_common.hpp"
#include "hif8_host.hpp"

namespace hif8gemm {

using namespace hif8dev;
using namespace hif8host;

typedef uint16_t u16x2 __attribute__((ext_vector_type(2)));

#ifndef HIF8_GEMM_PAD
#define HIF8_GEMM_PAD 8
#endif
constexpr int kPad = HIF8_GEMM_PAD;  // bf16 elements of padding per LDS row
constexpr int kLutCopies = 32;    // one copy of the code -> bf16 table per LDS bank

// code -> bfloat16 pattern (the top half of the binary32 pattern; exact for every code)
static __device__ __attribute__((aligned(16))) uint16_t g_bf16_lut[256];
__global__ void k_build_gemm_lut() {
  const uint32_t i = threadIdx.x;
  if (i < 256u) g_bf16_lut[i] = (uint16_t)(decode_bits(i) >> 16);
}

// 16 codes (one 16-byte chunk) -> 16 bf16, written to LDS as two 16-byte stores.
// lut16: this lane's column of the replicated table, indexed by code * (2 * kLutCopies).
__device__ __forceinline__ void decode_chunk_to_lds(const uint4& c, const uint16_t* lut16, uint4* dst) {
  const uint32_t w[4] = {c.x, c.y, c.z, c.w};
  uint32_t o[8];
#pragma unroll
  for (int j = 0; j < 4; ++j) {
    u16x2 p0, p1;
    p0.x = lut16[(w[j] & 0xFFu) * (2 * kLutCopies)];
    p0.y = lut16[((w[j] >> 8) & 0xFFu) * (2 * kLutCopies)];
    p1.x = lut16[((w[j] >> 16) & 0xFFu) * (2 * kLutCopies)];
    p1.y = lut16[(w[j] >> 24) * (2 * kLutCopies)];
    o[2 * j] = __builtin_bit_cast(uint32_t, p0);
    o[2 * j + 1] = __builtin_bit_cast(uint32_t, p1);
  }
  dst[0] = make_uint4(o[0], o[1], o[2], o[3]);
  dst[1] = make_uint4(o[4], o[5], o[6], o[7]);
}

// 16 codes of row `row` at column k; rows / columns outside the matrix read as zero codes.  The
// address is clamped instead of branching so that the loop body stays one basic block.
__device__ __forceinline__ uint4 load_chunk(const uint8_t* __restrict__ P, uint32_t row, uint32_t rows,
                                            uint32_t k, uint32_t K) {
  const bool ok = row < rows && k < K;
  const uint4 v = *reinterpret_cast<const uint4*>(P + (size_t)(ok ? row : 0u) * K + (ok ? k : 0u));
  return ok ? v : make_uint4(0u, 0u, 0u, 0u);
}

template <int WM, int WN, int TM, int TN, int BK, int EPI>
__global__ void __launch_bounds__(64 * WM * WN)
k_gemm_nt(const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, void* __restrict__ out,
          const float* __restrict__ ref, double* __restrict__ err, uint32_t M, uint32_t N, uint32_t K,
          float descale, const uint16_t* __restrict__ g_lut, uint32_t tiles_n, uint32_t col_begin, Batch batch) {
  // batched form (the scale search of Algorithm 1): blockIdx.y = pair (i, j) of code matrices
  if (batch.nb != 0u) {
    const uint32_t bi = blockIdx.y / batch.nb, bj = blockIdx.y - bi * batch.nb;
    A += (size_t)bi * batch.a_stride;
    B += (size_t)bj * batch.b_stride;
    err += blockIdx.y;
    descale = pow2f(-(batch.e_base + (int)bi + (int)bj));
  }
  constexpr int kThreads = 64 * WM * WN;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr int LDA = BK + kPad;                       // LDS row stride in bf16
  constexpr int CPR = BK / 16;                         // 16-code chunks per tile row
  constexpr int CA = BM * CPR / kThreads, CB = BN * CPR / kThreads;  // chunks per thread
  static_assert(BM * CPR % kThreads == 0 && BN * CPR % kThreads == 0, "tile / thread mismatch");

  extern __shared__ __attribute__((aligned(16))) uint8_t smem[];
  uint32_t* lut32 = reinterpret_cast<uint32_t*>(smem);                     // [256][kLutCopies]
  __bf16* As = reinterpret_cast<__bf16*>(smem + 256 * kLutCopies * 4);     // [2][BM][LDA]
  __bf16* Bs = As + 2 * BM * LDA;                                          // [2][BN][LDA]

  const uint32_t tid = threadIdx.x, lane = tid & 63u, wave = tid >> 6;
  const uint32_t wm = wave / WN, wn = wave % WN;
  const uint32_t tile_m = blockIdx.x / tiles_n, tile_n = blockIdx.x - tile_m * tiles_n;
  const uint32_t m0 = tile_m * BM, n0 = col_begin + tile_n * BN;  // the launch covers columns from col_begin on

  // replicated table: entry (code, copy) at dword code * 32 + copy; lane l reads copy l % 32
  for (uint32_t i = tid; i < 256u * kLutCopies; i += kThreads) {
    const uint32_t v = g_lut[i / kLutCopies];
    lut32[i] = v | (v << 16);
  }
  const uint16_t* lut16 = reinterpret_cast<const uint16_t*>(lut32) + 2 * (lane & (kLutCopies - 1));

  // this thread's chunks of the A and B tiles.  Chunk q -> (row, 16-code column): 8 consecutive
  // lanes take 8 consecutive rows of the same column, so that their 16-byte LDS stores (row
  // stride 16 bytes more than a power of two) fall into 8 different groups of 4 banks; the lanes
  // 8 apart take the neighbouring columns, so a wavefront still loads whole 16 * CPR byte runs.
  auto chunk_row = [](uint32_t q) { return 8u * (q / (8u * CPR)) + (q & 7u); };
  auto chunk_col = [](uint32_t q) { return (q >> 3) % CPR; };
  // Two register sets: one holds the codes of the tile being expanded into LDS during this K step,
  // the other receives the loads for the tile after it, so a load has a whole K step to arrive.
  uint4 ra[2][CA], rb[2][CB];
  auto load_tiles = [&](int set, uint32_t k0) {
#pragma unroll
    for (int i = 0; i < CA; ++i) {
      const uint32_t q = tid + i * kThreads, r = chunk_row(q), kc = chunk_col(q);
      ra[set][i] = load_chunk(A, m0 + r, M, k0 + kc * 16, K);
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) {
      const uint32_t q = tid + i * kThreads, r = chunk_row(q), kc = chunk_col(q);
      rb[set][i] = load_chunk(B, n0 + r, N, k0 + kc * 16, K);
    }
  };
  auto store_tiles = [&](int set, int buf) {
#pragma unroll
    for (int i = 0; i < CA; ++i) {
      const uint32_t q = tid + i * kThreads, r = chunk_row(q), kc = chunk_col(q);
      decode_chunk_to_lds(ra[set][i], lut16, reinterpret_cast<uint4*>(As + ((size_t)buf * BM + r) * LDA + kc * 16));
    }
#pragma unroll
    for (int i = 0; i < CB; ++i) {
      const uint32_t q = tid + i * kThreads, r = chunk_row(q), kc = chunk_col(q);
      decode_chunk_to_lds(rb[set][i], lut16, reinterpret_cast<uint4*>(Bs + ((size_t)buf * BN + r) * LDA + kc * 16));
    }
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  const uint32_t frag_row = lane & 31u, frag_k = (lane >> 5) * 8u;
  // one K step: MFMAs on LDS buffer `buf` (tile kt) while the codes in register set `set`
  // (tile kt + 1) are expanded into the other buffer and tile kt + 2 is requested from memory
  auto k_step = [&](uint32_t kt, int buf, int set) {
    load_tiles(set ^ 1, (kt + 2) * BK);  // past the last tile this reads zeros (k >= K); never used
    const __bf16* a_base = As + ((size_t)buf * BM + wm * TM * 32 + frag_row) * LDA + frag_k;
    const __bf16* b_base = Bs + ((size_t)buf * BN + wn * TN * 32 + frag_row) * LDA + frag_k;
#pragma unroll
    for (int s = 0; s < BK / 16; ++s) {
      bf16x8 fa[TM], fb[TN];
#pragma unroll
      for (int i = 0; i < TM; ++i) fa[i] = *reinterpret_cast<const bf16x8*>(a_base + (size_t)i * 32 * LDA + s * 16);
#pragma unroll
      for (int j = 0; j < TN; ++j) fb[j] = *reinterpret_cast<const bf16x8*>(b_base + (size_t)j * 32 * LDA + s * 16);
#pragma unroll
      for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[i], fb[j], acc[i][j], 0, 0, 0);
    }
    store_tiles(set, buf ^ 1);
    __syncthreads();
  };

  const uint32_t nk = (K + BK - 1) / BK;
  load_tiles(0, 0);
  load_tiles(1, BK);
  __syncthreads();  // table staged
  store_tiles(0, 0);
  __syncthreads();
  // register sets alternate with the LDS buffers: tile kt + 1 sits in set (kt + 1) & 1
  uint32_t kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    k_step(kt, 0, 1);
    k_step(kt + 1, 1, 0);
  }
  if (kt < nk) k_step(kt, 0, 1);

  // the last K step ended with a barrier: the tile buffers (behind the table) are free for the error sums
  epilogue<EPI, TM, TN>(acc, out, ref, err, M, N, m0 + wm * TM * 32, n0 + wn * TN * 32, lane, descale,
                        reinterpret_cast<double*>(As), wave, WM * WN);
}

// any K, any alignment: one output element per lane, codes expanded with the integer decoder
template <int EPI>
__global__ void __launch_bounds__(256)
k_gemm_nt_simple(const uint8_t* __restrict__ A, const uint8_t* __restrict__ B, void* __restrict__ out,
                 const float* __restrict__ ref, double* __restrict__ err, uint32_t M, uint32_t N, uint32_t K,
                 float descale) {
  const size_t total = (size_t)M * N;
  double e2 = 0.0;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += (size_t)gridDim.x * blockDim.x) {
    const uint32_t row = (uint32_t)(idx / N), col = (uint32_t)(idx - (size_t)row * N);
    const uint8_t* a = A + (size_t)row * K;
    const uint8_t* b = B + (size_t)col * K;
    float s = 0.0f;
    for (uint32_t k = 0; k < K; ++k) s = fmaf(__uint_as_float(decode_bits(a[k])), __uint_as_float(decode_bits(b[k])), s);
    const float o = __fmul_rn(s, descale);
    if constexpr (EPI == EPI_F32) reinterpret_cast<float*>(out)[idx] = o;
    else if constexpr (EPI == EPI_BF16) reinterpret_cast<uint16_t*>(out)[idx] = (uint16_t)narrow_bf16(__float_as_uint(o));
    else if constexpr (EPI == EPI_F16) reinterpret_cast<_Float16*>(out)[idx] = (_Float16)o;
    else {
      const double d = (double)o - (double)ref[idx];
      e2 = fma(d, d, e2);
    }
  }
  if constexpr (EPI == EPI_ERR) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) e2 += __shfl_xor(e2, off, 64);
    if ((threadIdx.x & 63u) == 0u) unsafeAtomicAdd(err, e2);
  }
}

// ====================================================================================
// host side
// ====================================================================================
constexpr int kMaxDevices = 64;
static const uint16_t* g_lut_ptr[kMaxDevices] = {};

static hif8_status gemm_init(const uint16_t** lut_out, int* cus_out) {
  int cus = 0;
  hif8_status s = ensure_init(&cus, nullptr);
  if (s != HIF8_OK) return s;
  int dev = 0;
  if (!hip_ok(hipGetDevice(&dev))) return HIF8_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return HIF8_ERR_ARG;
  static std::mutex mu;
  std::lock_guard<std::mutex> lock(mu);
  if (!g_lut_ptr[dev]) {
    void* p = nullptr;
    if (!hip_ok(hipGetSymbolAddress(&p, HIP_SYMBOL(g_bf16_lut)))) return HIF8_ERR_HIP;
    hipLaunchKernelGGL(k_build_gemm_lut, dim3(1), dim3(256), 0, (hipStream_t)0);
    if (!hip_ok(hipGetLastError())) return HIF8_ERR_HIP;
    if (!hip_ok(hipStreamSynchronize((hipStream_t)0))) return HIF8_ERR_HIP;
    g_lut_ptr[dev] = reinterpret_cast<const uint16_t*>(p);
  }
  *lut_out = g_lut_ptr[dev];
  if (cus_out) *cus_out = cus;
  return HIF8_OK;
}

template <int WM, int WN, int TM, int TN, int BK>
constexpr size_t smem_bytes() {
  return 256 * kLutCopies * 4 + (size_t)2 * (WM * TM * 32 + WN * TN * 32) * (BK + kPad) * 2;
}

template <int WM, int WN, int TM, int TN, int BK, int EPI>
static hif8_status launch_tiled(const uint8_t* A, const uint8_t* B, void* out, const float* ref, double* err,
                                uint32_t M, uint32_t N, uint32_t K, float descale, const uint16_t* lut,
                                hipStream_t st, const Batch& batch = Batch{0u, 0, 0, 0}, uint32_t pairs = 1,
                                uint32_t col_begin = 0, uint32_t col_end = 0xFFFFFFFFu) {
  if (col_end > N) col_end = N;
  if (col_begin >= col_end) return HIF8_OK;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr size_t smem = smem_bytes<WM, WN, TM, TN, BK>();
  static bool attr_set[kMaxDevices] = {};
  int dev = 0;
  if (!hip_ok(hipGetDevice(&dev))) return HIF8_ERR_HIP;
  if (!attr_set[dev]) {
    if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_nt<WM, WN, TM, TN, BK, EPI>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem)))
      return HIF8_ERR_HIP;
    attr_set[dev] = true;
  }
  const uint32_t tiles_m = (M + BM - 1) / BM, tiles_n = (col_end - col_begin + BN - 1) / BN;
  if ((uint64_t)tiles_m * tiles_n > 0x7FFFFFFFull) return HIF8_ERR_ARG;
  hipLaunchKernelGGL((k_gemm_nt<WM, WN, TM, TN, BK, EPI>), dim3(tiles_m * tiles_n, pairs), dim3(64 * WM * WN), smem, st,
                     A, B, out, ref, err, M, N, K, descale, lut, tiles_n, col_begin, batch);
  return finish_launch();
}

static int g_gemm_variant = 0;  // 0 = default choice; tuning knob HIF8_TUNE_GEMM_TILE

template <int EPI>
static hif8_status gemm_dispatch(const uint8_t* A, const uint8_t* B, void* out, const float* ref, double* err,
                                 size_t M, size_t N, size_t K, float scale_a, float scale_b, hipStream_t st) {
  float inv_a = 1.0f, inv_b = 1.0f;
  if (!valid_scale(scale_a, &inv_a) || !valid_scale(scale_b, &inv_b)) return HIF8_ERR_SCALE;
  volatile float ds = inv_a * inv_b;
  const float descale = ds;
  if (!(descale > 0.0f) || std::isinf(descale)) return HIF8_ERR_SCALE;
  if (M == 0 || N == 0) return HIF8_OK;
  if (M > 0x7FFFFFFFu || N > 0x7FFFFFFFu || K > 0x7FFFFFFFu) return HIF8_ERR_ARG;
  if ((!A || !B) && K != 0) return HIF8_ERR_NULL;
  if (EPI == EPI_ERR ? (!ref || !err) : !out) return HIF8_ERR_NULL;
  if (EPI == EPI_ERR && !aligned_to(err, 8)) return HIF8_ERR_ARG;  // fp64 atomics need naturally aligned doubles
  const uint16_t* lut = nullptr;
  int cus = 0;
  hif8_status s = gemm_init(&lut, &cus);
  if (s != HIF8_OK) return s;
  const uint32_t m = (uint32_t)M, n = (uint32_t)N, k = (uint32_t)K;
  const bool fast = K != 0 && (K % 16) == 0 && aligned_to(A, 16) && aligned_to(B, 16);
  if (!fast) {
    hipLaunchKernelGGL(k_gemm_nt_simple<EPI>, dim3(grid_elem(M * N, cus)), dim3(256), 0, st, A, B, out, ref, err, m,
                       n, k, descale);
    return finish_launch();
  }
  int variant = g_gemm_variant;
  uint32_t split = 0;
  if (variant == 0 && ragged_round_split(M, N, (size_t)cus, &split)) {
    // complete rounds of 256 x 256 tiles, then the remaining columns in 128 x 128 tiles (second launch)
    s = launch_tiled<4, 2, 2, 4, 32, EPI>(A, B, out, ref, err, m, n, k, descale, lut, st, Batch{0u, 0, 0, 0}, 1u, 0u, split);
    if (s != HIF8_OK) return s;
    return launch_tiled<2, 2, 2, 2, 32, EPI>(A, B, out, ref, err, m, n, k, descale, lut, st, Batch{0u, 0, 0, 0}, 1u, split, n);
  }
  if (variant == 0)  // 256 x 256 tiles once there is one for every compute unit, else 128 x 128 (two workgroups per CU)
    variant = (((M + 255) / 256) * ((N + 255) / 256) >= (size_t)cus) ? 5 : 6;
  if (variant == 5) return launch_tiled<4, 2, 2, 4, 32, EPI>(A, B, out, ref, err, m, n, k, descale, lut, st);
  return launch_tiled<2, 2, 2, 2, 32, EPI>(A, B, out, ref, err, m, n, k, descale, lut, st);
}

// hif8_gemm_* through a workspace: expand both operands, then the expanded-operand kernel.
static size_t gemm_ws_bytes(size_t M, size_t N, size_t K) {
  if (M == 0 || N == 0 || K == 0) return 0;
  const size_t ld = expanded_ld(K);
  if (ld > kMaxLd || M > 0x7FFFFFFFu || N > 0x7FFFFFFFu) return 0;
  return 2 * (M + N) * ld;
}

template <int EPI>
static hif8_status gemm_ws(const uint8_t* A, const uint8_t* B, void* out, const float* ref, double* err, size_t M,
                           size_t N, size_t K, float scale_a, float scale_b, void* ws, size_t ws_bytes, hipStream_t st) {
  const size_t need = gemm_ws_bytes(M, N, K);
  if (need == 0)  // nothing to expand, or a shape beyond the expanded-operand kernel's limits
    return gemm_dispatch<EPI>(A, B, out, ref, err, M, N, K, scale_a, scale_b, st);
  float inv_a = 1.0f, inv_b = 1.0f;
  if (!valid_scale(scale_a, &inv_a) || !valid_scale(scale_b, &inv_b)) return HIF8_ERR_SCALE;
  volatile float ds = inv_a * inv_b;
  const float descale = ds;
  if (!(descale > 0.0f) || std::isinf(descale)) return HIF8_ERR_SCALE;
  if (!A || !B || !ws) return HIF8_ERR_NULL;
  if (EPI == EPI_ERR ? (!ref || !err) : !out) return HIF8_ERR_NULL;
  if (ws_bytes < need || !aligned_to(ws, 16)) return HIF8_ERR_ARG;
  if (EPI == EPI_ERR && !aligned_to(err, 8)) return HIF8_ERR_ARG;
  const size_t ld = expanded_ld(K);
  uint16_t* xa = reinterpret_cast<uint16_t*>(ws);
  uint16_t* xb = xa + M * ld;  // M * ld * 2 bytes is a multiple of 128: still 16-byte aligned
  hif8_status s = expand_rows(A, M, K, xa, ld, st);
  if (s != HIF8_OK) return s;
  s = expand_rows(B, N, K, xb, ld, st);
  if (s != HIF8_OK) return s;
  return gemm_expanded<EPI>(xa, xb, out, ref, err, M, N, ld, descale, st, Batch{0u, 0, 0, 0}, 1u);
}

// position of the smallest finite entry of err[rows * cols] -> best[0] = e_row_lo + row,
// best[1] = e_col_lo + col (first minimum in row-major order; {e_row_lo, e_col_lo} if none is finite)
__global__ void k_argmin_pair(const double* __restrict__ err, int rows, int cols, int e_row_lo, int e_col_lo,
                              int32_t* __restrict__ best) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  int bi = 0;
  double bv = INFINITY;
  for (int i = 0; i < rows * cols; ++i) {
    const double v = err[i];
    if (v < bv) { bv = v; bi = i; }  // NaN and +Inf never compare below
  }
  best[0] = e_row_lo + bi / cols;
  best[1] = e_col_lo + bi % cols;
}

static size_t calibrate_bytes(size_t M, size_t N, size_t K, int ea_count, int ew_count) {
  const size_t ld = expanded_ld(K);
  return ((M > N ? M : N) * K + 15) / 16 * 16 + 2 * ld * (M * (size_t)ea_count + N * (size_t)ew_count);
}

// Algorithm 1 for one layer: casts at every scale of the search square (each expanded to bfloat16
// once), then one error GEMM per pair.
template <int SRCK>
static hif8_status calibrate_layer(const void* a, const void* w, const float* o_ref, size_t M, size_t N, size_t K,
                                   int ea_lo, int ea_count, int ew_lo, int ew_count, uint32_t mode, void* workspace,
                                   size_t workspace_bytes, double* d_err, int32_t* d_best, hipStream_t st) {
  if (!valid_mode(mode)) return HIF8_ERR_MODE;
  if (ea_count < 1 || ew_count < 1 || ea_count > 64 || ew_count > 64 || ea_lo < -60 || ew_lo < -60 ||
      ea_lo + ea_count - 1 > 60 || ew_lo + ew_count - 1 > 60)
    return HIF8_ERR_ARG;
  if (!a || !w || !o_ref || !workspace || !d_err) return HIF8_ERR_NULL;
  if (!aligned_to(d_err, 8) || (d_best && !aligned_to(d_best, 4))) return HIF8_ERR_ARG;
  if (M == 0 || N == 0 || K == 0) return HIF8_ERR_ARG;
  if (M > 0x7FFFFFFFu || N > 0x7FFFFFFFu || K > kMaxLd) return HIF8_ERR_ARG;
  // workspace: one code matrix at a time (the stream runs the cast, then the expansion, before the
  // next cast overwrites it), then every cast operand expanded to bfloat16 for the matrix cores
  const size_t ld = expanded_ld(K);
  const size_t code_bytes = ((M > N ? M : N) * K + 15) / 16 * 16;
  const size_t a_elems = M * ld, w_elems = N * ld;  // multiples of 64 elements: every matrix stays 128-byte aligned
  if (workspace_bytes < calibrate_bytes(M, N, K, ea_count, ew_count) || !aligned_to(workspace, 16)) return HIF8_ERR_ARG;
  uint8_t* ws_codes = reinterpret_cast<uint8_t*>(workspace);
  uint16_t* ws_a = reinterpret_cast<uint16_t*>(ws_codes + code_bytes);
  uint16_t* ws_w = ws_a + a_elems * ea_count;
  hif8_status s = launch_fill_u32(reinterpret_cast<uint32_t*>(d_err), 0u, 2u * (uint32_t)(ea_count * ew_count), st);
  if (s != HIF8_OK) return s;
  for (int i = 0; i < ea_count; ++i) {
    s = hif8conv::conv_encode<SRCK>(a, ws_codes, M * K, std::ldexp(1.0f, ea_lo + i), nullptr, nullptr, mode, nullptr, st);
    if (s != HIF8_OK) return s;
    s = expand_rows(ws_codes, M, K, ws_a + a_elems * i, ld, st);
    if (s != HIF8_OK) return s;
  }
  for (int j = 0; j < ew_count; ++j) {
    s = hif8conv::conv_encode<SRCK>(w, ws_codes, N * K, std::ldexp(1.0f, ew_lo + j), nullptr, nullptr, mode, nullptr, st);
    if (s != HIF8_OK) return s;
    s = expand_rows(ws_codes, N, K, ws_w + w_elems * j, ld, st);
    if (s != HIF8_OK) return s;
  }
  // all pairs in one launch: the grid's second dimension runs over the search square
  const Batch batch{(uint32_t)ew_count, ea_lo + ew_lo, a_elems, w_elems};
  s = gemm_expanded<EPI_ERR>(ws_a, ws_w, nullptr, o_ref, d_err, M, N, ld, 1.0f, st, batch, (uint32_t)(ea_count * ew_count));
  if (s != HIF8_OK) return s;
  if (d_best) {
    hipLaunchKernelGGL(k_argmin_pair, dim3(1), dim3(64), 0, st, d_err, ea_count, ew_count, ea_lo, ew_lo, d_best);
    return finish_launch();
  }
  return HIF8_OK;
}

}  // namespace hif8gemm

using namespace hif8gemm;

extern "C" {

hif8_status hif8_gemm_set_variant(int variant) {
  if (variant != 0 && variant != 5 && variant != 6 && (variant < 9 || variant > 11)) return HIF8_ERR_ARG;
  if (variant == 0) {
    g_gemm_variant = 0;
    expanded_variant() = 0;
  } else if (variant <= 6) {
    g_gemm_variant = variant;
  } else {
    expanded_variant() = variant;
  }
  return HIF8_OK;
}

size_t hif8_calibrate_workspace_bytes(size_t M, size_t N, size_t K, int ea_count, int ew_count) {
  if (ea_count < 0 || ew_count < 0) return 0;
  return calibrate_bytes(M, N, K, ea_count, ew_count);
}

#define HIF8_DEFINE_CALIBRATE(SFX, T, KIND)                                                                       \
  hif8_status hif8_calibrate_layer_##SFX(const T* a, const T* w, const float* o_ref, size_t M, size_t N,          \
                                         size_t K, int ea_lo, int ea_count, int ew_lo, int ew_count,              \
                                         uint32_t mode, void* workspace, size_t workspace_bytes, double* d_err,   \
                                         int32_t* d_best_or_null, hif8_stream_t stream) {                         \
    return calibrate_layer<KIND>(a, w, o_ref, M, N, K, ea_lo, ea_count, ew_lo, ew_count, mode, workspace,         \
                                 workspace_bytes, d_err, d_best_or_null, (hipStream_t)stream);                    \
  }
HIF8_DEFINE_CALIBRATE(f32, float, kSrcF32)
HIF8_DEFINE_CALIBRATE(bf16, uint16_t, kSrcBF16)
HIF8_DEFINE_CALIBRATE(f16, uint16_t, kSrcF16)
#undef HIF8_DEFINE_CALIBRATE

size_t hif8_gemm_workspace_bytes(size_t M, size_t N, size_t K) { return gemm_ws_bytes(M, N, K); }
hif8_status hif8_gemm_ws_f32(const uint8_t* a_codes, const uint8_t* b_codes, float* out, size_t M, size_t N, size_t K,
                             float scale_a, float scale_b, void* workspace, size_t workspace_bytes, hif8_stream_t stream) {
  return gemm_ws<EPI_F32>(a_codes, b_codes, out, nullptr, nullptr, M, N, K, scale_a, scale_b, workspace, workspace_bytes,
                          (hipStream_t)stream);
}
hif8_status hif8_gemm_ws_bf16(const uint8_t* a_codes, const uint8_t* b_codes, uint16_t* out, size_t M, size_t N, size_t K,
                              float scale_a, float scale_b, void* workspace, size_t workspace_bytes, hif8_stream_t stream) {
  return gemm_ws<EPI_BF16>(a_codes, b_codes, out, nullptr, nullptr, M, N, K, scale_a, scale_b, workspace, workspace_bytes,
                           (hipStream_t)stream);
}
hif8_status hif8_gemm_ws_f16(const uint8_t* a_codes, const uint8_t* b_codes, uint16_t* out, size_t M, size_t N, size_t K,
                             float scale_a, float scale_b, void* workspace, size_t workspace_bytes, hif8_stream_t stream) {
  return gemm_ws<EPI_F16>(a_codes, b_codes, out, nullptr, nullptr, M, N, K, scale_a, scale_b, workspace, workspace_bytes,
                          (hipStream_t)stream);
}
hif8_status hif8_gemm_ws_sqerr(const uint8_t* a_codes, const uint8_t* b_codes, const float* ref, size_t M, size_t N,
                               size_t K, float scale_a, float scale_b, double* d_err, void* workspace,
                               size_t workspace_bytes, hif8_stream_t stream) {
  return gemm_ws<EPI_ERR>(a_codes, b_codes, nullptr, ref, d_err, M, N, K, scale_a, scale_b, workspace, workspace_bytes,
                          (hipStream_t)stream);
}

hif8_status hif8_gemm_f32(const uint8_t* a_codes, const uint8_t* b_codes, float* out, size_t M, size_t N, size_t K,
                          float scale_a, float scale_b, hif8_stream_t stream) {
  return gemm_dispatch<EPI_F32>(a_codes, b_codes, out, nullptr, nullptr, M, N, K, scale_a, scale_b, (hipStream_t)stream);
}
hif8_status hif8_gemm_bf16(const uint8_t* a_codes, const uint8_t* b_codes, uint16_t* out, size_t M, size_t N,
                           size_t K, float scale_a, float scale_b, hif8_stream_t stream) {
  return gemm_dispatch<EPI_BF16>(a_codes, b_codes, out, nullptr, nullptr, M, N, K, scale_a, scale_b, (hipStream_t)stream);
}
hif8_status hif8_gemm_f16(const uint8_t* a_codes, const uint8_t* b_codes, uint16_t* out, size_t M, size_t N,
                          size_t K, float scale_a, float scale_b, hif8_stream_t stream) {
  return gemm_dispatch<EPI_F16>(a_codes, b_codes, out, nullptr, nullptr, M, N, K, scale_a, scale_b, (hipStream_t)stream);
}
hif8_status hif8_gemm_sqerr(const uint8_t* a_codes, const uint8_t* b_codes, const float* ref, size_t M, size_t N,
                            size_t K, float scale_a, float scale_b, double* d_err, hif8_stream_t stream) {
  return gemm_dispatch<EPI_ERR>(a_codes, b_codes, nullptr, ref, d_err, M, N, K, scale_a, scale_b, (hipStream_t)stream);
}

}  // extern "C"
