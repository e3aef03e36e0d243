// Pieces shared by the two simulated-HiF8 GEMM kernels (u8 code operands expanded in the kernel,
// and operands already expanded to bfloat16): accumulator types, the batched-launch descriptor
// of Algorithm 1's scale search, and the epilogue (descale, then store or score against a reference).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "hif8.h"
#include "hif8_device.hpp"
#include "hif8_gemm_split.hpp"

namespace hif8gemm {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

enum : int { EPI_F32 = 0, EPI_BF16 = 1, EPI_F16 = 2, EPI_ERR = 3 };

// Batched launches: pair p = blockIdx.y uses A + (p / nb) * a_stride, B + (p % nb) * b_stride
// (strides in operand elements), err[p], and descale 2^-(e_base + p / nb + p % nb).
// nb == 0: a single GEMM.
struct Batch {
  uint32_t nb;
  int e_base;
  size_t a_stride, b_stride;
};

// Epilogue of one wavefront: TM x TN accumulator blocks of v_mfma_f32_32x32x16_bf16 whose top-left
// element is (row0, col0).  Element v of a 32 x 32 block sits at row (v / 4) * 8 + (lane / 32) * 4 + v % 4,
// column lane % 32.  EPI_ERR adds the squared differences to *err in fp64: the wavefronts of the workgroup
// combine through `wg_scratch` (LDS, at least one double per wavefront, free of other use by now; every
// wavefront of the workgroup must make this call) and issue one atomic per workgroup.
template <int EPI>
__device__ __forceinline__ void store_one(void* __restrict__ out, size_t idx, float o) {
  if constexpr (EPI == EPI_F32) reinterpret_cast<float*>(out)[idx] = o;
  else if constexpr (EPI == EPI_BF16) reinterpret_cast<uint16_t*>(out)[idx] = (uint16_t)hif8dev::narrow_bf16(__float_as_uint(o));
  else reinterpret_cast<_Float16*>(out)[idx] = (_Float16)o;
}

template <int EPI, int TM, int TN>
__device__ __forceinline__ void epilogue(const f32x16 (&acc)[TM][TN], void* __restrict__ out,
                                         const float* __restrict__ ref, double* __restrict__ err, uint32_t M,
                                         uint32_t N, uint32_t row0, uint32_t col0, uint32_t lane, float descale,
                                         double* wg_scratch, uint32_t wave, uint32_t n_waves) {
  double e2 = 0.0;
  // the whole wavefront tile inside the matrix (the usual case): no per-element bounds checks
  const bool inside = row0 + TM * 32 <= M && col0 + TN * 32 <= N;
#pragma unroll
  for (int i = 0; i < TM; ++i) {
#pragma unroll
    for (int j = 0; j < TN; ++j) {
      const uint32_t col = col0 + j * 32 + (lane & 31u);
      const uint32_t rbase = row0 + i * 32 + (lane >> 5) * 4;
      if constexpr (EPI == EPI_ERR) {
        // all 16 reference values of the block are requested before the first is used; positions
        // outside the matrix read element 0 and contribute nothing
        float r[16];
        bool ok[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const uint32_t row = rbase + (v >> 2) * 8 + (v & 3);
          ok[v] = inside || (row < M && col < N);
          r[v] = ref[ok[v] ? (size_t)row * N + col : (size_t)0];
        }
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const double d = (double)__fmul_rn(acc[i][j][v], descale) - (double)r[v];
          e2 = ok[v] ? fma(d, d, e2) : e2;
        }
      } else if (inside) {
#pragma unroll
        for (int v = 0; v < 16; ++v)
          store_one<EPI>(out, (size_t)(rbase + (v >> 2) * 8 + (v & 3)) * N + col, __fmul_rn(acc[i][j][v], descale));
      } else {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
          const uint32_t row = rbase + (v >> 2) * 8 + (v & 3);
          if (row < M && col < N) store_one<EPI>(out, (size_t)row * N + col, __fmul_rn(acc[i][j][v], descale));
        }
      }
    }
  }
  if constexpr (EPI == EPI_ERR) {
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) e2 += __shfl_xor(e2, off, 64);
    if (lane == 0) wg_scratch[wave] = e2;
    __syncthreads();
    if (wave == 0 && lane == 0) {
      double t = 0.0;
      for (uint32_t w = 0; w < n_waves; ++w) t += wg_scratch[w];
      unsafeAtomicAdd(err, t);  // hardware fp64 add at the L2, no compare-and-swap loop
    }
  }
}

// ---- operands expanded to bfloat16 (hif8_gemm_x.hip) ----
// Row pitch of an expanded operand: K rounded up to the K step of the kernel.
constexpr size_t kExpandK = 64;
inline size_t expanded_ld(size_t K) { return (K + kExpandK - 1) / kExpandK * kExpandK; }
// Largest pitch the GEMM accepts: 256 rows x pitch x 2 bytes must fit the 32-bit lane offsets of its tile loads.
constexpr size_t kMaxLd = (size_t)1 << 22;

// tile layout of the expanded-operand kernel: 0 = by problem size, 9 = 128 x 128 with 4 wavefronts,
// 10 / 11 = 256 x 256 as 2 x 2 / 2 x 4 wavefronts with the hand-placed K step (set through hif8_gemm_set_variant)
int& expanded_variant();

hif8_status expand_rows(const uint8_t* codes, size_t rows, size_t K, uint16_t* dst, size_t ld, hipStream_t st);
hif8_status expand_cols(const uint8_t* codes, size_t rows, size_t cols, uint16_t* dst, size_t ld, hipStream_t st);

// out = (A x B^T) * descale on operands of pitch ld (zero beyond K); batch.nb != 0: `pairs` GEMMs in one launch
template <int EPI>
hif8_status gemm_expanded(const uint16_t* A, const uint16_t* B, void* out, const float* ref, double* err, size_t M,
                          size_t N, size_t ld, float descale, hipStream_t st, const Batch& batch, uint32_t pairs);

}  // namespace hif8gemm
