// Simulated HiF8 GEMM on operands that were expanded to bfloat16 beforehand.
//
// Every HiF8 value is exact in bfloat16, so a code matrix can be expanded once (3 bytes of HBM
// traffic per element) and then multiplied any number of times without touching the decoder
// again -- the shape of Algorithm 1's scale search (10 + 10 casts, 100 products) and of a
// training step that uses a cast weight in the forward and the backward GEMM (Sec. 5).
//
//   expand:  X[r, k] = bf16(value(codes[r, k]))  for k < K,  0 for K <= k < ld,  ld = K rounded up to 64
//   GEMM:    O[M, N] = (A[M, ld] x B[N, ld]^T) * descale
//
// Kernel design (gfx950): a workgroup of WM x WN wavefronts owns a (WM TM 32) x (WN TN 32) tile of O.
// K advances in steps of 64 through two LDS stages.  Tiles go from global memory straight into LDS
// (buffer_load_dwordx4 ... lds: 64 lanes x 16 bytes land contiguously), so the operands never pass
// through registers.  A tile row is 128 bytes = 8 chunks of 16 bytes; chunk position p of tile row r
// holds k-chunk p ^ ((r >> 1) & 7).  LDS has 64 banks of 4 bytes and serves a 16-byte read 16 lanes
// at a time: the 16 lanes of a fragment read touch 16 consecutive rows of one k-chunk, which the
// permutation spreads over all 16 chunk slots of two adjacent rows -- no bank conflicts, no padding.
// Fragments are double-buffered in registers, and the workgroup barrier sits before the last of
// the four MFMA groups of a K step, so the first fragments of the next step are fetched under it.
#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>

#include "hif8.h"
#include "hif8_device.hpp"
#include "hif8_gemm_common.hpp"
#include "hif8_host.hpp"

namespace hif8gemm {

using namespace hif8dev;
using namespace hif8host;

constexpr int kBK = (int)kExpandK;  // K step
constexpr int kRowBytes = kBK * 2;  // one tile row in LDS
constexpr int kRowsPerLoad = 8;     // a wavefront-wide 16-byte load covers 8 tile rows

// s_waitcnt immediates (gfx9 encoding: vmcnt[3:0] | expcnt[6:4] | lgkmcnt[11:8] | vmcnt[15:14])
constexpr int kWaitLgkm0 = 0xC07F;        // lgkmcnt(0)
constexpr int kWaitVm0Lgkm0 = 0x0070;     // vmcnt(0) lgkmcnt(0)
constexpr int kWaitVm0 = 0x0F70;          // vmcnt(0)
constexpr int kRsrcFlags = 0x00020000;    // word 3 of a raw (unstructured, untyped) buffer descriptor on gfx9-family parts

template <int WM, int WN, int TM, int TN, int EPI, int FINE = 0>
__global__ void __launch_bounds__(64 * WM * WN)
k_gemm_x(const uint16_t* __restrict__ A, const uint16_t* __restrict__ B, void* __restrict__ out,
         const float* __restrict__ ref, double* __restrict__ err, uint32_t M, uint32_t N, uint32_t ld,
         float descale, uint32_t tiles_n, uint32_t col_begin, Batch batch) {
  if (batch.nb != 0u) {
    const uint32_t bi = blockIdx.y / batch.nb, bj = blockIdx.y - bi * batch.nb;
    A += (size_t)bi * batch.a_stride;
    B += (size_t)bj * batch.b_stride;
    err += blockIdx.y;
    descale = pow2f(-(batch.e_base + (int)bi + (int)bj));
  }
  constexpr int kWaves = WM * WN;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr int IA = BM / kRowsPerLoad / kWaves, IB = BN / kRowsPerLoad / kWaves;  // loads per wavefront and K step
  static_assert(BM % (kRowsPerLoad * kWaves) == 0 && BN % (kRowsPerLoad * kWaves) == 0, "tile / wavefront mismatch");
  constexpr int kStageBytes = (BM + BN) * kRowBytes;
  static_assert(kStageBytes == 65536 || kStageBytes == 32768, "stage size");
  extern __shared__ __attribute__((aligned(128))) uint8_t smem[];  // [2][BM + BN][128 bytes]

  const uint32_t tid = threadIdx.x, lane = tid & 63u;
  const uint32_t wave = __builtin_amdgcn_readfirstlane(tid >> 6);  // scalar: LDS destinations of the loads stay in SGPRs
  const uint32_t wm = wave / WN, wn = wave % WN;
  uint32_t tile_m, tile_n;  // in an order that keeps the workgroups of one die on neighbouring tiles
  if (!tile_order(blockIdx.x, (M - 1u) / BM + 1u, tiles_n, &tile_m, &tile_n)) return;  // the whole workgroup leaves
  const uint32_t m0 = tile_m * BM, n0 = col_begin + tile_n * BN;  // the launch covers columns from col_begin on

  // Tile loads are buffer loads into LDS: one descriptor per operand panel of this workgroup (SGPRs), a
  // 32-bit byte offset per lane that never changes, and a scalar offset that advances along K -- no vector
  // ALU work per load.  The descriptor ends with the matrix, so rows past it read as zeros.
  const size_t bytes_a = ((size_t)M - m0) * ld * 2u, bytes_b = ((size_t)N - n0) * ld * 2u;
  const __amdgpu_buffer_rsrc_t res_a = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(A + (size_t)m0 * ld), 0, (int)(bytes_a > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)bytes_a), kRsrcFlags);
  const __amdgpu_buffer_rsrc_t res_b = __builtin_amdgcn_make_buffer_rsrc(
      const_cast<uint16_t*>(B + (size_t)n0 * ld), 0, (int)(bytes_b > 0xFFFFFFFFull ? 0xFFFFFFFFu : (uint32_t)bytes_b), kRsrcFlags);
  // lane -> tile row 8 * (load index) + lane / 8, chunk position lane % 8 (which holds k-chunk position ^ ((row >> 1) & 7))
  const uint32_t lr = lane >> 3, lc = lane & 7u;
  uint32_t off_a[IA], off_b[IB];
#pragma unroll
  for (int i = 0; i < IA; ++i) {
    const uint32_t r = (wave * IA + i) * kRowsPerLoad + lr;
    off_a[i] = (r * ld + ((lc ^ ((r >> 1) & 7u)) * 8u)) * 2u;  // < 2^32: the host limits ld
  }
#pragma unroll
  for (int i = 0; i < IB; ++i) {
    const uint32_t r = (wave * IB + i) * kRowsPerLoad + lr;
    off_b[i] = (r * ld + ((lc ^ ((r >> 1) & 7u)) * 8u)) * 2u;
  }
  uint32_t koff = 0;  // byte offset along K of the next tile to request
  auto issue = [&](int stage) {
    uint8_t* sa = smem + stage * kStageBytes + wave * IA * kRowsPerLoad * kRowBytes;
    uint8_t* sb = smem + stage * kStageBytes + BM * kRowBytes + wave * IB * kRowsPerLoad * kRowBytes;
#pragma unroll
    for (int i = 0; i < IA; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(res_a, (__attribute__((address_space(3))) void*)(sa + i * kRowsPerLoad * kRowBytes),
                                               16, (int)off_a[i], (int)koff, 0, 0);
#pragma unroll
    for (int i = 0; i < IB; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(res_b, (__attribute__((address_space(3))) void*)(sb + i * kRowsPerLoad * kRowBytes),
                                               16, (int)off_b[i], (int)koff, 0, 0);
    koff += kBK * 2;
  };

  f32x16 acc[TM][TN];
#pragma unroll
  for (int i = 0; i < TM; ++i)
#pragma unroll
    for (int j = 0; j < TN; ++j)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

  // MFMA operand of lane l: row l % 32 of the block, k elements 8 * (l / 32) .. + 7 of the 16-wide step.
  // LDS address of the lane's A fragment of block row 0 for every (stage, step), computed once; the other
  // block rows and the B fragments are constant offsets from it.
  const uint32_t frow = lane & 31u, fk = lane >> 5;
  const uint32_t swz = (frow >> 1) & 7u;  // block row offsets are multiples of 32: the permutation depends on frow only
  uint32_t fbase[2][4];
#pragma unroll
  for (int st = 0; st < 2; ++st)
#pragma unroll
    for (int s = 0; s < 4; ++s)
      fbase[st][s] = st * kStageBytes + (wm * TM * 32 + frow) * kRowBytes + ((((uint32_t)(s * 2) + fk) ^ swz) * 16u);
  const uint32_t b_delta = BM * kRowBytes + (wn * TN * 32) * kRowBytes - (wm * TM * 32) * kRowBytes;  // scalar
  bf16x8 fa[2][TM], fb[2][TN];
  auto read_frags = [&](int buf, int stage, int s) {
    const uint8_t* base = smem + fbase[stage][s];
#pragma unroll
    for (int i = 0; i < TM; ++i) fa[buf][i] = *reinterpret_cast<const bf16x8*>(base + i * 32 * kRowBytes);
#pragma unroll
    for (int j = 0; j < TN; ++j) fb[buf][j] = *reinterpret_cast<const bf16x8*>(base + b_delta + j * 32 * kRowBytes);
  };
  auto mfmas = [&](int buf) {
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
      for (int j = 0; j < TN; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
  };

  // One K step on LDS stage `cur` (a compile-time constant at both call sites).  The scheduling barriers
  // pin "fetch the next fragments, then the MFMAs of the current ones"; each explicit wait sits where the
  // reads it covers were issued a whole MFMA group earlier.
  const uint32_t nk = ld / kBK;  // >= 1
  auto k_step = [&](int cur, uint32_t kt) {
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    read_frags(1, cur, 1);
    __builtin_amdgcn_sched_barrier(0);
    mfmas(0);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    read_frags(0, cur, 2);
    __builtin_amdgcn_sched_barrier(0);
    mfmas(1);
    __builtin_amdgcn_sched_barrier(0);
    __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
    read_frags(1, cur, 3);
    __builtin_amdgcn_sched_barrier(0);
    mfmas(0);
    __builtin_amdgcn_sched_barrier(0);
    // this wavefront's part of tile kt + 1 has landed and its last fragments of tile kt are in registers;
    // after the barrier that holds for the whole workgroup, so stage `cur` may be overwritten
    __builtin_amdgcn_s_waitcnt(kWaitVm0Lgkm0);
    __syncthreads();
    if (kt + 2 < nk) issue(cur);
    if (kt + 1 < nk) read_frags(0, cur ^ 1, 0);
    __builtin_amdgcn_sched_barrier(0);
    mfmas(1);
  };
  // The same K step with every instruction placed by hand (FINE): one fragment read behind each of the first
  // TM + TN MFMAs of a group, and the tile loads of the step after next spread over the last group, so that a
  // wavefront that has its SIMD to itself never leaves the matrix core waiting behind a burst of memory
  // instructions.  Used while two more tiles follow; the last steps run k_step.
  auto read_one = [&](int buf, int stage, int s, int r) {
    const uint8_t* base = smem + fbase[stage][s];
    if (r < TM) fa[buf][r] = *reinterpret_cast<const bf16x8*>(base + r * 32 * kRowBytes);
    else fb[buf][r - TM] = *reinterpret_cast<const bf16x8*>(base + b_delta + (r - TM) * 32 * kRowBytes);
  };
  auto issue_one = [&](int stage, int i) {
    uint8_t* sa = smem + stage * kStageBytes + wave * IA * kRowsPerLoad * kRowBytes;
    uint8_t* sb = smem + stage * kStageBytes + BM * kRowBytes + wave * IB * kRowsPerLoad * kRowBytes;
    if (i < IA)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(res_a, (__attribute__((address_space(3))) void*)(sa + i * kRowsPerLoad * kRowBytes),
                                               16, (int)off_a[i], (int)koff, 0, 0);
    else
      __builtin_amdgcn_raw_ptr_buffer_load_lds(res_b, (__attribute__((address_space(3))) void*)(sb + (i - IA) * kRowsPerLoad * kRowBytes),
                                               16, (int)off_b[i - IA], (int)koff, 0, 0);
  };
  auto fine_step = [&](int cur) {
    constexpr int NM = TM * TN, NR = TM + TN, NL = IA + IB;
    static_assert(NR <= NM, "one fragment read per MFMA");
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      const int buf = s & 1;
      __builtin_amdgcn_sched_barrier(0);
      if (s == 3) {
        // tile kt + 1 has landed and the last fragments of tile kt are in registers, for the whole workgroup
        __builtin_amdgcn_s_waitcnt(kWaitVm0Lgkm0);
        __syncthreads();
      } else {
        __builtin_amdgcn_s_waitcnt(kWaitLgkm0);
      }
      __builtin_amdgcn_sched_barrier(0);
#pragma unroll
      for (int idx = 0; idx < NM; ++idx) {
        const int i = idx / TN, j = idx % TN;
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[buf][i], fb[buf][j], acc[i][j], 0, 0, 0);
        __builtin_amdgcn_sched_barrier(0);  // the MFMA first: the memory instructions issue while it runs
        if (idx < NR) {
          if (s < 3) read_one(buf ^ 1, cur, s + 1, idx);
          else read_one(buf ^ 1, cur ^ 1, 0, idx);
        }
        if (s == 3) {
#pragma unroll
          for (int l = idx * NL / NM; l < (idx + 1) * NL / NM; ++l) issue_one(cur, l);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
    }
    koff += kBK * 2;
  };
  issue(0);
  __builtin_amdgcn_s_waitcnt(kWaitVm0);
  __syncthreads();
  if (nk > 1) issue(1);
  read_frags(0, 0, 0);
  uint32_t kt = 0;
  if constexpr (FINE != 0) {
    for (; kt + 3 < nk; kt += 2) {
      fine_step(0);
      fine_step(1);
    }
    // at most three steps are left, and kt is even
    if (kt < nk) k_step(0, kt);
    if (kt + 1 < nk) k_step(1, kt + 1);
    if (kt + 2 < nk) k_step(0, kt + 2);
  } else {
    for (; kt + 1 < nk; kt += 2) {
      k_step(0, kt);
      k_step(1, kt + 1);
    }
    if (kt < nk) k_step(0, kt);
  }

  // every fragment of the last step was in registers before the last barrier, so the tile LDS is free
  epilogue<EPI, TM, TN>(acc, out, ref, err, M, N, m0 + wm * TM * 32, n0 + wn * TN * 32, lane, descale,
                        reinterpret_cast<double*>(smem), wave, kWaves);
}

// codes [rows, K] -> bf16 [rows, ld]; one 16-byte output chunk (8 elements) per lane and step
__global__ void __launch_bounds__(256)
k_expand_rows(const uint8_t* __restrict__ codes, uint16_t* __restrict__ dst, size_t rows, uint32_t K, uint32_t ld,
              int vec_ok) {
  __shared__ uint16_t lut[256];
  lut[threadIdx.x] = (uint16_t)(decode_bits(threadIdx.x) >> 16);  // blockDim.x == 256
  __syncthreads();
  const uint32_t cpr = ld / 8u;  // output chunks per row
  const size_t total = rows * cpr;
  for (size_t q = (size_t)blockIdx.x * blockDim.x + threadIdx.x; q < total; q += (size_t)gridDim.x * blockDim.x) {
    const size_t row = q / cpr;
    const uint32_t k = (uint32_t)(q - row * cpr) * 8u;
    const uint8_t* src = codes + row * K + k;
    uint32_t c[8];
    if (vec_ok && k + 8u <= K) {
      const uint2 v = *reinterpret_cast<const uint2*>(src);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        c[j] = (v.x >> (8 * j)) & 0xFFu;
        c[4 + j] = (v.y >> (8 * j)) & 0xFFu;
      }
    } else {
#pragma unroll
      for (int j = 0; j < 8; ++j) c[j] = (k + j < K) ? (uint32_t)src[j] : 0u;  // code 0x00 is +0
    }
    uint4 o;
    o.x = lut[c[0]] | ((uint32_t)lut[c[1]] << 16);
    o.y = lut[c[2]] | ((uint32_t)lut[c[3]] << 16);
    o.z = lut[c[4]] | ((uint32_t)lut[c[5]] << 16);
    o.w = lut[c[6]] | ((uint32_t)lut[c[7]] << 16);
    *reinterpret_cast<uint4*>(dst + row * ld + k) = o;
  }
}

// codes [rows, cols] -> bf16 [cols, ld], transposed: dst[c * ld + r] = value(codes[r * cols + c]), zeros for
// rows <= r < ld.  64 x 64 tiles through LDS: 16 codes per lane on the way in, one 16-byte chunk of an
// output row per lane on the way out (8 consecutive lanes write 128 contiguous bytes).
constexpr int kTT = 64;           // tile edge
constexpr int kTPitch = kTT + 2;  // LDS row pitch in elements (33 dwords: consecutive rows start one bank apart)
__global__ void __launch_bounds__(256)
k_expand_cols(const uint8_t* __restrict__ codes, uint16_t* __restrict__ dst, uint32_t rows, uint32_t cols, uint32_t ld,
              uint32_t tiles_c, uint32_t n_tiles, int vec_ok) {
  __shared__ uint16_t lut[256];
  __shared__ __attribute__((aligned(16))) uint16_t tile[kTT * kTPitch];
  const uint32_t t = threadIdx.x;
  lut[t] = (uint16_t)(decode_bits(t) >> 16);  // blockDim.x == 256
  for (uint32_t id = blockIdx.x; id < n_tiles; id += gridDim.x) {
    const uint32_t tr = id / tiles_c, tc = id - tr * tiles_c;
    const uint32_t r0 = tr * kTT, c0 = tc * kTT;
    __syncthreads();  // table written (first pass) / previous tile fully read
    {
      const uint32_t r = r0 + (t >> 2), c = c0 + (t & 3u) * 16u;
      uint32_t w[4] = {0u, 0u, 0u, 0u};  // code 0x00 is +0: everything outside the matrix expands to zero
      if (r < rows && c < cols) {
        const uint8_t* src = codes + (size_t)r * cols + c;
        if (vec_ok && c + 16u <= cols) {
          const uint4 v = *reinterpret_cast<const uint4*>(src);
          w[0] = v.x; w[1] = v.y; w[2] = v.z; w[3] = v.w;
        } else {
          for (uint32_t j = 0; j < 16u && c + j < cols; ++j) w[j >> 2] |= (uint32_t)src[j] << (8u * (j & 3u));
        }
      }
      uint32_t* trow = reinterpret_cast<uint32_t*>(tile + (t >> 2) * kTPitch + (t & 3u) * 16u);
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        trow[2 * j] = lut[w[j] & 0xFFu] | ((uint32_t)lut[(w[j] >> 8) & 0xFFu] << 16);
        trow[2 * j + 1] = lut[(w[j] >> 16) & 0xFFu] | ((uint32_t)lut[w[j] >> 24] << 16);
      }
    }
    __syncthreads();
#pragma unroll
    for (int k = 0; k < 2; ++k) {
      const uint32_t q = t + k * 256u, c = q >> 3, rc = (q & 7u) * 8u;  // output row c0 + c, elements r0 + rc .. + 7
      if (c0 + c < cols) {
        const uint16_t* col = tile + rc * kTPitch + c;
        uint4 o;
        o.x = col[0] | ((uint32_t)col[kTPitch] << 16);
        o.y = col[2 * kTPitch] | ((uint32_t)col[3 * kTPitch] << 16);
        o.z = col[4 * kTPitch] | ((uint32_t)col[5 * kTPitch] << 16);
        o.w = col[6 * kTPitch] | ((uint32_t)col[7 * kTPitch] << 16);
        *reinterpret_cast<uint4*>(dst + (size_t)(c0 + c) * ld + r0 + rc) = o;
      }
    }
  }
}

// ====================================================================================
// host side
// ====================================================================================
hif8_status expand_rows(const uint8_t* codes, size_t rows, size_t K, uint16_t* dst, size_t ld, hipStream_t st) {
  if (rows == 0) return HIF8_OK;
  if (!dst || (!codes && K != 0)) return HIF8_ERR_NULL;
  if (ld == 0 || ld % kExpandK != 0 || ld < K || ld > 0x7FFFFFC0u || K > 0x7FFFFFFFu || !aligned_to(dst, 16))
    return HIF8_ERR_ARG;
  if (rows > ((size_t)1 << 60) / ld) return HIF8_ERR_ARG;
  int cus = 0;
  hif8_status s = ensure_init(&cus, nullptr);
  if (s != HIF8_OK) return s;
  const int vec_ok = (K % 8 == 0) && aligned_to(codes, 8);
  const size_t total = rows * (ld / 8);
  const size_t want = (total + 255) / 256;
  const unsigned grid = (unsigned)(want < (size_t)cus * 16 ? want : (size_t)cus * 16);
  hipLaunchKernelGGL(k_expand_rows, dim3(grid), dim3(256), 0, st, codes, dst, rows, (uint32_t)K, (uint32_t)ld, vec_ok);
  return finish_launch();
}

hif8_status expand_cols(const uint8_t* codes, size_t rows, size_t cols, uint16_t* dst, size_t ld, hipStream_t st) {
  if (cols == 0) return HIF8_OK;
  if (!dst || (!codes && rows != 0)) return HIF8_ERR_NULL;
  if (ld == 0 || ld % kExpandK != 0 || ld < rows || ld > 0x7FFFFFC0u || cols > 0x7FFFFFFFu || !aligned_to(dst, 16))
    return HIF8_ERR_ARG;
  if (cols > ((size_t)1 << 60) / ld) return HIF8_ERR_ARG;
  int cus = 0;
  hif8_status s = ensure_init(&cus, nullptr);
  if (s != HIF8_OK) return s;
  const int vec_ok = (cols % 16 == 0) && aligned_to(codes, 16);
  const size_t tiles_c = (cols + kTT - 1) / kTT, n_tiles = (ld / kTT) * tiles_c;
  if (n_tiles > 0x7FFFFFFFull) return HIF8_ERR_ARG;
  const unsigned grid = (unsigned)(n_tiles < (size_t)cus * 16 ? n_tiles : (size_t)cus * 16);
  hipLaunchKernelGGL(k_expand_cols, dim3(grid), dim3(256), 0, st, codes, dst, (uint32_t)rows, (uint32_t)cols, (uint32_t)ld,
                     (uint32_t)tiles_c, (uint32_t)n_tiles, vec_ok);
  return finish_launch();
}

constexpr int kMaxDevices = 64;

int& expanded_variant() {
  static int v = 0;
  return v;
}

template <int WM, int WN, int TM, int TN, int EPI, int FINE = 0>
static hif8_status launch_x(const uint16_t* A, const uint16_t* B, void* out, const float* ref, double* err, uint32_t M,
                            uint32_t N, uint32_t ld, float descale, hipStream_t st, const Batch& batch, uint32_t pairs,
                            uint32_t col_begin = 0, uint32_t col_end = 0xFFFFFFFFu) {
  if (col_end > N) col_end = N;
  constexpr int BM = WM * TM * 32, BN = WN * TN * 32;
  constexpr size_t smem = (size_t)2 * (BM + BN) * kRowBytes;
  static bool attr_set[kMaxDevices] = {};
  int dev = 0;
  if (!hip_ok(hipGetDevice(&dev))) return HIF8_ERR_HIP;
  if (dev < 0 || dev >= kMaxDevices) return HIF8_ERR_ARG;
  if (!attr_set[dev]) {
    if (!hip_ok(hipFuncSetAttribute(reinterpret_cast<const void*>(&k_gemm_x<WM, WN, TM, TN, EPI, FINE>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem)))
      return HIF8_ERR_HIP;
    attr_set[dev] = true;
  }
  if (col_begin >= col_end) return HIF8_OK;
  const uint32_t tiles_m = (M + BM - 1) / BM, tiles_n = (col_end - col_begin + BN - 1) / BN;
  if ((uint64_t)tiles_m * tiles_n > 0x7FFFFFFFull || pairs == 0 || pairs > 65535u) return HIF8_ERR_ARG;
  const uint32_t grid_x = tile_order_grid(tiles_m * tiles_n);  // a whole number of workgroups per die
  hipLaunchKernelGGL((k_gemm_x<WM, WN, TM, TN, EPI, FINE>), dim3(grid_x, pairs), dim3(64 * WM * WN), smem, st, A, B,
                     out, ref, err, M, N, ld, descale, tiles_n, col_begin, batch);
  return finish_launch();
}

template <int EPI>
hif8_status gemm_expanded(const uint16_t* A, const uint16_t* B, void* out, const float* ref, double* err, size_t M,
                          size_t N, size_t ld, float descale, hipStream_t st, const Batch& batch, uint32_t pairs) {
  if (M == 0 || N == 0) return HIF8_OK;
  // 256 rows x ld x 2 bytes of a workgroup's operand panel must fit the 32-bit lane offsets of the tile loads
  if (M > 0x7FFFFFFFu || N > 0x7FFFFFFFu || ld > kMaxLd || ld == 0 || ld % kExpandK != 0) return HIF8_ERR_ARG;
  if (!A || !B) return HIF8_ERR_NULL;
  if (EPI == EPI_ERR ? (!ref || !err) : !out) return HIF8_ERR_NULL;
  if (!aligned_to(A, 16) || !aligned_to(B, 16)) return HIF8_ERR_ARG;
  if (EPI == EPI_ERR && !aligned_to(err, 8)) return HIF8_ERR_ARG;
  if (batch.nb != 0u && ((batch.a_stride % 8) != 0 || (batch.b_stride % 8) != 0)) return HIF8_ERR_ARG;
  int cus = 0;
  hif8_status s = ensure_init(&cus, nullptr);
  if (s != HIF8_OK) return s;
  // 256 x 256 tiles once the launch has one for every compute unit, else 128 x 128 (4 wavefronts, two workgroups
  // per compute unit).  The large tile runs the hand-placed K step: as 2 x 2 wavefronts of 128 x 128 each (a third
  // fewer fragment reads per MFMA) when the launch lasts several rounds, as 2 x 4 wavefronts of 128 x 64 when it is
  // a single round, where the second wavefront per SIMD covers the start and the end of the tile.
  const size_t big_tiles = ((M + 255) / 256) * ((N + 255) / 256) * (size_t)pairs;
  int variant = expanded_variant();
  uint32_t split = 0;
  if (variant == 0 && pairs == 1 && ragged_round_split(M, N, (size_t)cus, &split)) {
    // complete rounds of 256 x 256 tiles, then the remaining columns in 128 x 128 tiles (second launch)
    s = launch_x<2, 2, 4, 4, EPI, 1>(A, B, out, ref, err, (uint32_t)M, (uint32_t)N, (uint32_t)ld, descale, st, batch, pairs,
                                     0u, split);
    if (s != HIF8_OK) return s;
    return launch_x<2, 2, 2, 2, EPI>(A, B, out, ref, err, (uint32_t)M, (uint32_t)N, (uint32_t)ld, descale, st, batch, pairs,
                                     split, (uint32_t)N);
  }
  if (variant == 0) variant = big_tiles >= 2 * (size_t)cus ? 10 : big_tiles >= (size_t)cus ? 11 : 9;
  if (variant == 10)
    return launch_x<2, 2, 4, 4, EPI, 1>(A, B, out, ref, err, (uint32_t)M, (uint32_t)N, (uint32_t)ld, descale, st, batch, pairs);
  if (variant == 11)
    return launch_x<2, 4, 4, 2, EPI, 1>(A, B, out, ref, err, (uint32_t)M, (uint32_t)N, (uint32_t)ld, descale, st, batch, pairs);
  return launch_x<2, 2, 2, 2, EPI>(A, B, out, ref, err, (uint32_t)M, (uint32_t)N, (uint32_t)ld, descale, st, batch, pairs);
}

template hif8_status gemm_expanded<EPI_F32>(const uint16_t*, const uint16_t*, void*, const float*, double*, size_t, size_t,
                                            size_t, float, hipStream_t, const Batch&, uint32_t);
template hif8_status gemm_expanded<EPI_BF16>(const uint16_t*, const uint16_t*, void*, const float*, double*, size_t, size_t,
                                             size_t, float, hipStream_t, const Batch&, uint32_t);
template hif8_status gemm_expanded<EPI_F16>(const uint16_t*, const uint16_t*, void*, const float*, double*, size_t, size_t,
                                            size_t, float, hipStream_t, const Batch&, uint32_t);
template hif8_status gemm_expanded<EPI_ERR>(const uint16_t*, const uint16_t*, void*, const float*, double*, size_t, size_t,
                                            size_t, float, hipStream_t, const Batch&, uint32_t);

// descale = fl32(fl32(1 / scale_a) * fl32(1 / scale_b)), as in the code-operand GEMM
static bool descale_of(float scale_a, float scale_b, float* out) {
  float inv_a = 1.0f, inv_b = 1.0f;
  if (!valid_scale(scale_a, &inv_a) || !valid_scale(scale_b, &inv_b)) return false;
  volatile float ds = inv_a * inv_b;
  *out = ds;
  return (*out > 0.0f) && !std::isinf(*out);
}

template <int EPI>
static hif8_status gemm_expanded_abi(const uint16_t* a, const uint16_t* b, void* out, const float* ref, double* err,
                                     size_t M, size_t N, size_t K, size_t ld, float scale_a, float scale_b,
                                     hipStream_t st) {
  float descale = 1.0f;
  if (!descale_of(scale_a, scale_b, &descale)) return HIF8_ERR_SCALE;
  if (K == 0 || ld < K) return HIF8_ERR_ARG;
  return gemm_expanded<EPI>(a, b, out, ref, err, M, N, ld, descale, st, Batch{0u, 0, 0, 0}, 1u);
}

}  // namespace hif8gemm

using namespace hif8gemm;

extern "C" {

size_t hif8_expanded_ld(size_t K) { return expanded_ld(K); }

hif8_status hif8_expand_bf16(const uint8_t* codes, size_t rows, size_t K, uint16_t* dst, size_t ld,
                             hif8_stream_t stream) {
  return expand_rows(codes, rows, K, dst, ld, (hipStream_t)stream);
}

hif8_status hif8_expand_bf16_t(const uint8_t* codes, size_t rows, size_t cols, uint16_t* dst, size_t ld,
                               hif8_stream_t stream) {
  return expand_cols(codes, rows, cols, dst, ld, (hipStream_t)stream);
}

hif8_status hif8_gemm_expanded_f32(const uint16_t* a, const uint16_t* b, float* out, size_t M, size_t N, size_t K,
                                   size_t ld, float scale_a, float scale_b, hif8_stream_t stream) {
  return gemm_expanded_abi<EPI_F32>(a, b, out, nullptr, nullptr, M, N, K, ld, scale_a, scale_b, (hipStream_t)stream);
}
hif8_status hif8_gemm_expanded_bf16(const uint16_t* a, const uint16_t* b, uint16_t* out, size_t M, size_t N, size_t K,
                                    size_t ld, float scale_a, float scale_b, hif8_stream_t stream) {
  return gemm_expanded_abi<EPI_BF16>(a, b, out, nullptr, nullptr, M, N, K, ld, scale_a, scale_b, (hipStream_t)stream);
}
hif8_status hif8_gemm_expanded_f16(const uint16_t* a, const uint16_t* b, uint16_t* out, size_t M, size_t N, size_t K,
                                   size_t ld, float scale_a, float scale_b, hif8_stream_t stream) {
  return gemm_expanded_abi<EPI_F16>(a, b, out, nullptr, nullptr, M, N, K, ld, scale_a, scale_b, (hipStream_t)stream);
}
hif8_status hif8_gemm_expanded_sqerr(const uint16_t* a, const uint16_t* b, const float* ref, size_t M, size_t N,
                                     size_t K, size_t ld, float scale_a, float scale_b, double* d_err,
                                     hif8_stream_t stream) {
  return gemm_expanded_abi<EPI_ERR>(a, b, nullptr, ref, d_err, M, N, K, ld, scale_a, scale_b, (hipStream_t)stream);
}

}  // extern "C"
