// Streaming skeleton shared by every HBM-bound kernel of libhif8 (gfx950): 16-byte
// non-temporal accesses, the tile walk of a workgroup, and the wavefront / workgroup
// maximum used by amax.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace hif8dev {

// How a workgroup walks the tiles of a tensor (tile t = vector units [t*tile, (t+1)*tile)):
// workgroup b visits tiles b*first_mul + i*stride for i in [0, count).
//   persistent grid : first_mul = 1, stride = gridDim.x, count = ceil(tiles / gridDim.x)
//   one-shot chunks : first_mul = count = tiles per workgroup, stride = 1; the hardware
//                     dispatcher hands out chunks in address order as workgroups retire, which
//                     keeps the set of DRAM pages being streamed compact.
struct Walk {
  uint32_t first_mul;
  uint32_t stride;
  uint32_t count;
};

// Streaming (non-temporal) 16 / 8 / 4-byte accesses: the data is touched once.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint4 ld_stream(const uint4* p) {
  const u32x4 t = __builtin_nontemporal_load(reinterpret_cast<const u32x4*>(p));
  return make_uint4(t.x, t.y, t.z, t.w);
}
__device__ __forceinline__ uint2 ld_stream(const uint2* p) {
  const u32x2 t = __builtin_nontemporal_load(reinterpret_cast<const u32x2*>(p));
  return make_uint2(t.x, t.y);
}
__device__ __forceinline__ uint32_t ld_stream(const uint32_t* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st_stream(uint4* p, const uint4& v) {
  const u32x4 t = {v.x, v.y, v.z, v.w};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x4*>(p));
}
__device__ __forceinline__ void st_stream(uint2* p, const uint2& v) {
  const u32x2 t = {v.x, v.y};
  __builtin_nontemporal_store(t, reinterpret_cast<u32x2*>(p));
}
__device__ __forceinline__ void st_stream(uint32_t* p, uint32_t v) { __builtin_nontemporal_store(v, p); }

// Vector unit = one 16-byte source load per lane (decode: one lane's worth of codes).  A tile
// is blockDim.x * U vector units.  The first tile's loads are issued before `prologue` (table
// staging + barrier) runs, so the staging latency overlaps with the first HBM round trip.
template <int U, typename V, typename LoadF, typename StoreF, typename PrologueF>
__device__ __forceinline__ void tile_loop(size_t nvec, const Walk w, LoadF load, StoreF store,
                                          PrologueF prologue) {
  const size_t tile = (size_t)blockDim.x * U;
  size_t base = (size_t)blockIdx.x * w.first_mul * tile;
  V v[U];
  auto load_tile = [&](size_t b) {
    const size_t first = b + threadIdx.x;
    if (b + tile <= nvec) {
#pragma unroll
      for (int j = 0; j < U; ++j) v[j] = load(first + (size_t)j * blockDim.x);
    } else {
#pragma unroll
      for (int j = 0; j < U; ++j) {
        const size_t idx = first + (size_t)j * blockDim.x;
        if (idx < nvec) v[j] = load(idx);
      }
    }
  };
  auto store_tile = [&](size_t b) {
    const size_t first = b + threadIdx.x;
    if (b + tile <= nvec) {
#pragma unroll
      for (int j = 0; j < U; ++j) store(first + (size_t)j * blockDim.x, v[j]);
    } else {
#pragma unroll
      for (int j = 0; j < U; ++j) {
        const size_t idx = first + (size_t)j * blockDim.x;
        if (idx < nvec) store(idx, v[j]);
      }
    }
  };
  if (w.count > 0 && base < nvec) load_tile(base);
  prologue();
  for (uint32_t i = 0; i < w.count && base < nvec; ++i) {
    store_tile(base);
    base += (size_t)w.stride * tile;
    if (i + 1 < w.count && base < nvec) load_tile(base);
  }
}

__device__ __forceinline__ uint32_t umax(uint32_t a, uint32_t b) { return a > b ? a : b; }

// Maximum over the 64 lanes of a wavefront with DPP row shifts and row broadcasts; the
// result is valid in lane 63 and returned to every lane through a scalar read of that lane.
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t v) {
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x111, 0xF, 0xF, false));  // row_shr:1
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x112, 0xF, 0xF, false));  // row_shr:2
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x114, 0xF, 0xF, false));  // row_shr:4
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x118, 0xF, 0xF, false));  // row_shr:8
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x142, 0xF, 0xF, false));  // row_bcast:15
  v = umax(v, (uint32_t)__builtin_amdgcn_update_dpp((int)v, (int)v, 0x143, 0xF, 0xF, false));  // row_bcast:31
  return (uint32_t)__builtin_amdgcn_readlane((int)v, 63);
}

// Workgroup maximum of m, valid in thread 0.  Every lane of the workgroup must call it (it contains a barrier).
__device__ __forceinline__ uint32_t block_max_thread0(uint32_t m) {
  __shared__ uint32_t wave_m[16];
  m = wave_max_u32(m);
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  if (lane == 0) wave_m[wave] = m;
  __syncthreads();
  uint32_t r = 0;
  if (threadIdx.x == 0) {
    const uint32_t nw = (blockDim.x + 63u) >> 6;
    r = wave_m[0];
    for (uint32_t w = 1; w < nw; ++w) r = umax(r, wave_m[w]);
  }
  return r;
}
// Workgroup maximum of m, then at most one atomic max into *out: it is skipped when the value read from
// *out just before is already as large.  Atomics of thousands of workgroups on one address are served one
// after the other at the L2 (measured: about 6 ns each -- a BF16 cast of 2^26 elements that accumulates the
// amax of its input took 57.6 us against 32.7 us without; 33.4 us with the check).  The accumulator only
// grows, so a stale read can only cause an atomic that was not needed, never skip one that was.
// CHECK = false (few workgroups per address, e.g. one row chunk each): the atomic whenever the maximum is not zero.
// Every lane of the workgroup must call it (it contains a barrier).
template <bool CHECK = true>
__device__ __forceinline__ void block_max_to_global(uint32_t m, uint32_t* out) {
  const uint32_t r = block_max_thread0(m);
  if (threadIdx.x == 0) {
    if (CHECK ? r > __hip_atomic_load(out, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) : r != 0u) atomicMax(out, r);
  }
}

}  // namespace hif8dev
