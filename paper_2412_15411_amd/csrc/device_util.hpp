// device_util.hpp -- device-side helpers shared by the gfx950 kernels: 128-bit streaming accesses,
// tile -> owner search, the XCD-aware workgroup -> tile mapping, wavefront / workgroup prefix sums.
// Included by the kernel translation units only.
#pragma once

#include "kernels.hpp"

namespace moev {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr uint32_t kVec = 16;  // bytes per lane access

// Tensor pointers come out of pointer tables in memory, so the compiler cannot know their
// address space and would emit flat accesses; every such pointer is device (global) memory.
#define MOEV_GLOBAL __attribute__((address_space(1)))

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T* p) {
  const MOEV_GLOBAL T* g = (const MOEV_GLOBAL T*)(p);
  if constexpr (NT) return __builtin_nontemporal_load(g);
  else return *g;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(T* p, T v) {
  MOEV_GLOBAL T* g = (MOEV_GLOBAL T*)(p);
  if constexpr (NT) __builtin_nontemporal_store(v, g);
  else *g = v;
}

__device__ __forceinline__ uint64_t round_up64(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

// Largest j in [0, n) with start[j] <= tile; requires start[0] <= tile < start[n].
// Empty items (start[j] == start[j+1]) are skipped because the LAST entry not above the tile wins.
template <typename P>
__device__ __forceinline__ uint32_t owner_of_tile(P start, uint32_t n, uint32_t tile) {
  uint32_t lo = 0, hi = n;
  while (hi - lo > 1) {
    const uint32_t mid = (lo + hi) >> 1;
    if (start[mid] <= tile) lo = mid;
    else hi = mid;
  }
  return lo;
}

// Tile of workgroup `b` in a launch over `n` tiles.  Workgroup ids are handed to the 8 XCDs round
// robin, so with the plain mapping (regions 0) every XCD touches every eighth tile.  regions 1: every XCD
// sweeps its own contiguous eighth of the tiles (the replay's default).  regions G >= 2, a power of two:
// chunks of G consecutive tiles are dealt to the XCDs round robin, so every XCD streams runs of G tiles
// while the chip-wide window of addresses in flight stays 8 G tiles wide (pack and unpack: G = 64); the
// grid must then be a multiple of 8 G workgroups.  Measured in one process per workload: no mapping
// loses 1-5 % on every kernel, eighths cost the unpack 3-6 % against chunks of 64 tiles, chunks of 4-16
// tiles are the worst choice.  Returns ~0u for workgroups beyond the last tile.
constexpr uint32_t kXcds = 8;
__device__ __forceinline__ uint32_t tile_of_workgroup(uint32_t b, uint32_t n, uint32_t regions) {
  if (!regions) return b < n ? b : ~0u;
  if (regions > 1) {  // chunks of `regions` (a power of two) consecutive tiles, dealt to the XCDs round robin
    const uint32_t g = 31u - __builtin_clz(regions), idx = b / kXcds;
    const uint32_t tile = ((idx >> g) << (g + 3)) + ((b % kXcds) << g) + (idx & (regions - 1u));
    return tile < n ? tile : ~0u;
  }
  const uint32_t per_xcd = (n + kXcds - 1) / kXcds;
  const uint32_t idx = b / kXcds;
  const uint32_t tile = (b % kXcds) * per_xcd + idx;
  return (idx < per_xcd && tile < n) ? tile : ~0u;
}

// bfloat16 bits of an FP32 value, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t bf16_bits(float x) {
  const uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// ------------------------------------------------------------------------------------
// prefix sums
// ------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t wave_inclusive_scan(uint64_t x) {
  const uint32_t lane = threadIdx.x & 63u;
#pragma unroll
  for (uint32_t d = 1; d < 64; d <<= 1) {
    const uint64_t y = __shfl_up(static_cast<unsigned long long>(x), d, 64);
    if (lane >= d) x += y;
  }
  return x;
}

// Exclusive scan of one value per thread across a 256-thread workgroup; also returns the
// workgroup total.  `lds` holds one slot per wavefront.
__device__ __forceinline__ uint64_t block_exclusive_scan(uint64_t x, uint64_t* lds, uint64_t* total) {
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  const uint64_t incl = wave_inclusive_scan(x);
  if (lane == 63) lds[wave] = incl;
  __syncthreads();
  uint64_t before = 0, all = 0;
#pragma unroll
  for (uint32_t w = 0; w < kThreads / 64; ++w) {
    if (w < wave) before += lds[w];
    all += lds[w];
  }
  __syncthreads();
  *total = all;
  return before + incl - x;
}

// copies the first `lds_entries` entries of a tile map into LDS (fixed-grid kernels); false: search in global memory
__device__ __forceinline__ bool stage_table(const uint32_t* __restrict__ global_table, uint32_t lds_entries,
                                            uint32_t* lds) {
  if (lds_entries == 0) return false;
  for (uint32_t i = threadIdx.x; i < lds_entries; i += kThreads) lds[i] = global_table[i];
  __syncthreads();
  return true;
}

// picks the <threads, unroll> instantiation of a one-tile-per-workgroup kernel (MOEV_LAUNCH_ARGS = its arguments)
#define MOEV_DIRECT_CASE(KERNEL, TT, UU)                                                              \
  if (threads == TT && unroll == UU) {                                                                \
    if (nt) hipLaunchKernelGGL((KERNEL<TT, UU, true>), dim3(blocks), dim3(TT), 0, s, MOEV_LAUNCH_ARGS); \
    else hipLaunchKernelGGL((KERNEL<TT, UU, false>), dim3(blocks), dim3(TT), 0, s, MOEV_LAUNCH_ARGS);   \
    return hipGetLastError();                                                                         \
  }

#define MOEV_DIRECT_ALL(KERNEL)     \
  MOEV_DIRECT_CASE(KERNEL, 64, 1)   \
  MOEV_DIRECT_CASE(KERNEL, 64, 2)   \
  MOEV_DIRECT_CASE(KERNEL, 64, 4)   \
  MOEV_DIRECT_CASE(KERNEL, 128, 1)  \
  MOEV_DIRECT_CASE(KERNEL, 128, 2)  \
  MOEV_DIRECT_CASE(KERNEL, 128, 4)  \
  MOEV_DIRECT_CASE(KERNEL, 256, 1)  \
  MOEV_DIRECT_CASE(KERNEL, 256, 2)  \
  MOEV_DIRECT_CASE(KERNEL, 256, 4)  \
  MOEV_DIRECT_CASE(KERNEL, 512, 1)  \
  MOEV_DIRECT_CASE(KERNEL, 512, 2)  \
  MOEV_DIRECT_CASE(KERNEL, 1024, 1) \
  return hipErrorInvalidValue;

}  // namespace
}  // namespace moev
