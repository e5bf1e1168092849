// copy_kernels.hip -- gfx950 (CDNA4) kernels that move bytes: layout scan, pack, unpack, copy probe.
//
//   k_layout_scan  packed-snapshot layout of a slot: exclusive prefix sums of the aligned
//                  segment sizes (segment offsets) and of the per-segment tile counts
//                  (tile -> segment map), wavefront-level scans combined through LDS.
//   k_pack_*       Sec. 3.2 sparse snapshot: gather of per-operator segments into one
//                  contiguous buffer, 128-bit streaming loads/stores.
//   k_unpack_*     Sec. 3.3 snapshot load: the inverse scatter, fused with the
//                  master -> bf16 compute-weight refresh of newly active operators and the
//                  active/frozen mask update.
//   k_copy_probe   plain contiguous copy: yardstick and counter calibration.
//
// All of these are bandwidth kernels with zero reuse.  Two launch shapes exist for each:
//   *_direct      one small tile (4-16 KB of each stream) per workgroup, grid = number of
//                 tiles; the tile -> segment map is searched with scalar loads (the table is a
//                 few KB and stays in the scalar/L2 caches).  The hardware dispatcher then
//                 keeps the chip-wide window of in-flight addresses small, contiguous and
//                 moving linearly, which is what HBM rewards (fewest DRAM row conflicts).
//   *_persistent  a fixed grid of workgroups walks the tile list with a stride; the map is
//                 staged in LDS once per workgroup.  Useful when compute units must be left
//                 to a concurrent kernel (the grid is the knob); slower when alone.
#include "device_util.hpp"

namespace moev {
namespace {

__global__ __launch_bounds__(kThreads) void k_layout_scan(const ScanJob* __restrict__ jobs) {
  const ScanJob job = jobs[blockIdx.x];
  __shared__ uint64_t lds_bytes[kThreads / 64], lds_tiles[kThreads / 64];
  uint64_t carry_bytes = job.first, carry_tiles = 0;
  for (uint32_t base = 0; base < job.n; base += kThreads) {
    const uint32_t i = base + threadIdx.x;
    uint64_t padded = 0, tiles = 0;
    if (i < job.n) {
      padded = round_up64(job.sizes[static_cast<uint64_t>(i) * job.stride], job.gran);
      tiles = (padded + job.tile - 1) / job.tile;
    }
    uint64_t all_bytes, all_tiles;
    const uint64_t excl_bytes = block_exclusive_scan(padded, lds_bytes, &all_bytes);
    const uint64_t excl_tiles = block_exclusive_scan(tiles, lds_tiles, &all_tiles);
    if (i < job.n) {
      if (job.prefix_out) job.prefix_out[i] = carry_bytes + excl_bytes;
      job.tile_start_out[i] = static_cast<uint32_t>(carry_tiles + excl_tiles);
    }
    carry_bytes += all_bytes;
    carry_tiles += all_tiles;
  }
  if (threadIdx.x == 0) {
    job.tile_start_out[job.n] = static_cast<uint32_t>(carry_tiles);
    if (job.total_out) *job.total_out = carry_bytes;
  }
}
// ------------------------------------------------------------------------------------
// pack (gather) and unpack (scatter): byte range [begin, end) of one segment
// ------------------------------------------------------------------------------------

// 16 bytes of a dense tensor at byte offset `o`; bytes at or beyond `nbytes` read as zero.
template <bool NT>
__device__ __forceinline__ u32x4 load_dense(const uint8_t* __restrict__ src, uint64_t o, uint64_t nbytes) {
  if (o + kVec <= nbytes) return ld<NT>(reinterpret_cast<const u32x4*>(src + o));
  u32x4 r = {0u, 0u, 0u, 0u};
  if (o < nbytes) {
    const uint32_t left = static_cast<uint32_t>(nbytes - o);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    for (uint32_t b = 0; b < left; ++b) w[b >> 2] |= static_cast<uint32_t>(ld<false>(src + o + b)) << (8 * (b & 3));
    r = u32x4{w[0], w[1], w[2], w[3]};
  }
  return r;
}

// dst[begin, end) = src[begin, end) with zeros beyond nbytes; end is a multiple of 16 within
// the segment's padded size.  T threads, U independent accesses in flight per lane.
template <uint32_t T, uint32_t U, bool NT>
__device__ __forceinline__ void pack_range(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst,
                                           uint64_t begin, uint64_t end, uint64_t nbytes) {
  constexpr uint64_t kRow = static_cast<uint64_t>(T) * kVec;
  for (uint64_t base = begin + static_cast<uint64_t>(threadIdx.x) * kVec; base < end; base += kRow * U) {
    u32x4 r[U];
#pragma unroll
    for (uint32_t u = 0; u < U; ++u) {
      const uint64_t o = base + u * kRow;
      if (o < end) r[u] = load_dense<NT>(src, o, nbytes);
    }
#pragma unroll
    for (uint32_t u = 0; u < U; ++u) {
      const uint64_t o = base + u * kRow;
      if (o < end) st<NT>(reinterpret_cast<u32x4*>(dst + o), r[u]);
    }
  }
}

// dst[begin, end) = src[begin, end), end <= nbytes (padding is never written back); for master
// segments of newly active operators `comp` also receives the bf16 cast of every value.
template <uint32_t T, uint32_t U, bool NT>
__device__ __forceinline__ void unpack_range(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst,
                                             uint8_t* __restrict__ comp, uint64_t begin, uint64_t end,
                                             uint64_t nbytes) {
  constexpr uint64_t kRow = static_cast<uint64_t>(T) * kVec;
  for (uint64_t base = begin + static_cast<uint64_t>(threadIdx.x) * kVec; base < end; base += kRow * U) {
    u32x4 r[U];
#pragma unroll
    for (uint32_t u = 0; u < U; ++u) {
      const uint64_t o = base + u * kRow;
      if (o < end) r[u] = ld<NT>(reinterpret_cast<const u32x4*>(src + o));  // padded: always 16 readable bytes
    }
#pragma unroll
    for (uint32_t u = 0; u < U; ++u) {
      const uint64_t o = base + u * kRow;
      if (o >= end) continue;
      if (o + kVec <= nbytes) {
        st<NT>(reinterpret_cast<u32x4*>(dst + o), r[u]);
        if (comp) {
          const u32x2 c = {bf16_bits(__uint_as_float(r[u].x)) | (bf16_bits(__uint_as_float(r[u].y)) << 16),
                           bf16_bits(__uint_as_float(r[u].z)) | (bf16_bits(__uint_as_float(r[u].w)) << 16)};
          st<NT>(reinterpret_cast<u32x2*>(comp + (o >> 1)), c);
        }
      } else {
        const uint32_t left = static_cast<uint32_t>(nbytes - o);
        const uint32_t w[4] = {r[u].x, r[u].y, r[u].z, r[u].w};
        for (uint32_t b = 0; b < left; ++b) st<false>(dst + o + b, static_cast<uint8_t>(w[b >> 2] >> (8 * (b & 3))));
        if (comp)
          for (uint32_t e = 0; e < left / 4; ++e)
            st<false>(reinterpret_cast<uint16_t*>(comp + (o >> 1)) + e, static_cast<uint16_t>(bf16_bits(__uint_as_float(w[e]))));
      }
    }
  }
}

// header (32 eight-byte words) and, for alignments above 256, the zero gap before the first segment
template <uint32_t T>
__device__ __forceinline__ void write_header(const CopyArgs& a) {
  const uint32_t tid = threadIdx.x;
  if (tid < 32) {
    uint64_t w = 0;
#pragma unroll
    for (uint32_t k = 0; k < 7; ++k)
      if (tid == k) w = a.header[k];
    reinterpret_cast<uint64_t*>(a.packed)[tid] = w;
  }
  const uint64_t first = a.align > 256 ? a.align : 256;  // roundup(256, align) for a power of two
  for (uint64_t o = 256 + static_cast<uint64_t>(tid) * kVec; o < first; o += static_cast<uint64_t>(T) * kVec)
    *reinterpret_cast<u32x4*>(a.packed + o) = u32x4{0u, 0u, 0u, 0u};
}

// A snapshot that does not belong to this plan and slot is refused: nothing is scattered.
// (word 3 is the iteration: any value is fine.)  Uniform across the workgroup.
__device__ __forceinline__ bool header_matches(const CopyArgs& a, const uint64_t* __restrict__ h) {
  bool ok = true;
#pragma unroll
  for (uint32_t k = 0; k < 7; ++k)
    if (k != 3 && h[k] != a.header[k]) ok = false;
  return ok;
}

// operator state machine: the slot's operators become active, later ones are frozen
template <uint32_t T>
__device__ __forceinline__ void update_mask(const CopyArgs& a) {
  if (!a.mask) return;
  for (uint32_t e = threadIdx.x; e < a.n_ops; e += T) {
    const uint32_t s = a.slot_of_op[e];
    if (s == a.slot) a.mask[e] = 1;
    else if (s > a.slot) a.mask[e] = 0;
  }
}

// Read-only tables of a copy launch.  They are separate `const __restrict__` kernel parameters
// (not members of the by-value argument block) so that the compiler may fetch them with scalar
// loads: every lookup is uniform across the workgroup.
#define MOEV_COPY_TABLES                                                                        \
  const uint32_t *__restrict__ tile_start, const SegDesc *__restrict__ segs,                    \
      const uint64_t *__restrict__ dst_off, void *const *__restrict__ ptrs
#define MOEV_COPY_TABLE_ARGS tile_start, segs, dst_off, ptrs

template <uint32_t T, uint32_t U, bool NT, typename Table>
__device__ __forceinline__ void pack_tile(const CopyArgs& a, Table start, const SegDesc* __restrict__ segs,
                                          const uint64_t* __restrict__ dst_off, void* const* __restrict__ ptrs,
                                          uint32_t tile) {
  const uint32_t j = owner_of_tile(start, a.n_seg, tile);
  const uint32_t local = tile - start[j];
  const SegDesc seg = segs[j];
  const uint8_t* src = static_cast<const uint8_t*>(ptrs[static_cast<uint64_t>(seg.kind) * a.n_tensors + seg.tensor]);
  uint8_t* dst = a.packed + dst_off[j];
  const uint64_t padded = (seg.nbytes + a.align - 1) & ~static_cast<uint64_t>(a.align - 1);  // align is a power of two
  const uint64_t begin = static_cast<uint64_t>(local) * a.tile_bytes;
  const uint64_t end = begin + a.tile_bytes < padded ? begin + a.tile_bytes : padded;
  pack_range<T, U, NT>(src, dst, begin, end, seg.nbytes);
}

template <uint32_t T, uint32_t U, bool NT, typename Table>
__device__ __forceinline__ void unpack_tile(const CopyArgs& a, Table start, const SegDesc* __restrict__ segs,
                                            const uint64_t* __restrict__ dst_off, void* const* __restrict__ ptrs,
                                            uint32_t tile) {
  const uint32_t j = owner_of_tile(start, a.n_seg, tile);
  const uint32_t local = tile - start[j];
  const SegDesc seg = segs[j];
  uint8_t* dst = static_cast<uint8_t*>(ptrs[static_cast<uint64_t>(seg.kind) * a.n_tensors + seg.tensor]);
  const uint8_t* src = a.packed + dst_off[j];
  uint8_t* comp = (a.derive_compute && seg.kind == 0u) ? static_cast<uint8_t*>(ptrs[3ull * a.n_tensors + seg.tensor])
                                                       : nullptr;
  const uint64_t begin = static_cast<uint64_t>(local) * a.tile_bytes;
  uint64_t end = begin + a.tile_bytes;
  if (end > seg.nbytes) end = seg.nbytes;
  unpack_range<T, U, NT>(src, dst, comp, begin, end, seg.nbytes);
}

// ---- one tile per workgroup ----
template <uint32_t T, uint32_t U, bool NT>
__global__ __launch_bounds__(T) void k_pack_direct(MOEV_COPY_TABLES, const CopyArgs a) {
  if (blockIdx.x == 0) write_header<T>(a);
  const uint32_t tile = tile_of_workgroup(blockIdx.x, tile_start[a.n_seg], a.xcd_regions);
  if (tile != ~0u) pack_tile<T, U, NT>(a, tile_start, segs, dst_off, ptrs, tile);
}

template <uint32_t T, uint32_t U, bool NT>
__global__ __launch_bounds__(T) void k_unpack_direct(MOEV_COPY_TABLES, const uint64_t* __restrict__ header,
                                                     const CopyArgs a) {
  if (!header_matches(a, header)) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *a.status = 1u;
    return;
  }
  if (blockIdx.x == 0) update_mask<T>(a);
  const uint32_t n_tiles = tile_start[a.n_seg];
  const uint32_t tile = tile_of_workgroup(blockIdx.x, n_tiles > a.tile_begin ? n_tiles - a.tile_begin : 0u, a.xcd_regions);
  if (tile != ~0u) unpack_tile<T, U, NT>(a, tile_start, segs, dst_off, ptrs, tile + a.tile_begin);
}

// ---- fixed grid walking the tile list, map staged in LDS ----
constexpr uint32_t kPersistentUnroll = 8;

template <bool NT>
__global__ __launch_bounds__(kThreads) void k_pack_persistent(MOEV_COPY_TABLES, const CopyArgs a) {
  extern __shared__ uint32_t lds_start[];
  const bool in_lds = stage_table(tile_start, a.lds_entries, lds_start);
  const uint32_t n_tiles = tile_start[a.n_seg];
  if (blockIdx.x == 0) write_header<kThreads>(a);
  for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    if (in_lds) pack_tile<kThreads, kPersistentUnroll, NT>(a, lds_start, segs, dst_off, ptrs, tile);
    else pack_tile<kThreads, kPersistentUnroll, NT>(a, tile_start, segs, dst_off, ptrs, tile);
  }
}

template <bool NT>
__global__ __launch_bounds__(kThreads) void k_unpack_persistent(MOEV_COPY_TABLES, const uint64_t* __restrict__ header,
                                                                const CopyArgs a) {
  extern __shared__ uint32_t lds_start[];
  if (!header_matches(a, header)) {
    if (blockIdx.x == 0 && threadIdx.x == 0) *a.status = 1u;
    return;
  }
  const bool in_lds = stage_table(tile_start, a.lds_entries, lds_start);
  const uint32_t n_tiles = tile_start[a.n_seg];
  if (blockIdx.x == 0) update_mask<kThreads>(a);
  for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    if (in_lds) unpack_tile<kThreads, kPersistentUnroll, NT>(a, lds_start, segs, dst_off, ptrs, tile);
    else unpack_tile<kThreads, kPersistentUnroll, NT>(a, tile_start, segs, dst_off, ptrs, tile);
  }
}
// ------------------------------------------------------------------------------------
// plain contiguous copy: the yardstick for the gather/scatter kernels and the known-size
// kernel against which the HBM traffic counters are calibrated
// ------------------------------------------------------------------------------------
// Workgroup -> tile mapping of the probes in their one-tile-per-workgroup form: the one pack and unpack use by default
// (chunks of 64 tiles dealt to the XCDs round robin), so that the yardsticks are not handicapped against the kernels.
constexpr uint32_t kProbeRegions = 64;

template <bool NT>
__global__ __launch_bounds__(kThreads) void k_copy_probe(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst,
                                                         uint64_t nbytes, uint32_t unroll) {
  const uint64_t row = static_cast<uint64_t>(kThreads) * kVec;
  const uint64_t chunk = row * unroll;
  if (unroll == 1) {  // one 4 KB tile per workgroup
    const uint32_t tile = tile_of_workgroup(blockIdx.x, static_cast<uint32_t>((nbytes + chunk - 1) / chunk), kProbeRegions);
    if (tile == ~0u) return;
    const uint64_t begin = tile * chunk;
    pack_range<kThreads, 1, NT>(src, dst, begin, begin + chunk < nbytes ? begin + chunk : nbytes, nbytes);
    return;
  }
  for (uint64_t begin = blockIdx.x * chunk; begin < nbytes; begin += static_cast<uint64_t>(gridDim.x) * chunk) {
    const uint64_t end = begin + chunk < nbytes ? begin + chunk : nbytes;
    pack_range<kThreads, 8, NT>(src, dst, begin, end, nbytes);
  }
}

// One-directional streams of the same access shape (one 4 KB tile per workgroup): what the memory
// system gives a kernel that only reads, or only writes.  Together with the copy they bracket what a
// kernel with a given read : write mix can reach on the box.
template <bool NT>
__global__ __launch_bounds__(kThreads) void k_read_probe(const uint8_t* __restrict__ src, uint8_t* __restrict__ sink,
                                                         uint64_t nbytes) {
  const uint32_t tile = tile_of_workgroup(blockIdx.x, static_cast<uint32_t>((nbytes + kThreads * kVec - 1) / (kThreads * kVec)), kProbeRegions);
  if (tile == ~0u) return;
  const uint64_t o = (static_cast<uint64_t>(tile) * kThreads + threadIdx.x) * kVec;
  if (o + kVec > nbytes) return;
  const u32x4 r = ld<NT>(reinterpret_cast<const u32x4*>(src + o));
  // keeps the load alive: a store that needs two 32-bit coincidences in the data
  if ((r.x ^ r.z) == 0x9e3779b9u && (r.y ^ r.w) == 0x7f4a7c15u) *reinterpret_cast<u32x4*>(sink) = r;
}

template <bool NT>
__global__ __launch_bounds__(kThreads) void k_write_probe(uint8_t* __restrict__ dst, uint64_t nbytes, uint32_t value) {
  const uint32_t tile = tile_of_workgroup(blockIdx.x, static_cast<uint32_t>((nbytes + kThreads * kVec - 1) / (kThreads * kVec)), kProbeRegions);
  if (tile == ~0u) return;
  const uint64_t o = (static_cast<uint64_t>(tile) * kThreads + threadIdx.x) * kVec;
  if (o + kVec > nbytes) return;
  st<NT>(reinterpret_cast<u32x4*>(dst + o), u32x4{value, value, value, value});
}

}  // namespace

// Copy in which every wavefront instruction covers two 512-byte pieces 2^dist_log2 bytes apart (512: 1 KB of consecutive
// bytes; 32768: the geometry of the replay's paired tiles).  The buffers are cut into blocks of twice that distance; wave
// w of a block takes bytes [512 w, 512 w + 512) of both halves.  Pointers aligned to the block size, so the pieces of a
// pair differ in that one address bit.
template <bool NT>
__global__ __launch_bounds__(kThreads) void k_pair_probe(const uint8_t* __restrict__ src, uint8_t* __restrict__ dst,
                                                         uint64_t nbytes, uint32_t dist_log2) {
  const uint32_t tile = tile_of_workgroup(blockIdx.x, static_cast<uint32_t>((nbytes + kThreads * kVec - 1) / (kThreads * kVec)), kProbeRegions);
  if (tile == ~0u) return;
  const uint64_t wave = static_cast<uint64_t>(tile) * (kThreads / 64) + (threadIdx.x >> 6);
  const uint32_t lane = threadIdx.x & 63;
  const uint64_t per_block = 1ull << (dist_log2 - 9);
  const uint64_t o = (wave / per_block) * (2ull << dist_log2) + (static_cast<uint64_t>(lane >> 5) << dist_log2) +
                     (wave % per_block) * 512 + (lane & 31) * kVec;
  if (o + kVec > nbytes) return;
  st<NT>(reinterpret_cast<u32x4*>(dst + o), ld<NT>(reinterpret_cast<const u32x4*>(src + o)));
}

// ------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------
hipError_t launch_stream_probe(int mode, const void* src, void* dst, uint64_t nbytes, uint32_t value, bool nontemporal,
                               hipStream_t s) {
  const uint32_t unit = 8 * kProbeRegions;  // the chunked mapping deals whole rounds of chunks
  const uint32_t blocks = static_cast<uint32_t>(((nbytes + kThreads * kVec - 1) / (kThreads * kVec) + unit - 1) / unit * unit);
  const uint8_t* sp = static_cast<const uint8_t*>(src);
  uint8_t* dp = static_cast<uint8_t*>(dst);
  if (mode == 3) {   // value = log2 of the distance between the two pieces of a wavefront
    if (nontemporal) hipLaunchKernelGGL(k_pair_probe<true>, dim3(blocks), dim3(kThreads), 0, s, sp, dp, nbytes, value);
    else hipLaunchKernelGGL(k_pair_probe<false>, dim3(blocks), dim3(kThreads), 0, s, sp, dp, nbytes, value);
  } else if (mode == 1) {
    if (nontemporal) hipLaunchKernelGGL(k_read_probe<true>, dim3(blocks), dim3(kThreads), 0, s, sp, dp, nbytes);
    else hipLaunchKernelGGL(k_read_probe<false>, dim3(blocks), dim3(kThreads), 0, s, sp, dp, nbytes);
  } else {
    if (nontemporal) hipLaunchKernelGGL(k_write_probe<true>, dim3(blocks), dim3(kThreads), 0, s, dp, nbytes, value);
    else hipLaunchKernelGGL(k_write_probe<false>, dim3(blocks), dim3(kThreads), 0, s, dp, nbytes, value);
  }
  return hipGetLastError();
}

hipError_t launch_layout_scan(const ScanJob* d_jobs, uint32_t n_jobs, hipStream_t s) {
  if (n_jobs == 0) return hipSuccess;
  hipLaunchKernelGGL(k_layout_scan, dim3(n_jobs), dim3(kThreads), 0, s, d_jobs);
  return hipGetLastError();
}

hipError_t launch_copy_probe(const void* src, void* dst, uint64_t nbytes, uint32_t blocks, uint32_t unroll,
                             bool nontemporal, hipStream_t s) {
  const uint8_t* sp = static_cast<const uint8_t*>(src);
  uint8_t* dp = static_cast<uint8_t*>(dst);
  if (unroll == 1) blocks = (blocks + 8 * kProbeRegions - 1) / (8 * kProbeRegions) * (8 * kProbeRegions);
  if (nontemporal) hipLaunchKernelGGL(k_copy_probe<true>, dim3(blocks), dim3(kThreads), 0, s, sp, dp, nbytes, unroll);
  else hipLaunchKernelGGL(k_copy_probe<false>, dim3(blocks), dim3(kThreads), 0, s, sp, dp, nbytes, unroll);
  return hipGetLastError();
}

bool direct_shape_supported(uint32_t threads, uint32_t unroll) {
  return (unroll == 1 && (threads == 64 || threads == 128 || threads == 256 || threads == 512 || threads == 1024)) ||
         (unroll == 2 && (threads == 64 || threads == 128 || threads == 256 || threads == 512)) ||
         (unroll == 4 && (threads == 64 || threads == 128 || threads == 256));
}

#define MOEV_LAUNCH_ARGS a.tile_start, a.segs, a.dst_off, a.ptrs, a
hipError_t launch_pack_direct(const CopyArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt,
                              hipStream_t s) {
  MOEV_DIRECT_ALL(k_pack_direct)
}
#undef MOEV_LAUNCH_ARGS

#define MOEV_LAUNCH_ARGS a.tile_start, a.segs, a.dst_off, a.ptrs, reinterpret_cast<const uint64_t*>(a.packed), a
hipError_t launch_unpack_direct(const CopyArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt,
                                hipStream_t s) {
  MOEV_DIRECT_ALL(k_unpack_direct)
}
#undef MOEV_LAUNCH_ARGS

hipError_t launch_pack_persistent(const CopyArgs& a, uint32_t blocks, bool nt, hipStream_t s) {
  const size_t lds = static_cast<size_t>(a.lds_entries) * sizeof(uint32_t);
  if (nt) hipLaunchKernelGGL(k_pack_persistent<true>, dim3(blocks), dim3(kThreads), lds, s, a.tile_start, a.segs, a.dst_off, a.ptrs, a);
  else hipLaunchKernelGGL(k_pack_persistent<false>, dim3(blocks), dim3(kThreads), lds, s, a.tile_start, a.segs, a.dst_off, a.ptrs, a);
  return hipGetLastError();
}

hipError_t launch_unpack_persistent(const CopyArgs& a, uint32_t blocks, bool nt, hipStream_t s) {
  const size_t lds = static_cast<size_t>(a.lds_entries) * sizeof(uint32_t);
  const uint64_t* header = reinterpret_cast<const uint64_t*>(a.packed);
  if (nt) hipLaunchKernelGGL(k_unpack_persistent<true>, dim3(blocks), dim3(kThreads), lds, s, a.tile_start, a.segs, a.dst_off, a.ptrs, header, a);
  else hipLaunchKernelGGL(k_unpack_persistent<false>, dim3(blocks), dim3(kThreads), lds, s, a.tile_start, a.segs, a.dst_off, a.ptrs, header, a);
  return hipGetLastError();
}

}  // namespace moev
