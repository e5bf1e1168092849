// kernels.hpp -- launch interface of the gfx950 kernels (layout scan, pack gather, unpack
// scatter, fused Adam replay).  Host code fills the argument blocks; every pointer in them
// is a device pointer.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

namespace moev {

// One segment of a packed snapshot as the kernels see it (16 bytes).
struct SegDesc {
  uint32_t tensor;
  uint32_t kind;    // MOEV_KIND_*
  uint64_t nbytes;
};

// One prefix-sum job, handled by one workgroup: over `n` items with sizes[i * stride],
//   prefix_out[i]     = first + sum_{j<i} roundup(size_j, gran)          (optional)
//   tile_start_out[i] = sum_{j<i} ceil(roundup(size_j, gran) / tile),  i = 0..n
//   *total_out        = first + sum_j roundup(size_j, gran)              (optional)
struct ScanJob {
  const uint64_t* sizes;
  uint64_t* prefix_out;
  uint32_t* tile_start_out;
  uint64_t* total_out;
  uint64_t first, gran, tile;
  uint32_t n, stride;
};

struct CopyArgs {
  const SegDesc* segs;         // the slot's segments
  const uint64_t* dst_off;     // device-computed segment offsets
  const uint32_t* tile_start;  // [n_seg + 1] device-computed
  void* const* ptrs;           // [4 * n_tensors]: kind-major table of dense tensor pointers
  uint8_t* packed;
  uint64_t header[7];          // magic, version | slot << 32, plan hash, iteration, segments, payload, align
  uint32_t n_seg, n_tensors, tile_bytes, align;
  uint32_t lds_entries;        // tile_start entries staged in LDS (0: search in global memory)
  // unpack only
  uint8_t* mask;
  const uint32_t* slot_of_op;
  uint32_t* status;
  uint32_t n_ops, slot, derive_compute;
  uint32_t tile_begin;         // first tile of the launch (unpack of the compute-weight segments only)
  uint32_t xcd_regions;        // 1: every XCD gets a contiguous eighth of the launch's tiles
};

struct AdamArgs {
  const uint32_t* tile_start;  // [n_tensors + 1]: all tensors (fixed grid) or the step's active ones
  const uint64_t* numel;
  const uint32_t* op_of_tensor;
  const uint8_t* mask;
  void* const* ptrs;           // [4 * n_tensors] master, m, v, compute
  void* const* grads;          // [n_tensors]
  uint32_t* status;            // raised when an active operator has no gradient pointer
  // fused load-and-replay only: FP32 state of the newly active tensors is read from the snapshot
  const uint64_t* src_off;     // [3 * n_tensors] offsets of master, m, v in `packed`, ~0 = read the dense tensor
  const uint8_t* packed;
  uint64_t header[7];
  uint32_t n_tensors, tile_elems, lds_entries, has_decay;
  uint32_t xcd_regions;        // as in CopyArgs
  uint32_t paired;             // 64 x 1 shape: paired tiles (per stream and wavefront two pieces of 128 elements, 2^paired ELEMENTS
                               // apart; 13 = 32 KiB for FP32 streams), 0 = consecutive tiles
  uint32_t master_wlog2;       // log2 of the bytes per master-weight element (the paired grid follows the master pointers)
  // state stored in other formats than FP32 / FP32 / FP32 / BF16 (k_adam_lp only)
  const float* scales;         // [4 * n_tensors] kind-major per-tensor scales, or null = all 1
  uint32_t fmt[4];             // kFmt* of master, m, v, compute
  uint32_t plain_divide_sqrt;  // 1: bias corrections and epsilon allow the divisions and the square root in their
                               //    plain form wherever the moments are in the middle exponent range
  float lr, beta1, beta2, eps, one_minus_beta1, one_minus_beta2, bc1, bc2, decay;
};

hipError_t launch_layout_scan(const ScanJob* d_jobs, uint32_t n_jobs, hipStream_t s);
hipError_t launch_copy_probe(const void* src, void* dst, uint64_t nbytes, uint32_t blocks, uint32_t unroll,
                             bool nontemporal, hipStream_t s);

// mode 1: read nbytes from src (dst: 16 writable bytes that may receive one store); mode 2: fill dst[nbytes] with value
hipError_t launch_stream_probe(int mode, const void* src, void* dst, uint64_t nbytes, uint32_t value, bool nontemporal,
                               hipStream_t s);

// one tile per workgroup: grid = number of tiles, tile = threads * 16 bytes (* 4 elements) * unroll
bool direct_shape_supported(uint32_t threads, uint32_t unroll);
hipError_t launch_pack_direct(const CopyArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt,
                              hipStream_t s);
hipError_t launch_unpack_direct(const CopyArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt,
                                hipStream_t s);
hipError_t launch_active_scan(const AdamArgs& a, uint32_t* d_out, hipStream_t s);
hipError_t launch_adam_direct(const AdamArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt,
                              hipStream_t s);
hipError_t launch_adam_fused(const AdamArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt,
                             hipStream_t s);

// Replay on state stored in other formats than FP32 / FP32 / FP32 / BF16: a.fmt = kFmt* of master, m, v,
// compute.  Same tile list and grid as launch_adam_direct (tile = threads * 4 elements * unroll).
bool lp_formats_supported(const uint8_t fmt[4]);
bool lp_shape_supported(uint32_t threads, uint32_t unroll);
hipError_t launch_adam_lp(const AdamArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt, hipStream_t s);

// Counts, into *d_mismatches, the inputs for which the plain division / square root sequences of the
// low-precision replay differ from hipcc's full IEEE expansions (see k_arith_check).
hipError_t launch_arith_check(uint32_t what, float divisor, uint32_t first_bits, uint64_t count, uint64_t seed,
                              unsigned long long* d_mismatches, hipStream_t s);

// fixed grid of 256-thread workgroups walking the tile list
hipError_t launch_pack_persistent(const CopyArgs& a, uint32_t blocks, bool nt, hipStream_t s);
hipError_t launch_unpack_persistent(const CopyArgs& a, uint32_t blocks, bool nt, hipStream_t s);
hipError_t launch_adam_persistent(const AdamArgs& a, uint32_t blocks, bool nt, hipStream_t s);

// storage formats (same values as the C interface's MOEV_FMT_*)
constexpr uint32_t kFmtF32 = 1, kFmtF16 = 2, kFmtBF16 = 3, kFmtE4M3 = 4, kFmtE5M2 = 5;


constexpr uint32_t kThreads = 256;           // 4 wavefronts of 64
constexpr uint32_t kMaxLdsEntries = 8192;    // 32 KB of tile_start in LDS at most; larger tables are searched in global memory

}  // namespace moev
