// kernels.hip -- gfx950 (CDNA4) kernels of the sparse-snapshot hot path.
//
//   k_layout_scan  packed-snapshot layout of a slot: exclusive prefix sums of the aligned
//                  segment sizes (segment offsets) and of the per-segment tile counts
//                  (tile -> segment map), wavefront-level scans combined through LDS.
//   k_pack         Sec. 3.2 sparse snapshot: gather of per-operator segments into one
//                  contiguous buffer.  Persistent workgroups walk the tile list; the
//                  tile -> segment table is staged in LDS; 128-bit streaming loads/stores.
//   k_unpack       Sec. 3.3 snapshot load: the inverse scatter, fused with the
//                  master -> bf16 compute-weight refresh of newly active operators and the
//                  active/frozen mask update.
//   k_adam         Sec. 3.3 replay: fused multi-tensor Adam step over the active operators
//                  (plain FP32 VALU work; nothing here is a contraction, so no MFMA).
//
// All four are bandwidth kernels: zero reuse, so the design goal is many independent
// 16-byte accesses in flight per lane, full-wave coalescing, and an even spread of tiles over
// all compute units whatever the segment sizes are.
#include "kernels.hpp"

namespace moev {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

namespace {

constexpr uint32_t kVec = 16;                       // bytes per lane access
constexpr uint32_t kRow = kThreads * kVec;          // bytes one workgroup moves per access wave

template <bool NT, typename T>
__device__ __forceinline__ T ld(const T* p) {
  if constexpr (NT) return __builtin_nontemporal_load(p);
  else return *p;
}
template <bool NT, typename T>
__device__ __forceinline__ void st(T* p, T v) {
  if constexpr (NT) __builtin_nontemporal_store(v, p);
  else *p = v;
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

// bfloat16 bits of an FP32 value, round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ uint32_t bf16_bits(float x) {
  const uint32_t u = __float_as_uint(x);
  if ((u & 0x7fffffffu) > 0x7f800000u) return (u >> 16) | 0x0040u;
  return (u + 0x7fffu + ((u >> 16) & 1u)) >> 16;
}

// ------------------------------------------------------------------------------------
// layout scan
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

__global__ __launch_bounds__(kThreads) void k_layout_scan(const ScanJob* __restrict__ jobs) {
  const ScanJob job = jobs[blockIdx.x];
  __shared__ uint64_t wave_total[2][kThreads / 64];
  const uint32_t lane = threadIdx.x & 63u, wave = threadIdx.x >> 6;
  uint64_t carry_bytes = job.first, carry_tiles = 0;
  for (uint32_t base = 0; base < job.n; base += kThreads) {
    const uint32_t i = base + threadIdx.x;
    uint64_t padded = 0, tiles = 0;
    if (i < job.n) {
      padded = round_up64(job.sizes[static_cast<uint64_t>(i) * job.stride], job.gran);
      tiles = (padded + job.tile - 1) / job.tile;
    }
    const uint64_t incl_bytes = wave_inclusive_scan(padded);
    const uint64_t incl_tiles = wave_inclusive_scan(tiles);
    if (lane == 63) {
      wave_total[0][wave] = incl_bytes;
      wave_total[1][wave] = incl_tiles;
    }
    __syncthreads();
    uint64_t before_bytes = carry_bytes, before_tiles = carry_tiles, all_bytes = 0, all_tiles = 0;
#pragma unroll
    for (uint32_t w = 0; w < kThreads / 64; ++w) {
      if (w < wave) {
        before_bytes += wave_total[0][w];
        before_tiles += wave_total[1][w];
      }
      all_bytes += wave_total[0][w];
      all_tiles += wave_total[1][w];
    }
    if (i < job.n) {
      if (job.prefix_out) job.prefix_out[i] = before_bytes + incl_bytes - padded;
      job.tile_start_out[i] = static_cast<uint32_t>(before_tiles + incl_tiles - tiles);
    }
    carry_bytes += all_bytes;
    carry_tiles += all_tiles;
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    job.tile_start_out[job.n] = static_cast<uint32_t>(carry_tiles);
    if (job.total_out) *job.total_out = carry_bytes;
  }
}

// ------------------------------------------------------------------------------------
// pack (gather) and unpack (scatter)
// ------------------------------------------------------------------------------------
constexpr uint32_t kCopyUnroll = 8;  // 16-byte accesses in flight per lane

// 16 bytes of a dense tensor at byte offset `o`; bytes at or beyond `nbytes` read as zero.
template <bool NT>
__device__ __forceinline__ u32x4 load_dense(const uint8_t* __restrict__ src, uint64_t o, uint64_t nbytes) {
  if (o + kVec <= nbytes) return ld<NT>(reinterpret_cast<const u32x4*>(src + o));
  u32x4 r = {0u, 0u, 0u, 0u};
  if (o < nbytes) {
    const uint32_t left = static_cast<uint32_t>(nbytes - o);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    for (uint32_t b = 0; b < left; ++b) w[b >> 2] |= static_cast<uint32_t>(src[o + b]) << (8 * (b & 3));
    r = u32x4{w[0], w[1], w[2], w[3]};
  }
  return r;
}

// Stages the tile_start table into LDS (if it fits) and returns the table to search.
__device__ __forceinline__ const uint32_t* stage_table(const uint32_t* __restrict__ global_table,
                                                       uint32_t lds_entries, uint32_t* lds) {
  if (lds_entries == 0) return global_table;
  for (uint32_t i = threadIdx.x; i < lds_entries; i += kThreads) lds[i] = global_table[i];
  __syncthreads();
  return nullptr;  // caller uses the LDS copy
}

template <bool NT>
__global__ __launch_bounds__(kThreads) void k_pack(const CopyArgs a) {
  extern __shared__ uint32_t lds_start[];
  const uint32_t tid = threadIdx.x;
  const bool in_global = stage_table(a.tile_start, a.lds_entries, lds_start) != nullptr;
  const uint32_t n_tiles = a.tile_start[a.n_seg];

  if (blockIdx.x == 0) {
    // header (32 eight-byte words) and, for alignments above 256, the gap before the first segment
    if (tid < 32) {
      uint64_t w = 0;
#pragma unroll
      for (uint32_t k = 0; k < 7; ++k)
        if (tid == k) w = a.header[k];
      reinterpret_cast<uint64_t*>(a.packed)[tid] = w;
    }
    const uint64_t first = round_up64(256, a.align);
    for (uint64_t o = 256 + static_cast<uint64_t>(tid) * kVec; o < first; o += kRow)
      *reinterpret_cast<u32x4*>(a.packed + o) = u32x4{0u, 0u, 0u, 0u};
  }

  for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const uint32_t j = in_global ? owner_of_tile(a.tile_start, a.n_seg, tile)
                                 : owner_of_tile(lds_start, a.n_seg, tile);
    const uint32_t local = tile - (in_global ? a.tile_start[j] : lds_start[j]);
    const SegDesc seg = a.segs[j];
    const uint8_t* __restrict__ src =
        static_cast<const uint8_t*>(a.ptrs[static_cast<uint64_t>(seg.kind) * a.n_tensors + seg.tensor]);
    uint8_t* __restrict__ dst = a.packed + a.dst_off[j];
    const uint64_t padded = round_up64(seg.nbytes, a.align);
    const uint64_t begin = static_cast<uint64_t>(local) * a.tile_bytes;
    const uint64_t end = begin + a.tile_bytes < padded ? begin + a.tile_bytes : padded;

    for (uint64_t base = begin + static_cast<uint64_t>(tid) * kVec; base < end; base += kRow * kCopyUnroll) {
      u32x4 r[kCopyUnroll];
#pragma unroll
      for (uint32_t u = 0; u < kCopyUnroll; ++u) {
        const uint64_t o = base + static_cast<uint64_t>(u) * kRow;
        if (o < end) r[u] = load_dense<NT>(src, o, seg.nbytes);
      }
#pragma unroll
      for (uint32_t u = 0; u < kCopyUnroll; ++u) {
        const uint64_t o = base + static_cast<uint64_t>(u) * kRow;
        if (o < end) st<NT>(reinterpret_cast<u32x4*>(dst + o), r[u]);
      }
    }
  }
}

template <bool NT>
__global__ __launch_bounds__(kThreads) void k_unpack(const CopyArgs a) {
  extern __shared__ uint32_t lds_start[];
  __shared__ uint32_t header_ok;
  const uint32_t tid = threadIdx.x;

  // Refuse a snapshot that does not belong to this plan and slot: nothing is scattered.
  if (tid == 0) {
    const uint64_t* h = reinterpret_cast<const uint64_t*>(a.packed);
    uint32_t ok = 1;
#pragma unroll
    for (uint32_t k = 0; k < 7; ++k)
      if (k != 3 && h[k] != a.header[k]) ok = 0;  // word 3 is the iteration: any value is fine
    header_ok = ok;
    if (!ok && blockIdx.x == 0) *a.status = 1u;
  }
  __syncthreads();
  if (!header_ok) return;

  const bool in_global = stage_table(a.tile_start, a.lds_entries, lds_start) != nullptr;
  const uint32_t n_tiles = a.tile_start[a.n_seg];

  if (blockIdx.x == 0 && a.mask) {
    // operator state machine: the slot's operators become active, later ones are frozen
    for (uint32_t e = tid; e < a.n_ops; e += kThreads) {
      const uint32_t s = a.slot_of_op[e];
      if (s == a.slot) a.mask[e] = 1;
      else if (s > a.slot) a.mask[e] = 0;
    }
  }

  for (uint32_t tile = blockIdx.x; tile < n_tiles; tile += gridDim.x) {
    const uint32_t j = in_global ? owner_of_tile(a.tile_start, a.n_seg, tile)
                                 : owner_of_tile(lds_start, a.n_seg, tile);
    const uint32_t local = tile - (in_global ? a.tile_start[j] : lds_start[j]);
    const SegDesc seg = a.segs[j];
    uint8_t* __restrict__ dst =
        static_cast<uint8_t*>(a.ptrs[static_cast<uint64_t>(seg.kind) * a.n_tensors + seg.tensor]);
    const uint8_t* __restrict__ src = a.packed + a.dst_off[j];
    const bool derive = a.derive_compute && seg.kind == 0u;
    uint8_t* __restrict__ comp =
        derive ? static_cast<uint8_t*>(a.ptrs[3ull * a.n_tensors + seg.tensor]) : nullptr;
    const uint64_t begin = static_cast<uint64_t>(local) * a.tile_bytes;
    uint64_t end = begin + a.tile_bytes;
    if (end > seg.nbytes) end = seg.nbytes;  // padding is never written back

    for (uint64_t base = begin + static_cast<uint64_t>(tid) * kVec; base < end; base += kRow * kCopyUnroll) {
      u32x4 r[kCopyUnroll];
#pragma unroll
      for (uint32_t u = 0; u < kCopyUnroll; ++u) {
        const uint64_t o = base + static_cast<uint64_t>(u) * kRow;
        if (o < end) r[u] = ld<NT>(reinterpret_cast<const u32x4*>(src + o));  // padded: always 16 readable bytes
      }
#pragma unroll
      for (uint32_t u = 0; u < kCopyUnroll; ++u) {
        const uint64_t o = base + static_cast<uint64_t>(u) * kRow;
        if (o >= end) continue;
        if (o + kVec <= seg.nbytes) {
          st<NT>(reinterpret_cast<u32x4*>(dst + o), r[u]);
          if (derive) {
            const u32x2 c = {bf16_bits(__uint_as_float(r[u].x)) | (bf16_bits(__uint_as_float(r[u].y)) << 16),
                             bf16_bits(__uint_as_float(r[u].z)) | (bf16_bits(__uint_as_float(r[u].w)) << 16)};
            st<NT>(reinterpret_cast<u32x2*>(comp + (o >> 1)), c);
          }
        } else {
          const uint32_t left = static_cast<uint32_t>(seg.nbytes - o);
          const uint32_t w[4] = {r[u].x, r[u].y, r[u].z, r[u].w};
          for (uint32_t b = 0; b < left; ++b) dst[o + b] = static_cast<uint8_t>(w[b >> 2] >> (8 * (b & 3)));
          if (derive)
            for (uint32_t e = 0; e < left / 4; ++e)
              reinterpret_cast<uint16_t*>(comp + (o >> 1))[e] =
                  static_cast<uint16_t>(bf16_bits(__uint_as_float(w[e])));
        }
      }
    }
  }
}

// ------------------------------------------------------------------------------------
// fused Adam replay
// ------------------------------------------------------------------------------------
constexpr uint32_t kAdamUnroll = 2;  // float4 groups per lane per pass: 8 loads in flight

struct AdamConst {
  float lr, beta1, beta2, eps, one_minus_beta1, one_minus_beta2, bc1, bc2, decay;
  bool has_decay;
};

// One element.  Operation order is part of the contract (every product and sum rounded
// separately; this file is compiled with floating-point contraction off).
__device__ __forceinline__ void adam_element(float& p, float& m, float& v, float g, const AdamConst& c) {
  if (c.has_decay) p = p - c.decay * p;
  m = c.beta1 * m + c.one_minus_beta1 * g;
  const float g2 = g * g;
  v = c.beta2 * v + c.one_minus_beta2 * g2;
  const float m_hat = m / c.bc1;
  const float v_hat = v / c.bc2;
  const float denom = sqrtf(v_hat) + c.eps;
  p = p - c.lr * (m_hat / denom);
}

template <bool NT>
__global__ __launch_bounds__(kThreads) void k_adam(const AdamArgs a) {
  extern __shared__ uint32_t lds_start[];
  const uint32_t tid = threadIdx.x;
  const bool in_global = stage_table(a.tile_start, a.lds_entries, lds_start) != nullptr;
  const uint32_t n_tiles = a.tile_start[a.n_tensors];
  const AdamConst c = {a.lr, a.beta1, a.beta2, a.eps, a.one_minus_beta1, a.one_minus_beta2,
                       a.bc1, a.bc2, a.decay, a.has_decay != 0};

  uint32_t tile = blockIdx.x;
  while (tile < n_tiles) {
    const uint32_t t = in_global ? owner_of_tile(a.tile_start, a.n_tensors, tile)
                                 : owner_of_tile(lds_start, a.n_tensors, tile);
    const uint32_t t_first = in_global ? a.tile_start[t] : lds_start[t];
    const float* __restrict__ G = static_cast<const float*>(a.grads[t]);
    const bool active = a.mask[a.op_of_tensor[t]] != 0;
    if (active && !G && tid == 0) *a.status = 2u;  // an active operator without gradients: reported, skipped
    if (!active || !G) {
      // frozen operator: jump to this workgroup's first tile at or beyond the next tensor
      const uint32_t t_end = in_global ? a.tile_start[t + 1] : lds_start[t + 1];
      const uint32_t skip = (t_end - tile + gridDim.x - 1) / gridDim.x;
      tile += skip * gridDim.x;
      continue;
    }
    const uint64_t numel = a.numel[t];
    float* __restrict__ P = static_cast<float*>(a.ptrs[t]);
    float* __restrict__ M = static_cast<float*>(a.ptrs[static_cast<uint64_t>(a.n_tensors) + t]);
    float* __restrict__ V = static_cast<float*>(a.ptrs[2ull * a.n_tensors + t]);
    uint16_t* __restrict__ C = static_cast<uint16_t*>(a.ptrs[3ull * a.n_tensors + t]);
    const uint64_t begin = static_cast<uint64_t>(tile - t_first) * a.tile_elems;
    const uint64_t end = begin + a.tile_elems < numel ? begin + a.tile_elems : numel;

    for (uint64_t base = begin + 4ull * tid; base < end; base += 4ull * kThreads * kAdamUnroll) {
      f32x4 p[kAdamUnroll], m[kAdamUnroll], v[kAdamUnroll], g[kAdamUnroll];
#pragma unroll
      for (uint32_t u = 0; u < kAdamUnroll; ++u) {
        const uint64_t i = base + 4ull * kThreads * u;
        if (i + 4 <= end) {
          p[u] = ld<NT>(reinterpret_cast<const f32x4*>(P + i));
          m[u] = ld<NT>(reinterpret_cast<const f32x4*>(M + i));
          v[u] = ld<NT>(reinterpret_cast<const f32x4*>(V + i));
          g[u] = ld<NT>(reinterpret_cast<const f32x4*>(G + i));
        }
      }
#pragma unroll
      for (uint32_t u = 0; u < kAdamUnroll; ++u) {
        const uint64_t i = base + 4ull * kThreads * u;
        if (i + 4 <= end) {
#pragma unroll
          for (uint32_t e = 0; e < 4; ++e) {
            float pe = p[u][e], me = m[u][e], ve = v[u][e];
            adam_element(pe, me, ve, g[u][e], c);
            p[u][e] = pe;
            m[u][e] = me;
            v[u][e] = ve;
          }
          st<NT>(reinterpret_cast<f32x4*>(P + i), p[u]);
          st<NT>(reinterpret_cast<f32x4*>(M + i), m[u]);
          st<NT>(reinterpret_cast<f32x4*>(V + i), v[u]);
          const u32x2 cw = {bf16_bits(p[u].x) | (bf16_bits(p[u].y) << 16),
                            bf16_bits(p[u].z) | (bf16_bits(p[u].w) << 16)};
          st<NT>(reinterpret_cast<u32x2*>(C + i), cw);
        } else if (i < end) {
          // ragged tail of a tensor whose length is not a multiple of four
          for (uint64_t e = i; e < end; ++e) {
            float pe = P[e], me = M[e], ve = V[e];
            adam_element(pe, me, ve, G[e], c);
            P[e] = pe;
            M[e] = me;
            V[e] = ve;
            C[e] = static_cast<uint16_t>(bf16_bits(pe));
          }
        }
      }
    }
    tile += gridDim.x;
  }
}

}  // namespace

// ------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------
hipError_t launch_layout_scan(const ScanJob* d_jobs, uint32_t n_jobs, hipStream_t s) {
  if (n_jobs == 0) return hipSuccess;
  hipLaunchKernelGGL(k_layout_scan, dim3(n_jobs), dim3(kThreads), 0, s, d_jobs);
  return hipGetLastError();
}

hipError_t launch_pack(const CopyArgs& a, uint32_t blocks, bool nontemporal, hipStream_t s) {
  const size_t lds = static_cast<size_t>(a.lds_entries) * sizeof(uint32_t);
  if (nontemporal) hipLaunchKernelGGL(k_pack<true>, dim3(blocks), dim3(kThreads), lds, s, a);
  else hipLaunchKernelGGL(k_pack<false>, dim3(blocks), dim3(kThreads), lds, s, a);
  return hipGetLastError();
}

hipError_t launch_unpack(const CopyArgs& a, uint32_t blocks, bool nontemporal, hipStream_t s) {
  const size_t lds = static_cast<size_t>(a.lds_entries) * sizeof(uint32_t);
  if (nontemporal) hipLaunchKernelGGL(k_unpack<true>, dim3(blocks), dim3(kThreads), lds, s, a);
  else hipLaunchKernelGGL(k_unpack<false>, dim3(blocks), dim3(kThreads), lds, s, a);
  return hipGetLastError();
}

hipError_t launch_adam(const AdamArgs& a, uint32_t blocks, bool nontemporal, hipStream_t s) {
  const size_t lds = static_cast<size_t>(a.lds_entries) * sizeof(uint32_t);
  if (nontemporal) hipLaunchKernelGGL(k_adam<true>, dim3(blocks), dim3(kThreads), lds, s, a);
  else hipLaunchKernelGGL(k_adam<false>, dim3(blocks), dim3(kThreads), lds, s, a);
  return hipGetLastError();
}

}  // namespace moev
