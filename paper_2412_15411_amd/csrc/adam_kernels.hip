// adam_kernels.hip -- gfx950 (CDNA4) kernels of the optimizer replay (Sec. 3.3, steps 2, 4, 6).
//
//   k_active_scan  compacts the tile list of a replay step to the active operators that have
//                  gradients (wavefront prefix sum over the per-tensor tile counts).
//   k_adam_*       fused multi-tensor Adam step over the active operators, FP32 state with
//                  bfloat16 compute weights (plain FP32 VALU work; nothing here is a
//                  contraction, so no MFMA); k_adam_fused reads the newly active operators'
//                  state straight from the packed snapshot.
//   k_adam_lp      the same step on state stored in FP16 / BF16 / 8-bit formats (Sec. 5.6).
//   k_arith_check  self-check of the plain division / square-root sequences.
//
// Launch shapes as for the copy kernels: one small tile per workgroup (default) or a fixed
// grid walking the tile list with the tile map staged in LDS.
#include "device_util.hpp"

namespace moev {
namespace {

// ------------------------------------------------------------------------------------
// Paired tiles.  On this part two 512-byte pieces of a stream whose addresses differ only in bit 15
// (32 KiB apart, the lower one with that bit clear) are served markedly faster when they are requested
// together than when each is requested with its neighbours (replay, same process and tensors: +5-10 % over
// consecutive 1 KB tiles; pairs that straddle, i.e. the lower piece has the bit set, are slower than
// consecutive tiles, and so is every other distance from 1 KiB to 4 MiB).  A paired tile is one wavefront's work: lanes 0-31 take 128 consecutive FP32
// elements, lanes 32-63 the 128 elements 2^L further (L = 13: 32 KiB, the default; the distance is a launch
// parameter so that it can be swept); 2^(L-7) such tiles cover a block of 2^(L+1) elements.  The block grid
// is laid over the ADDRESSES of the master weights: element e of a tensor whose master pointer sits `shift`
// elements into a block has grid position e + shift, so that the pairing is right for the master stream and
// for every other stream whose pointer is congruent to it modulo the block size (separately allocated
// tensors usually are); positions below `shift` and beyond the tensor's end are idle lanes.
// ------------------------------------------------------------------------------------
// elements between the start of the address block (2^(L+1) elements of 2^wlog2 bytes) and the tensor's first element
__device__ __forceinline__ uint32_t pair_shift(const void* master, uint32_t L, uint32_t wlog2) {
  return (static_cast<uint32_t>(reinterpret_cast<uintptr_t>(master)) & (((2u << L) << wlog2) - 1u)) >> wlog2;
}
// first element of this lane's quad in paired tile `tile` of a tensor (tiles count from the tensor's first), or ~0 when
// the quad lies in front of the tensor's first element
__device__ __forceinline__ uint64_t paired_quad(uint32_t tile, uint32_t L, uint32_t shift) {
  const uint64_t grid_pos = (static_cast<uint64_t>(tile >> (L - 7)) << (L + 1)) + (static_cast<uint64_t>(threadIdx.x >> 5) << L) +
                            ((tile & ((1u << (L - 7)) - 1u)) << 7) + 4u * (threadIdx.x & 31u);
  return grid_pos >= shift ? grid_pos - shift : ~0ull;  // shift and grid_pos are multiples of four
}
__device__ __forceinline__ uint64_t paired_tiles(uint64_t numel, uint32_t shift, uint32_t L) {
  return numel ? ((numel + shift + (2u << L) - 1) >> (L + 1)) << (L - 7) : 0;
}

// Tile list of one replay step: a tensor contributes its tiles only if its operator is active
// and it has gradients.  out[t] = first compacted tile of tensor t, out[n] = number of tiles.
__global__ __launch_bounds__(kThreads) void k_active_scan(const AdamArgs a, uint32_t* __restrict__ out) {
  // (not hot: one workgroup per replay step)
  __shared__ uint64_t lds[kThreads / 64];
  uint64_t carry = 0;
  for (uint32_t base = 0; base < a.n_tensors; base += kThreads) {
    const uint32_t t = base + threadIdx.x;
    uint64_t tiles = 0;
    if (t < a.n_tensors) {
      const uint64_t numel = a.numel[t];
      const bool active = a.mask[a.op_of_tensor[t]] != 0;
      const bool has_grad = a.grads[t] != nullptr;
      if (active && !has_grad && numel) *a.status = 2u;  // reported by the status query, tensor skipped
      if (active && has_grad) tiles = a.paired ? paired_tiles(numel, pair_shift(a.ptrs[t], a.paired, a.master_wlog2), a.paired) : (numel + a.tile_elems - 1) / a.tile_elems;
    }
    uint64_t all;
    const uint64_t excl = block_exclusive_scan(tiles, lds, &all);
    if (t < a.n_tensors) out[t] = static_cast<uint32_t>(carry + excl);
    carry += all;
  }
  if (threadIdx.x == 0) out[a.n_tensors] = static_cast<uint32_t>(carry);
}

// ------------------------------------------------------------------------------------
// fused Adam replay
// ------------------------------------------------------------------------------------
struct AdamConst {
  float lr, beta1, beta2, eps, one_minus_beta1, one_minus_beta2, bc1, bc2, decay;
  bool has_decay;
};

__device__ __forceinline__ AdamConst adam_const(const AdamArgs& a) {
  return AdamConst{a.lr, a.beta1, a.beta2, a.eps, a.one_minus_beta1, a.one_minus_beta2, a.bc1, a.bc2, a.decay,
                   a.has_decay != 0};
}

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

// ---- correctly rounded division and square root for operands in a middle exponent range ----
// hipcc expands an IEEE FP32 division n / d into: rescaling of both operands (v_div_scale_f32 twice), a
// reciprocal estimate, one Newton step on it, a quotient estimate, two residual corrections with fused
// multiply-adds, the final fused step that also undoes the rescaling (v_div_fmas_f32) and the fix-up of
// the special cases (v_div_fixup_f32).  When neither operand is zero, infinite, NaN or subnormal, the
// exponents differ by less than 96, the numerator is at least 2^-103 and neither 1/d nor n/d is
// subnormal, nothing is rescaled or fixed up, and the sequence reduces to the one below: the same
// instructions on the same values, hence the same (correctly rounded) quotient.  The reciprocal part
// depends on the divisor alone, so a divisor shared by all elements (a bias correction) pays it once.
struct Recip {
  float d, r;  // the divisor and its refined reciprocal
};
__device__ __forceinline__ Recip refined_reciprocal(float d) {
  const float r0 = __builtin_amdgcn_rcpf(d);
  const float e = __builtin_fmaf(-d, r0, 1.0f);
  return Recip{d, __builtin_fmaf(e, r0, r0)};
}
__device__ __forceinline__ float divide_in_range(float n, const Recip& k) {
  const float q0 = n * k.r;
  const float e1 = __builtin_fmaf(-k.d, q0, n);
  const float q1 = __builtin_fmaf(e1, k.r, q0);
  const float e2 = __builtin_fmaf(-k.d, q1, n);
  return __builtin_fmaf(e2, k.r, q1);
}
// Likewise the square root: hipcc's expansion scales arguments below 2^-96 up and the result back,
// and passes zero and infinity through; in between it is the hardware estimate moved by at most one
// unit in the last place according to the signs of two exact residuals.
__device__ __forceinline__ float sqrt_in_range(float x) {
  const float s = __builtin_amdgcn_sqrtf(x);
  const float s_down = __uint_as_float(__float_as_uint(s) - 1u), s_up = __uint_as_float(__float_as_uint(s) + 1u);
  const float r_down = __builtin_fmaf(-s_down, s, x), r_up = __builtin_fmaf(-s_up, s, x);
  float out = r_down <= 0.0f ? s_down : s;
  out = r_up > 0.0f ? s_up : out;
  return out;
}
// Magnitudes in [2^-60, 2^40): with bias corrections in [2^-20, 1] and epsilon in [0, 2^20] every
// division and the square root of the step then stay inside the ranges above
// (m_hat, v_hat in [2^-60, 2^60), sqrt in [2^-30, 2^30), denominator in [2^-30, 2^31)).
constexpr uint32_t kRangeLo = (127u - 60u) << 23, kRangeHi = (127u + 40u) << 23;

// The step of adam_element() on four elements at once, with the divisions and the square root taken in
// their plain form when every updated moment of every active lane of the wavefront is in range (the usual
// case; the decision is uniform across the wavefront, so there is no divergence).
__device__ __forceinline__ void adam_quad(float (&p)[4], float (&m)[4], float (&v)[4], const f32x4& g, const AdamConst& c,
                                          bool plain, const Recip& k1, const Recip& k2) {
  uint32_t lo = ~0u, hi = 0u;
  if (c.has_decay) {
    asm volatile("");  // keeps this a branch (uniform, usually not taken) instead of three selected instructions per element
#pragma unroll
    for (int e = 0; e < 4; ++e) p[e] = p[e] - c.decay * p[e];
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    m[e] = c.beta1 * m[e] + c.one_minus_beta1 * g[e];
    const float g2 = g[e] * g[e];
    v[e] = c.beta2 * v[e] + c.one_minus_beta2 * g2;
    const uint32_t mb = __float_as_uint(m[e]) & 0x7fffffffu, vb = __float_as_uint(v[e]);
    lo = min(lo, min(mb, vb));
    hi = max(hi, max(mb, vb));
  }
  const bool out_of_range = lo < kRangeLo || hi >= kRangeHi;
  if (plain && __builtin_amdgcn_ballot_w64(out_of_range) == 0) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float m_hat = divide_in_range(m[e], k1);
      const float v_hat = divide_in_range(v[e], k2);
      const float denom = sqrt_in_range(v_hat) + c.eps;
      p[e] = p[e] - c.lr * divide_in_range(m_hat, refined_reciprocal(denom));
    }
  } else {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const float m_hat = m[e] / c.bc1;
      const float v_hat = v[e] / c.bc2;
      const float denom = sqrtf(v_hat) + c.eps;
      p[e] = p[e] - c.lr * (m_hat / denom);
    }
  }
}

#define MOEV_ADAM_TABLES                                                                              \
  const uint32_t *__restrict__ tile_start, const uint64_t *__restrict__ numel_of,                     \
      const uint32_t *__restrict__ op_of_tensor, const uint8_t *__restrict__ mask,                    \
      void *const *__restrict__ ptrs, void *const *__restrict__ grads

// Elements [begin, end) of one tensor; begin is a multiple of four.  The old state is read from
// Ps, Ms, Vs (the dense tensors themselves, or their copies inside a packed snapshot) and the new
// state is written to P, M, V, C.
template <uint32_t T, uint32_t U, bool NT>
__device__ __forceinline__ void adam_range(const float* Ps, const float* Ms, const float* Vs,
                                           const float* __restrict__ G, float* P, float* M, float* V,
                                           uint16_t* __restrict__ C, uint64_t begin, uint64_t end, const AdamConst& c,
                                           bool plain) {
  const Recip k1 = refined_reciprocal(c.bc1), k2 = refined_reciprocal(c.bc2);
  for (uint64_t base = begin + 4ull * threadIdx.x; base < end; base += 4ull * T * U) {
    f32x4 p[U], m[U], v[U], g[U];
#pragma unroll
    for (uint32_t u = 0; u < U; ++u) {
      const uint64_t i = base + 4ull * T * u;
      if (i + 4 <= end) {
        p[u] = ld<NT>(reinterpret_cast<const f32x4*>(Ps + i));
        m[u] = ld<NT>(reinterpret_cast<const f32x4*>(Ms + i));
        v[u] = ld<NT>(reinterpret_cast<const f32x4*>(Vs + i));
        g[u] = ld<NT>(reinterpret_cast<const f32x4*>(G + i));
      }
    }
#pragma unroll
    for (uint32_t u = 0; u < U; ++u) {
      const uint64_t i = base + 4ull * T * u;
      if (i + 4 <= end) {
        float pe[4] = {p[u].x, p[u].y, p[u].z, p[u].w}, me[4] = {m[u].x, m[u].y, m[u].z, m[u].w},
              ve[4] = {v[u].x, v[u].y, v[u].z, v[u].w};
        adam_quad(pe, me, ve, g[u], c, plain, k1, k2);
        p[u] = f32x4{pe[0], pe[1], pe[2], pe[3]};
        m[u] = f32x4{me[0], me[1], me[2], me[3]};
        v[u] = f32x4{ve[0], ve[1], ve[2], ve[3]};
        st<NT>(reinterpret_cast<f32x4*>(P + i), p[u]);
        st<NT>(reinterpret_cast<f32x4*>(M + i), m[u]);
        st<NT>(reinterpret_cast<f32x4*>(V + i), v[u]);
        const u32x2 cw = {bf16_bits(p[u].x) | (bf16_bits(p[u].y) << 16), bf16_bits(p[u].z) | (bf16_bits(p[u].w) << 16)};
        st<NT>(reinterpret_cast<u32x2*>(C + i), cw);
      } else if (i < end) {
        // ragged tail of a tensor whose length is not a multiple of four
        for (uint64_t e = i; e < end; ++e) {
          float pe = ld<false>(Ps + e), me = ld<false>(Ms + e), ve = ld<false>(Vs + e);
          adam_element(pe, me, ve, ld<false>(G + e), c);
          st<false>(P + e, pe);
          st<false>(M + e, me);
          st<false>(V + e, ve);
          st<false>(C + e, static_cast<uint16_t>(bf16_bits(pe)));
        }
      }
    }
  }
}

// One paired tile (64 lanes) of one tensor; `tile` counts from the tensor's first tile.
template <bool NT>
__device__ __forceinline__ void adam_tile_paired(const float* Ps, const float* Ms, const float* Vs,
                                                 const float* __restrict__ G, float* P, float* M, float* V,
                                                 uint16_t* __restrict__ C, uint64_t numel, uint32_t L, uint32_t tile,
                                                 const AdamConst& c, bool plain) {
  const uint64_t i = paired_quad(tile, L, pair_shift(P, L, 2));
  if (i == ~0ull) return;
  if (i + 4 <= numel) {
    const Recip k1 = refined_reciprocal(c.bc1), k2 = refined_reciprocal(c.bc2);
    // streaming (nontemporal) accesses for the six FP32 state streams; the gradient load and the bf16 store are plain:
    // measured +0.6 % over streaming everything, while a plain access on any of the state streams costs 4-10 %
    const f32x4 p = ld<NT>(reinterpret_cast<const f32x4*>(Ps + i)), m = ld<NT>(reinterpret_cast<const f32x4*>(Ms + i)),
                v = ld<NT>(reinterpret_cast<const f32x4*>(Vs + i)), g = ld<false>(reinterpret_cast<const f32x4*>(G + i));
    float pe[4] = {p.x, p.y, p.z, p.w}, me[4] = {m.x, m.y, m.z, m.w}, ve[4] = {v.x, v.y, v.z, v.w};
    adam_quad(pe, me, ve, g, c, plain, k1, k2);
    st<NT>(reinterpret_cast<f32x4*>(P + i), f32x4{pe[0], pe[1], pe[2], pe[3]});
    st<NT>(reinterpret_cast<f32x4*>(M + i), f32x4{me[0], me[1], me[2], me[3]});
    st<NT>(reinterpret_cast<f32x4*>(V + i), f32x4{ve[0], ve[1], ve[2], ve[3]});
    const u32x2 cw = {bf16_bits(pe[0]) | (bf16_bits(pe[1]) << 16), bf16_bits(pe[2]) | (bf16_bits(pe[3]) << 16)};
    st<false>(reinterpret_cast<u32x2*>(C + i), cw);
  } else if (i < numel) {
    // ragged tail of a tensor whose length is not a multiple of four
    for (uint64_t e = i; e < numel; ++e) {
      float pe = ld<false>(Ps + e), me = ld<false>(Ms + e), ve = ld<false>(Vs + e);
      adam_element(pe, me, ve, ld<false>(G + e), c);
      st<false>(P + e, pe);
      st<false>(M + e, me);
      st<false>(V + e, ve);
      st<false>(C + e, static_cast<uint16_t>(bf16_bits(pe)));
    }
  }
}

// one tile per workgroup over the compacted tile list written by k_active_scan
template <uint32_t T, uint32_t U, bool NT>
__global__ __launch_bounds__(T) void k_adam_direct(MOEV_ADAM_TABLES, const AdamArgs a) {
  const uint32_t tile = tile_of_workgroup(blockIdx.x, tile_start[a.n_tensors], a.xcd_regions);
  if (tile == ~0u) return;
  const uint32_t t = owner_of_tile(tile_start, a.n_tensors, tile);
  const uint64_t numel = numel_of[t];
  (void)op_of_tensor;
  (void)mask;
  float* P = static_cast<float*>(ptrs[t]);
  float* M = static_cast<float*>(ptrs[static_cast<uint64_t>(a.n_tensors) + t]);
  float* V = static_cast<float*>(ptrs[2ull * a.n_tensors + t]);
  uint16_t* C = static_cast<uint16_t*>(ptrs[3ull * a.n_tensors + t]);
  if constexpr (T == 64 && U == 1) {
    if (a.paired) {
      adam_tile_paired<NT>(P, M, V, static_cast<const float*>(grads[t]), P, M, V, C, numel, a.paired, tile - tile_start[t],
                           adam_const(a), a.plain_divide_sqrt != 0);
      return;
    }
  }
  const uint64_t begin = static_cast<uint64_t>(tile - tile_start[t]) * a.tile_elems;
  const uint64_t end = begin + a.tile_elems < numel ? begin + a.tile_elems : numel;
  adam_range<T, U, NT>(P, M, V, static_cast<const float*>(grads[t]), P, M, V, C, begin, end, adam_const(a),
                       a.plain_divide_sqrt != 0);
}

// Fused snapshot load + replay (steps 1+2, 3+4, 5+6 of the Sec. 3.3 walk-through in one pass): for
// the tensors whose FP32 state the snapshot carries, the old state is read straight from the packed
// buffer instead of being scattered to the dense tensors first and read back.
template <uint32_t T, uint32_t U, bool NT>
__global__ __launch_bounds__(T) void k_adam_fused(MOEV_ADAM_TABLES, const uint64_t* __restrict__ src_off,
                                                  const uint64_t* __restrict__ header, const AdamArgs a) {
  bool ok = true;
#pragma unroll
  for (uint32_t k = 0; k < 7; ++k)
    if (k != 3 && header[k] != a.header[k]) ok = false;
  if (!ok) return;  // foreign snapshot: the unpack launch in front of this one has raised the status word
  const uint32_t tile = tile_of_workgroup(blockIdx.x, tile_start[a.n_tensors], a.xcd_regions);
  if (tile == ~0u) return;
  const uint32_t t = owner_of_tile(tile_start, a.n_tensors, tile);
  const uint64_t numel = numel_of[t];
  (void)op_of_tensor;
  (void)mask;
  float* P = static_cast<float*>(ptrs[t]);
  float* M = static_cast<float*>(ptrs[static_cast<uint64_t>(a.n_tensors) + t]);
  float* V = static_cast<float*>(ptrs[2ull * a.n_tensors + t]);
  uint16_t* C = static_cast<uint16_t*>(ptrs[3ull * a.n_tensors + t]);
  const float *Ps = P, *Ms = M, *Vs = V;
  const uint64_t op = src_off[t];
  if (op != ~0ull) {
    Ps = reinterpret_cast<const float*>(a.packed + op);
    Ms = reinterpret_cast<const float*>(a.packed + src_off[static_cast<uint64_t>(a.n_tensors) + t]);
    Vs = reinterpret_cast<const float*>(a.packed + src_off[2ull * a.n_tensors + t]);
  }
  if constexpr (T == 64 && U == 1) {
    if (a.paired) {
      adam_tile_paired<NT>(Ps, Ms, Vs, static_cast<const float*>(grads[t]), P, M, V, C, numel, a.paired, tile - tile_start[t],
                           adam_const(a), a.plain_divide_sqrt != 0);
      return;
    }
  }
  const uint64_t begin = static_cast<uint64_t>(tile - tile_start[t]) * a.tile_elems;
  const uint64_t end = begin + a.tile_elems < numel ? begin + a.tile_elems : numel;
  adam_range<T, U, NT>(Ps, Ms, Vs, static_cast<const float*>(grads[t]), P, M, V, C, begin, end, adam_const(a),
                       a.plain_divide_sqrt != 0);
}

// fixed grid over the static (all tensors) tile list; frozen tensors are jumped over
template <bool NT>
__global__ __launch_bounds__(kThreads) void k_adam_persistent(MOEV_ADAM_TABLES, const AdamArgs a) {
  extern __shared__ uint32_t lds_start[];
  const bool in_lds = stage_table(tile_start, a.lds_entries, lds_start);
  const uint32_t* start = in_lds ? lds_start : tile_start;  // generic pointer: LDS or global
  const uint32_t n_tiles = tile_start[a.n_tensors];
  const AdamConst c = adam_const(a);
  uint32_t tile = blockIdx.x;
  while (tile < n_tiles) {
    const uint32_t t = owner_of_tile(start, a.n_tensors, tile);
    const bool active = mask[op_of_tensor[t]] != 0;
    const bool has_grad = grads[t] != nullptr;
    if (active && !has_grad && threadIdx.x == 0) *a.status = 2u;
    if (!active || !has_grad) {
      // jump to this workgroup's first tile at or beyond the next tensor
      const uint32_t t_end = start[t + 1];
      tile += (t_end - tile + gridDim.x - 1) / gridDim.x * gridDim.x;
      continue;
    }
    const uint64_t numel = numel_of[t];
    const uint64_t begin = static_cast<uint64_t>(tile - start[t]) * a.tile_elems;
    const uint64_t end = begin + a.tile_elems < numel ? begin + a.tile_elems : numel;
    float* P = static_cast<float*>(ptrs[t]);
    float* M = static_cast<float*>(ptrs[static_cast<uint64_t>(a.n_tensors) + t]);
    float* V = static_cast<float*>(ptrs[2ull * a.n_tensors + t]);
    uint16_t* C = static_cast<uint16_t*>(ptrs[3ull * a.n_tensors + t]);
    adam_range<kThreads, 2, NT>(P, M, V, static_cast<const float*>(grads[t]), P, M, V, C, begin, end, c,
                                a.plain_divide_sqrt != 0);
    tile += gridDim.x;
  }
}

// ------------------------------------------------------------------------------------
// replay on low-precision state (Sec. 5.6 regimes): widen to FP32, the same FP32 step, narrow
// ------------------------------------------------------------------------------------
typedef float f32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef __bf16 bf16x2 __attribute__((ext_vector_type(2)));

// Per storage format: the register holding four consecutive elements, the element type of a
// single (ragged tail) access, and the conversions of four values at a time.  The conversions
// are the hardware's (round to nearest even; FP16 / BF16 overflow to infinity, NaN stays NaN);
// the 8-bit ones do not saturate by themselves (overflow gives NaN / infinity), so the value
// is clamped to the largest finite magnitude first, in a way that lets NaN through.
template <uint32_t F> struct Fmt;

// Keeps the compiler from folding the scale multiplication into the FP16 conversion next to it (a
// mixed-precision fused multiply-add "x * s + 0": one rounding instead of two, and -0 becomes +0).
__device__ __forceinline__ float opaque(float x) {
  asm("" : "+v"(x));
  return x;
}

template <> struct Fmt<kFmtF32> {
  using Quad = u32x4;
  using One = uint32_t;
  static constexpr uint32_t kBytes = 4;
  static __device__ __forceinline__ void widen(const Quad& q, float, float (&x)[4]) {
    x[0] = __uint_as_float(q.x);
    x[1] = __uint_as_float(q.y);
    x[2] = __uint_as_float(q.z);
    x[3] = __uint_as_float(q.w);
  }
  static __device__ __forceinline__ Quad narrow(const float (&x)[4], float) {
    return Quad{__float_as_uint(x[0]), __float_as_uint(x[1]), __float_as_uint(x[2]), __float_as_uint(x[3])};
  }
};

template <> struct Fmt<kFmtF16> {
  using Quad = u32x2;
  using One = uint16_t;
  static constexpr uint32_t kBytes = 2;
  static __device__ __forceinline__ void widen(const Quad& q, float inv, float (&x)[4]) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t pair = h == 0 ? q.x : q.y;  // (a scalar copy: bit_cast straight from a vector element miscompiles)
      const f32x2 w = __builtin_convertvector(__builtin_bit_cast(f16x2, pair), f32x2);
      x[2 * h] = opaque(w.x) * inv;
      x[2 * h + 1] = opaque(w.y) * inv;
    }
  }
  static __device__ __forceinline__ Quad narrow(const float (&x)[4], float s) {
    const uint32_t lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{opaque(x[0] * s), opaque(x[1] * s)}, f16x2));
    const uint32_t hi = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{opaque(x[2] * s), opaque(x[3] * s)}, f16x2));
    return Quad{lo, hi};
  }
};

template <> struct Fmt<kFmtBF16> {
  using Quad = u32x2;
  using One = uint16_t;
  static constexpr uint32_t kBytes = 2;
  static __device__ __forceinline__ void widen(const Quad& q, float inv, float (&x)[4]) {
#pragma unroll
    for (int h = 0; h < 2; ++h) {
      const uint32_t pair = h == 0 ? q.x : q.y;
      x[2 * h] = __uint_as_float(pair << 16) * inv;
      x[2 * h + 1] = __uint_as_float(pair & 0xffff0000u) * inv;
    }
  }
  static __device__ __forceinline__ Quad narrow(const float (&x)[4], float s) {
    const uint32_t lo = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x[0] * s, x[1] * s}, bf16x2));
    const uint32_t hi = __builtin_bit_cast(uint32_t, __builtin_convertvector(f32x2{x[2] * s, x[3] * s}, bf16x2));
    return Quad{lo, hi};
  }
};

// clamp to [-limit, limit]; NaN passes (IEEE 754-2019 minimum / maximum propagate NaN)
__device__ __forceinline__ float clamp_keep_nan(float x, float limit) {
  return __builtin_elementwise_minimum(__builtin_elementwise_maximum(x, -limit), limit);
}

template <> struct Fmt<kFmtE4M3> {   // 4 exponent bits (bias 7), 3 mantissa bits, no infinities, largest value 448
  using Quad = uint32_t;
  using One = uint8_t;
  static constexpr uint32_t kBytes = 1;
  static __device__ __forceinline__ void widen(const Quad& q, float inv, float (&x)[4]) {
    const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_fp8(q, false), hi = __builtin_amdgcn_cvt_pk_f32_fp8(q, true);
    x[0] = lo.x * inv;
    x[1] = lo.y * inv;
    x[2] = hi.x * inv;
    x[3] = hi.y * inv;
  }
  static __device__ __forceinline__ Quad narrow(const float (&x)[4], float s) {
    int q = 0;
    q = __builtin_amdgcn_cvt_pk_fp8_f32(clamp_keep_nan(x[0] * s, 448.0f), clamp_keep_nan(x[1] * s, 448.0f), q, false);
    q = __builtin_amdgcn_cvt_pk_fp8_f32(clamp_keep_nan(x[2] * s, 448.0f), clamp_keep_nan(x[3] * s, 448.0f), q, true);
    return static_cast<Quad>(q);
  }
};

template <> struct Fmt<kFmtE5M2> {   // 5 exponent bits (bias 15), 2 mantissa bits, largest finite value 57344
  using Quad = uint32_t;
  using One = uint8_t;
  static constexpr uint32_t kBytes = 1;
  static __device__ __forceinline__ void widen(const Quad& q, float inv, float (&x)[4]) {
    const f32x2 lo = __builtin_amdgcn_cvt_pk_f32_bf8(q, false), hi = __builtin_amdgcn_cvt_pk_f32_bf8(q, true);
    x[0] = lo.x * inv;
    x[1] = lo.y * inv;
    x[2] = hi.x * inv;
    x[3] = hi.y * inv;
  }
  static __device__ __forceinline__ Quad narrow(const float (&x)[4], float s) {
    int q = 0;
    q = __builtin_amdgcn_cvt_pk_bf8_f32(clamp_keep_nan(x[0] * s, 57344.0f), clamp_keep_nan(x[1] * s, 57344.0f), q, false);
    q = __builtin_amdgcn_cvt_pk_bf8_f32(clamp_keep_nan(x[2] * s, 57344.0f), clamp_keep_nan(x[3] * s, 57344.0f), q, true);
    return static_cast<Quad>(q);
  }
};

struct LpScales {
  float s[4], inv[4];  // scale and its reciprocal (rounded once) of master, m, v, compute
};

// Four elements: codes in, codes out.  The compute weights are cast from the master weights as stored.
template <uint32_t FP, uint32_t FM, uint32_t FV, uint32_t FC>
__device__ __forceinline__ void adam_lp_quad(typename Fmt<FP>::Quad& p, typename Fmt<FM>::Quad& m, typename Fmt<FV>::Quad& v,
                                             typename Fmt<FC>::Quad& cw, const f32x4& g, const LpScales& sc,
                                             const AdamConst& c, bool fast, const Recip& k1, const Recip& k2) {
  float pf[4], mf[4], vf[4];
  Fmt<FP>::widen(p, sc.inv[0], pf);
  Fmt<FM>::widen(m, sc.inv[1], mf);
  Fmt<FV>::widen(v, sc.inv[2], vf);
  adam_quad(pf, mf, vf, g, c, fast, k1, k2);
  p = Fmt<FP>::narrow(pf, sc.s[0]);
  m = Fmt<FM>::narrow(mf, sc.s[1]);
  v = Fmt<FV>::narrow(vf, sc.s[2]);
  float stored[4];
  Fmt<FP>::widen(p, sc.inv[0], stored);
  cw = Fmt<FC>::narrow(stored, sc.s[3]);
}

// a quad whose first element is the single value at `ptr` (ragged tails)
template <uint32_t F>
__device__ __forceinline__ typename Fmt<F>::Quad quad_of_one(const uint8_t* base, uint64_t e) {
  using One = typename Fmt<F>::One;
  typename Fmt<F>::Quad q{};
  const uint32_t bits = ld<false>(reinterpret_cast<const One*>(base) + e);
  if constexpr (Fmt<F>::kBytes == 1) q = bits;
  else q.x = bits;
  return q;
}
template <uint32_t F>
__device__ __forceinline__ void store_first(uint8_t* base, uint64_t e, const typename Fmt<F>::Quad& q) {
  using One = typename Fmt<F>::One;
  uint32_t bits;
  if constexpr (Fmt<F>::kBytes == 1) bits = q;
  else bits = q.x;
  st<false>(reinterpret_cast<One*>(base) + e, static_cast<One>(bits));
}

// The quads at elements pos[0..U) of one tensor (multiples of four; a position at or beyond `end` is skipped), in place.
template <uint32_t FP, uint32_t FM, uint32_t FV, uint32_t FC, uint32_t U, bool NT>
__device__ __forceinline__ void adam_lp_quads(uint8_t* P, uint8_t* M, uint8_t* V, const float* __restrict__ G,
                                              uint8_t* __restrict__ C, const uint64_t (&pos)[U], uint64_t end, const LpScales& sc,
                                              const AdamConst& c, bool fast, const Recip& k1, const Recip& k2) {
  using QP = typename Fmt<FP>::Quad;
  using QM = typename Fmt<FM>::Quad;
  using QV = typename Fmt<FV>::Quad;
  using QC = typename Fmt<FC>::Quad;
  constexpr uint32_t WP = Fmt<FP>::kBytes, WM = Fmt<FM>::kBytes, WV = Fmt<FV>::kBytes, WC = Fmt<FC>::kBytes;
  QP p[U];
  QM m[U];
  QV v[U];
  f32x4 g[U];
#pragma unroll
  for (uint32_t u = 0; u < U; ++u) {
    const uint64_t i = pos[u];
    if (i < end && i + 4 <= end) {
      p[u] = ld<NT>(reinterpret_cast<const QP*>(P + i * WP));
      m[u] = ld<NT>(reinterpret_cast<const QM*>(M + i * WM));
      v[u] = ld<NT>(reinterpret_cast<const QV*>(V + i * WV));
      g[u] = ld<NT>(reinterpret_cast<const f32x4*>(G + i));
    }
  }
#pragma unroll
  for (uint32_t u = 0; u < U; ++u) {
    const uint64_t i = pos[u];
    if (i >= end) continue;
    if (i + 4 <= end) {
      QC cw;
      adam_lp_quad<FP, FM, FV, FC>(p[u], m[u], v[u], cw, g[u], sc, c, fast, k1, k2);
      st<NT>(reinterpret_cast<QP*>(P + i * WP), p[u]);
      st<NT>(reinterpret_cast<QM*>(M + i * WM), m[u]);
      st<NT>(reinterpret_cast<QV*>(V + i * WV), v[u]);
      st<NT>(reinterpret_cast<QC*>(C + i * WC), cw);
    } else {
      // ragged tail of a tensor whose length is not a multiple of four: one element at a time,
      // in the first position of a quad
      for (uint64_t e = i; e < end; ++e) {
        QP p1 = quad_of_one<FP>(P, e);
        QM m1 = quad_of_one<FM>(M, e);
        QV v1 = quad_of_one<FV>(V, e);
        QC c1;
        const f32x4 g1 = {ld<false>(G + e), 0.0f, 0.0f, 0.0f};
        adam_lp_quad<FP, FM, FV, FC>(p1, m1, v1, c1, g1, sc, c, false, k1, k2);
        store_first<FP>(P, e, p1);
        store_first<FM>(M, e, m1);
        store_first<FV>(V, e, v1);
        store_first<FC>(C, e, c1);
      }
    }
  }
}

// Elements [begin, end) of one tensor, in place; begin is a multiple of four.
template <uint32_t FP, uint32_t FM, uint32_t FV, uint32_t FC, uint32_t T, uint32_t U, bool NT>
__device__ __forceinline__ void adam_lp_range(uint8_t* P, uint8_t* M, uint8_t* V, const float* __restrict__ G,
                                              uint8_t* __restrict__ C, uint64_t begin, uint64_t end, const LpScales& sc,
                                              const AdamConst& c, bool fast) {
  const Recip k1 = refined_reciprocal(c.bc1), k2 = refined_reciprocal(c.bc2);
  for (uint64_t base = begin + 4ull * threadIdx.x; base < end; base += 4ull * T * U) {
    uint64_t pos[U];
#pragma unroll
    for (uint32_t u = 0; u < U; ++u) pos[u] = base + 4ull * T * u;
    adam_lp_quads<FP, FM, FV, FC, U, NT>(P, M, V, G, C, pos, end, sc, c, fast, k1, k2);
  }
}

// one tile per workgroup over the compacted tile list written by k_active_scan
template <uint32_t FP, uint32_t FM, uint32_t FV, uint32_t FC, uint32_t T, uint32_t U, bool NT>
__global__ __launch_bounds__(T) void k_adam_lp(MOEV_ADAM_TABLES, const float* __restrict__ scales, const AdamArgs a) {
  const uint32_t tile = tile_of_workgroup(blockIdx.x, tile_start[a.n_tensors], a.xcd_regions);
  if (tile == ~0u) return;
  const uint32_t t = owner_of_tile(tile_start, a.n_tensors, tile);
  const uint64_t numel = numel_of[t];
  const uint64_t begin = static_cast<uint64_t>(tile - tile_start[t]) * a.tile_elems;
  const uint64_t end = begin + a.tile_elems < numel ? begin + a.tile_elems : numel;
  (void)op_of_tensor;
  (void)mask;
  LpScales sc;
#pragma unroll
  for (uint32_t k = 0; k < 4; ++k) {
    sc.s[k] = scales ? scales[static_cast<uint64_t>(k) * a.n_tensors + t] : 1.0f;
    sc.inv[k] = 1.0f / sc.s[k];
  }
  if constexpr (T == 64 && U == 1) {
    if (a.paired) {   // paired tile: this lane's quad of the tensor, see adam_tile_paired
      uint8_t* P = static_cast<uint8_t*>(ptrs[t]);
      constexpr uint32_t kMasterLog2 = Fmt<FP>::kBytes == 4 ? 2u : Fmt<FP>::kBytes == 2 ? 1u : 0u;
      const uint64_t pos[1] = {paired_quad(tile - tile_start[t], a.paired, pair_shift(P, a.paired, kMasterLog2))};
      if (pos[0] == ~0ull) return;
      const AdamConst c = adam_const(a);
      adam_lp_quads<FP, FM, FV, FC, 1, NT>(P, static_cast<uint8_t*>(ptrs[static_cast<uint64_t>(a.n_tensors) + t]),
                                           static_cast<uint8_t*>(ptrs[2ull * a.n_tensors + t]), static_cast<const float*>(grads[t]),
                                           static_cast<uint8_t*>(ptrs[3ull * a.n_tensors + t]), pos, numel, sc, c,
                                           a.plain_divide_sqrt != 0, refined_reciprocal(c.bc1), refined_reciprocal(c.bc2));
      return;
    }
  }
  adam_lp_range<FP, FM, FV, FC, T, U, NT>(static_cast<uint8_t*>(ptrs[t]),
                                          static_cast<uint8_t*>(ptrs[static_cast<uint64_t>(a.n_tensors) + t]),
                                          static_cast<uint8_t*>(ptrs[2ull * a.n_tensors + t]),
                                          static_cast<const float*>(grads[t]),
                                          static_cast<uint8_t*>(ptrs[3ull * a.n_tensors + t]), begin, end, sc,
                                          adam_const(a), a.plain_divide_sqrt != 0);
}

// ------------------------------------------------------------------------------------
// self-check of divide_in_range / sqrt_in_range against hipcc's full IEEE expansions
// ------------------------------------------------------------------------------------
__device__ __forceinline__ uint64_t mix64(uint64_t x) {
  x += 0x9e3779b97f4a7c15ull;
  x = (x ^ (x >> 30)) * 0xbf58476d1ce4e5b9ull;
  x = (x ^ (x >> 27)) * 0x94d049bb133111ebull;
  return x ^ (x >> 31);
}

// what 0: n / divisor for the `count` consecutive FP32 patterns n starting at first_bits, both signs;
// what 1: sqrt(x) for those patterns; what 2: n / d for `count` pseudo-random pairs with |n| in
// [2^-60, 2^60) and d in [2^-30, 2^31) (the ranges the replay's last division sees).
__global__ __launch_bounds__(kThreads) void k_arith_check(uint32_t what, float divisor, uint32_t first_bits, uint64_t count,
                                                          uint64_t seed, unsigned long long* __restrict__ mismatches) {
  const Recip k = refined_reciprocal(divisor);
  unsigned long long bad = 0;
  for (uint64_t i = static_cast<uint64_t>(blockIdx.x) * kThreads + threadIdx.x; i < count;
       i += static_cast<uint64_t>(gridDim.x) * kThreads) {
    if (what == 0) {
      const float n = __uint_as_float(first_bits + static_cast<uint32_t>(i));
      bad += __float_as_uint(divide_in_range(n, k)) != __float_as_uint(n / divisor);
      bad += __float_as_uint(divide_in_range(-n, k)) != __float_as_uint(-n / divisor);
    } else if (what == 1) {
      const float x = __uint_as_float(first_bits + static_cast<uint32_t>(i));
      bad += __float_as_uint(sqrt_in_range(x)) != __float_as_uint(sqrtf(x));
    } else {
      const uint64_t h = mix64(seed ^ mix64(i));
      const uint32_t n_bits = (static_cast<uint32_t>(h) % (120u << 23)) + ((127u - 60u) << 23);
      const uint32_t d_bits = (static_cast<uint32_t>(h >> 32) % (61u << 23)) + ((127u - 30u) << 23);
      const float n = __uint_as_float(n_bits | (static_cast<uint32_t>(h >> 31) & 0x80000000u)), d = __uint_as_float(d_bits);
      bad += __float_as_uint(divide_in_range(n, refined_reciprocal(d))) != __float_as_uint(n / d);
    }
  }
  if (bad) atomicAdd(mismatches, bad);
}

}  // namespace

// ------------------------------------------------------------------------------------
// launchers
// ------------------------------------------------------------------------------------
#define MOEV_LAUNCH_ARGS a.tile_start, a.numel, a.op_of_tensor, a.mask, a.ptrs, a.grads, a
hipError_t launch_adam_direct(const AdamArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt,
                              hipStream_t s) {
  MOEV_DIRECT_ALL(k_adam_direct)
}
#undef MOEV_LAUNCH_ARGS

#define MOEV_LAUNCH_ARGS \
  a.tile_start, a.numel, a.op_of_tensor, a.mask, a.ptrs, a.grads, a.src_off, reinterpret_cast<const uint64_t*>(a.packed), a
hipError_t launch_adam_fused(const AdamArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt,
                             hipStream_t s) {
  MOEV_DIRECT_ALL(k_adam_fused)
}
#undef MOEV_LAUNCH_ARGS

// ---- replay on low-precision state: dispatch over format combinations and launch shapes ----
bool lp_shape_supported(uint32_t threads, uint32_t unroll) {
  return (threads == 64 || threads == 128 || threads == 256) && (unroll == 1 || unroll == 2);
}

namespace {

constexpr uint32_t lp_key(uint32_t p, uint32_t m, uint32_t v, uint32_t c) { return ((p * 8 + m) * 8 + v) * 8 + c; }

template <uint32_t FP, uint32_t FM, uint32_t FV, uint32_t FC>
hipError_t launch_adam_lp_formats(const AdamArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt,
                                  hipStream_t s) {
#define MOEV_LP_CASE(TT, UU)                                                                                         \
  if (threads == TT && unroll == UU) {                                                                               \
    if (nt) hipLaunchKernelGGL((k_adam_lp<FP, FM, FV, FC, TT, UU, true>), dim3(blocks), dim3(TT), 0, s, a.tile_start, a.numel, \
                               a.op_of_tensor, a.mask, a.ptrs, a.grads, a.scales, a);                                \
    else hipLaunchKernelGGL((k_adam_lp<FP, FM, FV, FC, TT, UU, false>), dim3(blocks), dim3(TT), 0, s, a.tile_start, a.numel,   \
                            a.op_of_tensor, a.mask, a.ptrs, a.grads, a.scales, a);                                   \
    return hipGetLastError();                                                                                        \
  }
  MOEV_LP_CASE(64, 1)
  MOEV_LP_CASE(64, 2)
  MOEV_LP_CASE(128, 1)
  MOEV_LP_CASE(128, 2)
  MOEV_LP_CASE(256, 1)
  MOEV_LP_CASE(256, 2)
#undef MOEV_LP_CASE
  return hipErrorInvalidValue;
}

// the format combinations (master, m, v, compute) that have a kernel
#define MOEV_LP_COMBOS(X)                         \
  X(kFmtF32, kFmtF32, kFmtF32, kFmtF16)           \
  X(kFmtF16, kFmtF16, kFmtF16, kFmtF16)           \
  X(kFmtF16, kFmtF16, kFmtF16, kFmtBF16)          \
  X(kFmtF32, kFmtF32, kFmtF32, kFmtE4M3)          \
  X(kFmtF16, kFmtF32, kFmtF32, kFmtE4M3)          \
  X(kFmtF16, kFmtE4M3, kFmtF16, kFmtE4M3)         \
  X(kFmtE4M3, kFmtE4M3, kFmtF16, kFmtE4M3)        \
  X(kFmtBF16, kFmtBF16, kFmtBF16, kFmtBF16)       \
  X(kFmtF16, kFmtE5M2, kFmtF16, kFmtE5M2)         \
  X(kFmtE5M2, kFmtE4M3, kFmtBF16, kFmtE5M2)

}  // namespace

bool lp_formats_supported(const uint8_t f[4]) {
  switch (lp_key(f[0], f[1], f[2], f[3])) {
#define MOEV_LP_X(P, M, V, C) case lp_key(P, M, V, C):
    MOEV_LP_COMBOS(MOEV_LP_X)
#undef MOEV_LP_X
    return true;
    default: return false;
  }
}

hipError_t launch_adam_lp(const AdamArgs& a, uint32_t blocks, uint32_t threads, uint32_t unroll, bool nt, hipStream_t s) {
  switch (lp_key(a.fmt[0], a.fmt[1], a.fmt[2], a.fmt[3])) {
#define MOEV_LP_X(P, M, V, C) case lp_key(P, M, V, C): return launch_adam_lp_formats<P, M, V, C>(a, blocks, threads, unroll, nt, s);
    MOEV_LP_COMBOS(MOEV_LP_X)
#undef MOEV_LP_X
    default: return hipErrorInvalidValue;
  }
}

hipError_t launch_arith_check(uint32_t what, float divisor, uint32_t first_bits, uint64_t count, uint64_t seed,
                              unsigned long long* d_mismatches, hipStream_t s) {
  hipLaunchKernelGGL(k_arith_check, dim3(256 * 16), dim3(kThreads), 0, s, what, divisor, first_bits, count, seed, d_mismatches);
  return hipGetLastError();
}

hipError_t launch_active_scan(const AdamArgs& a, uint32_t* d_out, hipStream_t s) {
  hipLaunchKernelGGL(k_active_scan, dim3(1), dim3(kThreads), 0, s, a, d_out);
  return hipGetLastError();
}

hipError_t launch_adam_persistent(const AdamArgs& a, uint32_t blocks, bool nt, hipStream_t s) {
  const size_t lds = static_cast<size_t>(a.lds_entries) * sizeof(uint32_t);
  if (nt) hipLaunchKernelGGL(k_adam_persistent<true>, dim3(blocks), dim3(kThreads), lds, s, a.tile_start, a.numel, a.op_of_tensor, a.mask, a.ptrs, a.grads, a);
  else hipLaunchKernelGGL(k_adam_persistent<false>, dim3(blocks), dim3(kThreads), lds, s, a.tile_start, a.numel, a.op_of_tensor, a.mask, a.ptrs, a.grads, a);
  return hipGetLastError();
}

}  // namespace moev
