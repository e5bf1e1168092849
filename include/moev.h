/*
 * moev.h -- C ABI of libmoev: sparse snapshot of MoE expert state and sparse-to-dense
 * checkpoint conversion (MoEvement, arXiv 2412.15411) on one MI355X (gfx950).
 *
 * The five calls follow the paper's statement of the problem:
 *   ckpt_plan       Sec. 3.5 / Algorithm 1: window size, operator order, per-slot active and
 *                   frozen sets; plus this library's packed-snapshot layout for every slot.
 *   snapshot_pack   Sec. 3.2: gather the slot's sparse snapshot (full FP32 state of the active
 *                   operators, compute weights of the frozen ones) into one packed buffer.
 *   snapshot_drain  Sec. 3.2 / Sec. 4: move the snapshot to pinned host memory on a side
 *                   stream, overlapped with training.
 *   restore_unpack  Sec. 3.3 (steps 1, 3, 5 of the walk-through): load one sparse snapshot,
 *                   activate the operators whose FP32 state it carries.
 *   convert_replay  Sec. 3.3 (steps 2, 4, 6): one replayed optimizer step on the active
 *                   operators; frozen operators are skipped.
 *
 * Conventions
 *   - Every call returns 0 (MOEV_OK) or a negative MOEV_E_* code; moev_last_error() gives
 *     a thread-local message for the last failure.  No exception crosses the boundary.
 *   - "host" pointers are ordinary process memory; "device" pointers are HIP device memory
 *     of the GPU that was current when the plan was first used on the GPU.
 *   - All data buffers are owned by the caller.  The library owns only the opaque plan and
 *     its small device tables, released by ckpt_plan_free().
 *   - GPU calls enqueue work on the given stream and return; they never synchronise the
 *     device (the two ckpt_plan_device_* queries do, they exist for tests).
 *   - Streams and events are passed as void* (hipStream_t / hipEvent_t); NULL stream = the
 *     default stream.
 *   - There is no CPU fallback: GPU calls fail with MOEV_E_HIP when no device is usable.
 *   - A plan may be used from several host threads (its calls are serialised by a mutex) and on
 *     several streams.  Its device tables (layout, tile maps, the cached tables of state and
 *     gradient pointers) are written on the stream of the call that (re)builds them; a later call
 *     on another stream waits for that write.  The pointer tables are shared by all calls on a
 *     plan: a call that passes DIFFERENT state or gradient pointers than the previous one rewrites
 *     them, so it must not be enqueued while a kernel of that plan may still run on ANOTHER
 *     stream (order the streams, or use one plan per concurrently processed state).  Replay
 *     steps (convert_replay, convert_window_step) of ONE plan must be stream-ordered among
 *     themselves even with unchanged pointers: every step rewrites the plan's list of active tiles.
 *   - HIP graphs: a call whose tables are resident (same plan settings, same state and gradient
 *     pointers as an earlier call) enqueues kernels only and may be captured into a graph; pass
 *     every gradient pointer in every iteration (frozen operators' entries are not read) so that
 *     the table does not change.  A call that would have to build or upload a table while its
 *     stream is capturing fails with MOEV_E_INVAL and records nothing.  Calls given a pinned host
 *     snapshot (h_pinned) record a host-to-device copy node.
 *
 * Packed snapshot format (this library's definition; the paper copies per operator and
 * defines none).  Little endian.
 *   [256-byte header][segment 0][zero pad][segment 1][zero pad]...
 *   header: +0 u64 magic "MOEVSNAP", +8 u32 version = 1, +12 u32 slot, +16 u64 plan hash,
 *           +24 u64 iteration, +32 u64 segment count, +40 u64 payload bytes (all bytes after
 *           the header), +48 u32 align, rest zero.
 *   segments of slot k: walking the checkpoint order, for every operator active in slot k and
 *           each of its tensors: master, Adam m, Adam v; then, walking the order again, for
 *           every operator active in a later slot and each of its tensors: compute weights.
 *   offsets: first segment at roundup(256, align); each next one roundup(nbytes, align)
 *           further; padding bytes are zero.
 *   plan hash: 64-bit FNV-1a over u32 n_ops, u32 n_tensors, u32 window, u32 align, u8 element
 *           widths (master, m, v, compute), u8 storage formats (MOEV_FMT_* of master, m, v,
 *           compute, after the defaults by width have been filled in), per tensor (u32 op,
 *           u64 numel), per operator u32 slot, per position u32 order.  A snapshot therefore
 *           loads only into a plan with the same operators, schedule, alignment and precision
 *           regime.
 */
#ifndef MOEV_H
#define MOEV_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  MOEV_OK = 0,
  MOEV_E_INVAL = -1,    /* bad argument (null, misaligned, not a schedule, ...) */
  MOEV_E_NOMEM = -2,    /* host or device allocation failed */
  MOEV_E_RANGE = -3,    /* slot >= window, buffer too small */
  MOEV_E_MISMATCH = -4, /* snapshot header does not belong to this plan / slot */
  MOEV_E_HIP = -5       /* a HIP runtime call failed; see moev_last_error() */
};

enum { MOEV_KIND_MASTER = 0, MOEV_KIND_ADAM_M = 1, MOEV_KIND_ADAM_V = 2, MOEV_KIND_COMPUTE = 3 };

/* storage formats of the training state (the low-precision regimes of Sec. 5.6 keep master weights,
 * optimizer state and compute weights in FP16 or 8-bit floating point):
 *   F32  IEEE binary32          F16  IEEE binary16          BF16  upper half of binary32
 *   E4M3 8 bits, 4 exponent (bias 7) + 3 mantissa, no infinities, NaN = S.1111.111, largest value 448
 *   E5M2 8 bits, 5 exponent (bias 15) + 2 mantissa, IEEE-like, largest finite value 57344
 * Conversions round to nearest even.  F16 and BF16 overflow to infinity; E4M3 and E5M2 saturate
 * (anything beyond the largest finite value, infinities included, becomes that value); NaN stays NaN
 * (which of the format's NaN patterns is written is not specified). */
enum { MOEV_FMT_DEFAULT = 0, MOEV_FMT_F32 = 1, MOEV_FMT_F16 = 2, MOEV_FMT_BF16 = 3, MOEV_FMT_E4M3 = 4, MOEV_FMT_E5M2 = 5 };

enum {
  MOEV_EXPLICIT = 0, /* slot_of_op given by the caller */
  MOEV_FIXED = 1,    /* GenerateSchedule of Algorithm 1 from `order` and `n_active` */
  MOEV_AUTO = 2      /* FindWindowSize of Algorithm 1 from t_iter_s and host_link_Bps, then FIXED */
};

#define MOEV_HEADER_BYTES 256u

typedef struct moev_plan moev_plan; /* opaque */

/* one parameter tensor of operator `op`.  Tensors are listed grouped by operator, operators
 * in ascending id starting at 0. */
typedef struct {
  uint32_t op;
  uint64_t numel;
} moev_tensor;

typedef struct {
  uint32_t n_ops, n_tensors;
  const moev_tensor *tensors;  /* host, [n_tensors] */
  int mode;                    /* MOEV_EXPLICIT / MOEV_FIXED / MOEV_AUTO */
  uint32_t window;             /* EXPLICIT: W_sparse.  Ignored otherwise (derived). */
  uint32_t n_active;           /* FIXED: operators checkpointed with full state per slot (O_Active) */
  const uint32_t *order;       /* host, [n_ops]: O_Ordered, the checkpoint order (ascending popularity).
                                  FIXED/AUTO: NULL = identity.  EXPLICIT: NULL = by (slot, id); if given,
                                  slots must not decrease along it. */
  const uint32_t *slot_of_op;  /* host, [n_ops]: EXPLICIT only */
  double t_iter_s;             /* AUTO: T_Iter */
  double host_link_Bps;        /* AUTO: B_PCIe, bytes per second */
  uint32_t align;              /* segment alignment in the packed buffer: power of two >= 16; 0 = 256 */
  uint8_t master_bytes;        /* element widths in bytes (1, 2, 4 or 8); 0 = defaults 4, 4, 4, 2.  Other */
  uint8_t m_bytes;             /* values describe the low-precision regimes of Sec. 5.6 (e.g. FP8 master, */
  uint8_t v_bytes;             /* FP8 + FP16 moments, FP8 compute = 1, 1, 2, 1): pack, drain and unpack */
  uint8_t compute_bytes;       /* are byte copies and work for any widths */
  uint8_t master_fmt;          /* MOEV_FMT_* of each kind, used by the replay only.  0 = by width: 4 -> F32, */
  uint8_t m_fmt;               /* 2 -> F16 (compute weights: BF16), 1 -> E4M3, 8 -> none (no replay).  A format */
  uint8_t v_fmt;               /* given with width 0 sets the width; a format that contradicts a given width */
  uint8_t compute_fmt;         /* is MOEV_E_INVAL. */
} moev_plan_cfg;

typedef struct {
  uint32_t kind;   /* MOEV_KIND_* */
  uint32_t tensor;
  uint64_t nbytes;
  uint64_t dst_off;
} moev_segment;

/* dense training state: four host arrays [n_tensors] of device pointers.  Each tensor is
 * contiguous and 16-byte aligned. */
typedef struct {
  void *const *master;
  void *const *m;
  void *const *v;
  void *const *compute;
} moev_state;

/* Adam hyper-parameters and the global iteration number of the step to replay (all operators
 * share it; it drives the bias corrections 1 - beta^step). */
typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
  uint64_t step;
  const float *d_scales; /* device, [4][n_tensors] kind-major (master, m, v, compute), or NULL = all 1:
                            per-tensor scale s of the kinds stored narrower than FP32, bits = encode(x * s),
                            x = decode(bits) * (1 / s) in FP32.  Kinds stored as FP32 ignore theirs.  Scales
                            must be positive and finite (they are not checked: the array lives on the
                            device).  The array must stay valid until the replay has run. */
} moev_adam;

typedef struct {
  uint64_t magic;
  uint32_t version, slot;
  uint64_t plan_hash, iter, n_segments, payload_bytes;
  uint32_t align;
} moev_header;

/* launch knobs for moev_tune().  Two launch shapes exist for pack, unpack and replay:
 *   one tile per workgroup (default): grid = number of tiles, tile = threads x 16 bytes (4 elements
 *     for the replay) x unroll; fastest when the kernel has the GPU to itself;
 *   fixed grid (MOEV_TUNE_PERSISTENT = 1): at most *_MAX_BLOCKS workgroups of 256 threads walk the
 *     tile list, tile table staged in LDS; lower the cap to leave compute units to a concurrent kernel.
 * Changing a knob while GPU work of the plan is in flight is not allowed. */
enum {
  MOEV_TUNE_COPY_TILE_BYTES = 0, /* fixed grid: bytes of packed buffer per tile (multiple of 4096) */
  MOEV_TUNE_COPY_MAX_BLOCKS = 1, /* fixed grid: cap on the pack/unpack grid (0 = 8 per compute unit) */
  MOEV_TUNE_ADAM_TILE_ELEMS = 2, /* fixed grid: elements per tile (multiple of 1024) */
  MOEV_TUNE_ADAM_MAX_BLOCKS = 3,
  MOEV_TUNE_NONTEMPORAL = 4,     /* 1 = streaming (nontemporal) loads and stores, 0 = default caching */
  MOEV_TUNE_PERSISTENT = 5,      /* 0 = one tile per workgroup, 1 = fixed grid */
  MOEV_TUNE_COPY_THREADS = 6,    /* one tile per workgroup: threads (64..1024) and accesses per lane (1, 2, 4); */
  MOEV_TUNE_COPY_UNROLL = 7,     /*   supported pairs: (64|128|256|512|1024, 1), (64|128|256|512, 2), (64|128|256, 4).
                                      Until either is set the pack uses 256 threads and picks the accesses per lane
                                      per slot: 2 where the slot gathers compute-weight segments averaging under
                                      64 MiB, else 1 (moev_tune_get returns 0 for MOEV_TUNE_COPY_UNROLL then) */
  MOEV_TUNE_ADAM_THREADS = 8,
  MOEV_TUNE_ADAM_UNROLL = 9,
  MOEV_TUNE_UNPACK_THREADS = 10, /* the unpack's own shape (MOEV_TUNE_COPY_* is the pack's) */
  MOEV_TUNE_UNPACK_UNROLL = 11,
  MOEV_TUNE_XCD_REGIONS = 12,    /* replay, one tile per workgroup (workgroup ids go to the 8 XCDs round robin): 1 (default)
                                    = each XCD sweeps a contiguous eighth of the launch's tiles; 0 = consecutive workgroups
                                    take consecutive tiles; G = 2 .. 65536 (a power of two) = chunks of G consecutive tiles are
                                    dealt to the XCDs round robin, so every XCD streams runs of G tiles while the chip-wide
                                    window of addresses in flight stays 8 G tiles wide */
  MOEV_TUNE_PLAIN_DIVIDE_SQRT = 13, /* replay on low-precision state: 1 (default) = where every first and second moment
                                    of a wavefront has a magnitude in [2^-60, 2^40) (and the bias corrections are in
                                    [2^-20, 1], epsilon in [0, 2^20]) the three divisions and the square root run as the
                                    compiler's IEEE sequences WITHOUT their rescaling and special-case steps, which do
                                    nothing for such operands: same results, ~20% fewer instructions; 0 = always the
                                    full sequences */
  MOEV_TUNE_PAIRED_TILES = 14,     /* replay in its 64 x 1 shape (the default of the FP32 regime and of the regimes with more than 6
                                    bytes of master weights and moments per parameter): every wavefront takes, per stream, two
                                    pieces of 128 elements instead of 256 consecutive elements; the value is their distance in
                                    bytes for an FP32 stream (narrower streams proportionally less).  32768 (default; 1 selects
                                    it too): the addresses of a pair differ in bit 15 only, and on MI355X the memory system
                                    serves such pairs faster.  0 = consecutive tiles; any power of two in [512, 4 MiB] is
                                    accepted so that the distance can be swept (512 is the consecutive layout again).  The
                                    pairing follows the address of each tensor's master weights; other streams profit when
                                    their pointers are congruent to it modulo twice the distance.  Same results either way. */
  MOEV_TUNE_COPY_XCD_REGIONS = 15  /* MOEV_TUNE_XCD_REGIONS for pack and unpack; default 64 (every XCD streams runs of 64 tiles =
                                    256 KB) */
};

const char *moev_last_error(void);

/* ---- plan (host only; needs no GPU) -------------------------------------------------
 * Algorithm 1 / Sec. 3.5.  Builds slot(e) for every operator, validates that every operator
 * is active in exactly one slot, and lays out the packed snapshot of every slot.  On success
 * *out holds a new plan.  Errors: MOEV_E_INVAL, MOEV_E_NOMEM. */
int ckpt_plan(const moev_plan_cfg *cfg, moev_plan **out);
void ckpt_plan_free(moev_plan *plan);

/* Algorithm 1 helpers, usable without a plan.  FindWindowSize with per-operator sizes in
 * bytes; OrderOperators (ascending popularity, stable, ties by ascending id); the re-order
 * trigger of Sec. 3.5 (returns 1 when the activation frequency changed by more than
 * rel_change for at least min_fraction of the operators; the paper uses 0.10 and 0.25). */
int moev_find_window_size(uint32_t n_ops, double t_iter_s, double compute_bytes_per_op,
                          double master_bytes_per_op, double optim_bytes_per_op, double host_link_Bps,
                          uint32_t *window, uint32_t *n_active);
int moev_order_operators(uint32_t n_ops, const double *popularity, uint32_t *order);
int moev_reorder_needed(uint32_t n_ops, const double *old_freq, const double *new_freq,
                        double rel_change, double min_fraction);

/* App. B alternatives to the hard activation count, to be fed to moev_order_operators:
 * time-decayed popularity out = alpha * previous + (1 - alpha) * batch_count (exponential moving
 * average over mini-batches), and capacity-aware popularity out = popularity / capacity.
 * (Soft-count popularity is the sum of gating probabilities: the caller's own reduction.)
 * `out` may alias `previous` / `popularity`.  MOEV_E_INVAL on null pointers, alpha outside [0, 1] or
 * a non-positive capacity. */
int moev_popularity_time_decayed(uint32_t n_ops, double alpha, const double *previous, const double *batch_count,
                                 double *out);
int moev_popularity_capacity_aware(uint32_t n_ops, const double *popularity, const double *capacity, double *out);

/* Efficiency model.  Sec. 2.4 / App. C: ETTR = 1/(1 + T_ckpt/(T_iter*interval)) * 1/(1 + E[R]/MTBF);
 * returns NaN on non-positive t_iter_s, interval or mtbf_s.  Sec. 3.6: expected and worst-case
 * recovery time; sparse = 0: dense checkpoint every `interval_or_window` iterations (E[R] = half the
 * interval, worst = the interval); sparse = 1: sparse window of that many iterations (E[R] = 3/2 W
 * T_iter, worst = 2 W T_iter). */
double moev_ettr(double t_ckpt_s, double t_iter_s, double ckpt_interval_iters, double expected_recovery_s,
                 double mtbf_s);
int moev_recovery_time(int sparse, double interval_or_window, double t_iter_s, double *expected_s, double *worst_s);

/* The two bias corrections 1 - beta^step of the replayed Adam step, exactly as convert_replay passes them to
 * its kernel: evaluated in double precision, rounded to FP32 once.  MOEV_E_INVAL on null pointers or step 0. */
int moev_bias_corrections(float beta1, float beta2, uint64_t step, float *bc1, float *bc2);

/* queries (host) */
uint32_t ckpt_plan_window(const moev_plan *plan);
uint32_t ckpt_plan_n_ops(const moev_plan *plan);
uint32_t ckpt_plan_n_tensors(const moev_plan *plan);
uint32_t ckpt_plan_n_active(const moev_plan *plan);            /* O_Active (0 for EXPLICIT) */
uint64_t ckpt_plan_hash(const moev_plan *plan);
/* element width in bytes / MOEV_FMT_* (0: none, the kind is only ever copied) of a MOEV_KIND_*; 0 on bad arguments */
uint32_t ckpt_plan_width(const moev_plan *plan, uint32_t kind);
uint32_t ckpt_plan_format(const moev_plan *plan, uint32_t kind);
int ckpt_plan_slot_of_op(const moev_plan *plan, uint32_t *out /* host [n_ops] */);
int ckpt_plan_order(const moev_plan *plan, uint32_t *out /* host [n_ops] */);
uint64_t ckpt_plan_packed_bytes(const moev_plan *plan, uint32_t slot); /* 0 if slot >= window */
uint64_t ckpt_plan_max_packed_bytes(const moev_plan *plan);
uint32_t ckpt_plan_n_segments(const moev_plan *plan, uint32_t slot);
/* copies up to cap entries of the slot's segment table (host-computed offsets); returns the
 * number of segments of the slot or a negative error */
int64_t ckpt_plan_segments(const moev_plan *plan, uint32_t slot, moev_segment *out, uint64_t cap);
/* bytes of packed buffer one workgroup of snapshot_pack(slot) handles (0 if slot >= window) */
uint64_t ckpt_plan_pack_tile_bytes(const moev_plan *plan, uint32_t slot);
/* parameters updated by replay iteration i of a conversion: operators with slot <= i */
uint64_t ckpt_plan_active_params(const moev_plan *plan, uint32_t i);

int moev_tune(moev_plan *plan, int knob, int64_t value);
int64_t moev_tune_get(const moev_plan *plan, int knob);

/* ---- device side of the plan ---------------------------------------------------------
 * Uploads the segment tables and computes, ON THE DEVICE with wavefront prefix sums, the
 * offset of every segment and the tile-to-segment map of every slot.  Called implicitly by
 * the first GPU call; call it yourself to keep that cost out of the first snapshot.
 * Enqueues on `stream`. */
int ckpt_plan_upload(moev_plan *plan, void *stream);
/* test hook: copy the device-computed layout of a slot back (synchronises `stream`).
 * dst_off_out: host [n_segments]; tile_start_out: host [n_segments + 1] or NULL. */
int ckpt_plan_device_layout(moev_plan *plan, uint32_t slot, uint64_t *dst_off_out,
                            uint32_t *tile_start_out, uint64_t *packed_bytes_out, void *stream);
/* device status word (synchronises `stream`): 0; MOEV_E_MISMATCH if a restore_unpack found a
 * foreign header in a device-resident snapshot and skipped it; MOEV_E_INVAL if a
 * convert_replay met an active operator with a null gradient pointer and skipped it.
 * Reading clears it. */
int ckpt_plan_device_status(moev_plan *plan, void *stream);

/* ---- snapshot (Sec. 3.2) ---------------------------------------------------------------
 * snapshot_pack: one gather kernel.  Copies master, m, v of every tensor of the operators
 * active in `slot` and the compute weights of every tensor of the operators active in later
 * slots from `state` into d_packed (device, 256-byte aligned, cap >= packed_bytes(slot)),
 * writes the header (with `iter` = the iteration whose post-update state this is) and zero
 * padding.  Errors: MOEV_E_INVAL (null / misaligned pointer), MOEV_E_RANGE, MOEV_E_HIP. */
int snapshot_pack(moev_plan *plan, uint32_t slot, uint64_t iter, const moev_state *state,
                  void *d_packed, size_t cap, void *stream);

/* snapshot_drain: packed_bytes(slot) bytes from d_packed (device) to h_pinned (pinned host,
 * cap >= packed_bytes(slot)) with one asynchronous copy on `side_stream`.  If pack_done is
 * non-NULL the copy waits for that event (record it on the pack stream after snapshot_pack);
 * if drained is non-NULL it is recorded after the copy.  The host buffer is complete once
 * `drained` (or the side stream) has been synchronised. */
int snapshot_drain(moev_plan *plan, uint32_t slot, const void *d_packed, void *h_pinned, size_t cap,
                   void *side_stream, void *pack_done, void *drained);

/* snapshot_drain_range: the same for bytes [offset, offset + nbytes) of the slot's packed snapshot, for
 * hosts that cannot pin a whole slot: the caller drains through a ring of pinned chunks, consuming
 * (persisting, sending) each chunk after its `drained` event and reusing it.  MOEV_E_RANGE if the range
 * leaves the slot's packed bytes. */
int snapshot_drain_range(moev_plan *plan, uint32_t slot, const void *d_packed, uint64_t offset, void *h_pinned,
                         size_t nbytes, void *side_stream, void *pack_done, void *drained);

/* parse and validate a snapshot header that lies in HOST memory against the plan and slot.
 * Returns MOEV_OK, MOEV_E_MISMATCH or MOEV_E_INVAL; *out (optional) receives the fields. */
int snapshot_peek(const moev_plan *plan, uint32_t slot, const void *h_packed, moev_header *out);

/* ---- conversion (Sec. 3.3) -------------------------------------------------------------
 * restore_unpack: load the snapshot of `slot`.  If h_pinned is non-NULL its header is checked
 * on the host (MOEV_E_MISMATCH on a foreign snapshot; nothing is enqueued then) and
 * packed_bytes(slot) bytes are first copied host-to-device into d_packed on `stream`;
 * otherwise d_packed must already hold the snapshot and the header is checked by the
 * kernel, which skips a foreign snapshot and raises the device status word.  Then one
 * scatter kernel writes every segment back into `state`, sets compute = bf16(master)
 * (round to nearest even) for the tensors of the newly active operators (FP32-master /
 * 2-byte-compute regime only), and updates d_active_mask (device, [n_ops] bytes): 1 for the
 * operators active in `slot`, 0 for the operators of later slots, earlier ones untouched. */
int restore_unpack(moev_plan *plan, uint32_t slot, const void *h_pinned, void *d_packed,
                   const moev_state *state, uint8_t *d_active_mask, void *stream);

/* convert_replay: one fused Adam step of iteration adam->step on every tensor whose operator
 * has d_active_mask != 0, with gradients grads (host array [n_tensors] of device pointers to
 * fp32 gradients; entries of frozen operators are not read and may be NULL):
 *     m = beta1*m + (1-beta1)*g;  v = beta2*v + (1-beta2)*(g*g);
 *     p = p - lr*weight_decay*p            (only if weight_decay != 0)
 *     p = p - lr * ((m/bc1) / (sqrt(v/bc2) + eps)),   bc = 1 - beta^step
 *     compute = bf16(p)
 * all in FP32, every operation rounded separately (no fused multiply-add), division and
 * square root correctly rounded.  Tensors of frozen operators are not touched.
 * State stored in other formats than FP32 / FP32 / FP32 / BF16 (Sec. 5.6) is widened to FP32
 * (decode, times the reciprocal of its scale), takes exactly the step above, and is narrowed
 * again (times the scale, encode); the compute weights are then cast from the master weights
 * AS STORED.  Format combinations with a kernel (master, m, v, compute): the five regimes of
 * Sec. 5.6  F16 F16 F16 F16 | F32 F32 F32 E4M3 | F16 F32 F32 E4M3 | F16 E4M3 F16 E4M3 |
 * E4M3 E4M3 F16 E4M3,  FP32 state with FP16 compute weights  F32 F32 F32 F16,  and
 * F16 F16 F16 BF16 | BF16 BF16 BF16 BF16 | F16 E5M2 F16 E5M2 | E5M2 E4M3 BF16 E5M2;
 * others are MOEV_E_INVAL.  These regimes run with 64, 128 or 256 threads and unroll 1 or 2
 * (MOEV_TUNE_ADAM_*), one tile per workgroup.
 * Placement and speed (results do not depend on it): the step reads and writes eight streams at the same element
 * index; on MI355X it runs fastest (6.2-6.5 TB/s against 5.8-6.0) when the master weights, both moments and the gradient
 * of a tensor start at the same offset modulo 64 KiB, which allocations of 2 MiB granularity and equal offsets inside
 * per-kind flat buffers give (see MOEV_TUNE_PAIRED_TILES).
 * Errors: MOEV_E_INVAL, MOEV_E_HIP. */
int convert_replay(moev_plan *plan, const moev_adam *adam, const uint8_t *d_active_mask,
                   void *const *grads, const moev_state *state, void *stream);

/* convert_replay_static: convert_replay for callers that cannot allocate device memory (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc).  Same step, same kernels, same results as
 * convert_replay, but the call allocates, frees and uploads nothing:
 *   - the plan's device tables must be resident already (ckpt_plan_upload, or any earlier GPU call with the
 *     same launch knobs); MOEV_E_INVAL otherwise;
 *   - the tables of pointers are passed ON THE DEVICE and owned by the caller: d_state_table = device array
 *     [4 * n_tensors] of device pointers, kind-major (all master, all m, all v, all compute), d_grad_table =
 *     device array [n_tensors] (entries of frozen operators are not read and may be null); both 8-byte aligned,
 *     every tensor they name 16-byte aligned (not checked: the tables live on the device);
 *   - the step's scratch (the compacted tile list the kernels hand from one to the other) lives in a static
 *     device array inside the library, sized for plans of at most MOEV_STATIC_MAX_TENSORS tensors (256 KiB per
 *     GPU, held from library load until the process ends); larger plans are refused with MOEV_E_RANGE.
 * All calls on one GPU share that array and each call rewrites the part it uses, so two calls that may run
 * at the same time on one GPU (different streams, different threads) race: order them.  One-tile-per-workgroup
 * launch shape only (MOEV_E_INVAL if MOEV_TUNE_PERSISTENT is set).  A null gradient of an active operator is
 * reported through ckpt_plan_device_status like in convert_replay.
 * Errors: MOEV_E_INVAL, MOEV_E_RANGE, MOEV_E_HIP. */
#define MOEV_STATIC_MAX_TENSORS 65536u
int convert_replay_static(moev_plan *plan, const moev_adam *adam, const uint8_t *d_active_mask,
                          void *const *d_grad_table, void *const *d_state_table, void *stream);

/* convert_window_step: one step of the conversion loop (Sec. 3.3: load SS_t, then replay iteration
 * t+1), i.e. restore_unpack(slot) followed by convert_replay(adam) with bit-identical results, but
 * fused: the FP32 state of the operators the snapshot activates is read straight from the packed
 * buffer by the replay kernel instead of being scattered to the dense tensors and read back
 * (26 fewer bytes of HBM traffic per newly active parameter).  Arguments as in the two calls;
 * d_active_mask is updated like restore_unpack does and then used like convert_replay does.
 * For state in other formats than FP32 / FP32 / FP32 / BF16 the two kernels run unfused.
 * Every tensor of an operator active in `slot` must have a gradient (MOEV_E_INVAL otherwise).
 * A foreign device-resident snapshot is refused as a whole (status word, nothing is modified). */
int convert_window_step(moev_plan *plan, uint32_t slot, const void *h_pinned, void *d_packed,
                        const moev_adam *adam, uint8_t *d_active_mask, void *const *grads,
                        const moev_state *state, void *stream);

/* ---- upstream logging ring (Sec. 3.4) ---------------------------------------------------
 * Stage-boundary tensors (kind 0: activations passed downstream in the forward pass, kind 1:
 * gradients passed upstream in the backward pass) are copied to pinned host memory at the
 * sender, tagged (iteration, micro-batch), kept until the sparse checkpoint that supersedes
 * them has persisted, and copied back to the GPU when a neighbouring stage recovers locally.
 * The ring lives in ONE caller-owned pinned buffer; entries are laid out in arrival order and
 * never wrap (a tail too short for the next entry is skipped); iterations must not go backwards.
 *
 * uplog_create   ring over h_pinned_ring[ring_bytes] (16-byte aligned), at most max_entries live entries.
 * uplog_reserve  host bookkeeping only: claims room for an entry and returns its offset
 *                (MOEV_E_NOMEM when the ring is full: run uplog_gc, or the training loop must stall;
 *                MOEV_E_INVAL for a duplicate tag or a kind other than 0 / 1).
 * uplog_append   uplog_reserve + one async device-to-host copy on side_stream, after `ready`
 *                (an event recorded when the tensor is complete; may be NULL).
 * uplog_find     host pointer and size of a logged tensor (valid after the side stream has been
 *                synchronised), MOEV_E_RANGE if it is not (or no longer) in the ring.
 * uplog_replay   async host-to-device copy of a logged tensor into d_dst[cap] on `stream`.
 * uplog_gc       "stale log cleanup": drops every entry with iteration < first_kept_iter; returns
 *                the number of entries dropped.
 */
typedef struct moev_uplog moev_uplog;
int uplog_create(void *h_pinned_ring, size_t ring_bytes, uint32_t max_entries, moev_uplog **out);
void uplog_free(moev_uplog *log);
int uplog_reserve(moev_uplog *log, uint64_t iter, uint32_t micro_batch, uint32_t kind, size_t nbytes,
                  uint64_t *offset_out);
int uplog_append(moev_uplog *log, uint64_t iter, uint32_t micro_batch, uint32_t kind, const void *d_tensor,
                 size_t nbytes, void *side_stream, void *ready);
int uplog_find(moev_uplog *log, uint64_t iter, uint32_t micro_batch, uint32_t kind, const void **h_ptr,
               size_t *nbytes);
int uplog_replay(moev_uplog *log, uint64_t iter, uint32_t micro_batch, uint32_t kind, void *d_dst, size_t cap,
                 void *stream);
int64_t uplog_gc(moev_uplog *log, uint64_t first_kept_iter);
int uplog_stats(moev_uplog *log, uint64_t *entries, uint64_t *bytes_in_use, uint64_t *capacity);

/* ---- measurement hook --------------------------------------------------------------------
 * moev_copy_probe: plain contiguous device-to-device copy of nbytes (multiple of 16, both
 * pointers 16-byte aligned) with the same access shape as the gather kernel.  It is the
 * yardstick the pack/unpack throughput is compared with and the known-size kernel against
 * which HBM traffic counters are calibrated.  blocks = 0: one 4 KB tile per workgroup (the default
 * gather shape, with the gather's default workgroup -> tile mapping: chunks of 64 tiles dealt to the XCDs round
 * robin); blocks > 0: a fixed grid of that many workgroups, 32 KB per step. */
int moev_copy_probe(void *d_dst, const void *d_src, size_t nbytes, uint32_t blocks, int nontemporal,
                    void *stream);

/* moev_stream_probe: the one-directional companions of the copy probe, same access shape and mapping (one 4 KB tile
 * per workgroup, chunks of 64 tiles per XCD).  mode 1: read nbytes from d_src and discard them (d_dst: 16 writable device bytes, which receive a
 * store only if the data happens to contain one particular 128-bit pattern); mode 2: fill d_dst[nbytes] with the
 * 32-bit `value`, d_src is not used.  nbytes a multiple of 16, pointers 16-byte aligned.  Read-only, write-only and
 * copy rates bracket what a kernel with a given read : write mix can reach on the box.
 * mode 3: copy d_src to d_dst with every wavefront instruction covering two 512-byte pieces `value` bytes apart
 * (a power of two in [512, 2^30]; 512 = 1 KB of consecutive bytes, 32768 = the geometry of the replay's paired tiles,
 * MOEV_TUNE_PAIRED_TILES); nbytes and both pointers must be multiples of 2 x value (MOEV_E_INVAL otherwise).  Sweeping
 * the distance shows which address bit the memory system rewards. */
int moev_stream_probe(int mode, void *d_dst, const void *d_src, size_t nbytes, uint32_t value, int nontemporal,
                      void *stream);

/* ---- arithmetic self-check -----------------------------------------------------------------
 * moev_arith_selfcheck: runs, on the GPU, the plain division / square-root sequences of
 * MOEV_TUNE_PLAIN_DIVIDE_SQRT beside the compiler's full IEEE expansions and counts the inputs on
 * which the two differ (the count must be 0).
 *   what 0: n / divisor for the `count` consecutive FP32 bit patterns n starting at first_bits,
 *           with both signs;
 *   what 1: sqrt(x) for those patterns;
 *   what 2: n / d for `count` pseudo-random pairs (seed), |n| in [2^-60, 2^60), d in [2^-30, 2^31).
 * Allocates a counter, synchronises the stream, frees the counter.  Errors: MOEV_E_INVAL,
 * MOEV_E_RANGE (patterns beyond the finite positive values), MOEV_E_HIP. */
int moev_arith_selfcheck(int what, float divisor, uint32_t first_bits, uint64_t count, uint64_t seed,
                         uint64_t *mismatches, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOEV_H */
