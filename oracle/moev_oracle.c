/*
 * moev_oracle.c -- plain CPU oracle (TEST INFRASTRUCTURE ONLY, see moev_oracle.h).
 *
 * Written from the paper's statement of the method; no blocking, fusion, threading or
 * reordering beyond what the text states.  Build: gcc -std=c99 -O2 -ffp-contract=off.
 */
#include "moev_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ===================================================================================
 * Schedule -- Algorithm 1 ("Sparse Checkpoint Scheduling"), Sec. 3.5
 * =================================================================================== */

/*
 * Window size (Sec. 3.5, FindWindowSize of Algorithm 1).  A snapshot that checkpoints `a` of the
 * O_Total operators with full state carries (S_Master + S_Optim) * a + S_Compute * (O_Total - a)
 * bytes and must cross the host link within one iteration.  The method wants the SMALLEST window,
 * i.e. the LARGEST such `a`; it considers a = O_Total, O_Total - 1, ..., 3 and, when none of them
 * fits, settles for two operators per slot without asking whether two fit (all of them when
 * there are fewer than three).  W_sparse = ceil(O_Total / O_Active).
 */
static int snapshot_fits(uint32_t o_total, uint32_t a, double t_iter, double s_compute, double s_master,
                         double s_optim, double b_pcie) {
  double bytes = (s_master + s_optim) * (double)a + s_compute * (double)(o_total - a);
  return bytes / b_pcie <= t_iter;
}

int orc_find_window_size(uint32_t o_total, double t_iter, double s_compute, double s_master,
                         double s_optim, double b_pcie, uint32_t *w_sparse, uint32_t *o_active) {
  if (o_total == 0 || !w_sparse || !o_active || !(b_pcie > 0.0)) return ORC_BAD_ARG;
  uint32_t best = o_total < 2 ? o_total : 2;            /* the floor, taken unchecked */
  for (uint32_t a = 3; a <= o_total; ++a)               /* every candidate; the largest fitting one wins */
    if (snapshot_fits(o_total, a, t_iter, s_compute, s_master, s_optim, b_pcie)) best = a;
  *o_active = best;
  *w_sparse = o_total / best + (o_total % best != 0);
  return ORC_OK;
}

/*
 * Schedule (Sec. 3.5, GenerateSchedule of Algorithm 1).  O_Ordered is cut into consecutive runs
 * of O_Active operators, one run per slot, the last run possibly shorter: the operator at
 * position j of O_Ordered is checkpointed with full state in slot floor(j / O_Active).  A slot's
 * frozen set is everything behind its run in O_Ordered, i.e. the operators of later slots.
 * Stored as the slot of every operator: active set of slot i = {e : slot_of_op[e] == i},
 * frozen set = {e : slot_of_op[e] > i}.
 */
int orc_generate_schedule(uint32_t n_ops, const uint32_t *order, uint32_t o_active,
                          uint32_t *slot_of_op, uint32_t *w_sparse) {
  if (n_ops == 0 || o_active == 0 || !order || !slot_of_op || !w_sparse) return ORC_BAD_ARG;
  for (uint32_t j = 0; j < n_ops; ++j) {
    if (order[j] >= n_ops) return ORC_BAD_ARG;
    slot_of_op[order[j]] = j / o_active;
  }
  *w_sparse = (n_ops - 1) / o_active + 1;
  return ORC_OK;
}

/*
 * OrderOperators (Sec. 3.5): ascending popularity, so that popular operators are
 * checkpointed late in the window and stay frozen longest during conversion.  The paper
 * gives no tie-break; reading taken: stable, equal popularity keeps ascending operator id.
 * Plain insertion sort.
 */
int orc_order_by_popularity(uint32_t n_ops, const double *popularity, uint32_t *order) {
  if (!popularity || !order) return ORC_BAD_ARG;
  for (uint32_t e = 0; e < n_ops; ++e) {
    uint32_t j = e;
    while (j > 0 && popularity[order[j - 1]] > popularity[e]) {
      order[j] = order[j - 1];
      --j;
    }
    order[j] = e;
  }
  return ORC_OK;
}

/*
 * A valid window (Sec. 3.2: after W_sparse iterations every operator has exactly one
 * FP32 snapshot): `order` is a permutation, every operator has one slot below the window
 * size, and walking O_Ordered never goes back to an earlier slot (the active sets are
 * consecutive runs of O_Ordered, Algorithm 1).
 */
int orc_check_schedule(uint32_t n_ops, const uint32_t *order, const uint32_t *slot_of_op,
                       uint32_t window) {
  if (n_ops == 0 || window == 0 || !order || !slot_of_op) return ORC_BAD_ARG;
  for (uint32_t e = 0; e < n_ops; ++e) {
    uint32_t seen = 0;
    for (uint32_t j = 0; j < n_ops; ++j)
      if (order[j] == e) ++seen;
    if (seen != 1) return ORC_NOT_A_SCHEDULE;
    if (slot_of_op[e] >= window) return ORC_NOT_A_SCHEDULE;
  }
  for (uint32_t j = 1; j < n_ops; ++j)
    if (slot_of_op[order[j]] < slot_of_op[order[j - 1]]) return ORC_NOT_A_SCHEDULE;
  return ORC_OK;
}

/*
 * App. B, time-decayed popularity: an exponential moving average over mini-batches,
 *   A(t) = alpha * A(t-1) + (1 - alpha) * (number of tokens of batch t routed to the expert).
 */
void orc_popularity_time_decayed(uint32_t n_ops, double alpha, const double *previous, const double *batch_count,
                                 double *out) {
  for (uint32_t e = 0; e < n_ops; ++e) out[e] = alpha * previous[e] + (1.0 - alpha) * batch_count[e];
}

/* App. B, capacity-aware ordering: popularity divided by the expert's capacity factor. */
void orc_popularity_capacity_aware(uint32_t n_ops, const double *popularity, const double *capacity, double *out) {
  for (uint32_t e = 0; e < n_ops; ++e) out[e] = popularity[e] / capacity[e];
}

/*
 * Sec. 2.4 (and App. C): ETTR ~ 1 / (1 + T_ckpt / (T_iter * Ckpt_interval)) * 1 / (1 + E[R] / MTBF),
 * runtime overhead of checkpointing times recovery overhead under Poisson failures.
 */
double orc_ettr(double t_ckpt, double t_iter, double ckpt_interval, double expected_recovery, double mtbf) {
  double runtime_overhead = t_ckpt / (t_iter * ckpt_interval);
  double recovery_overhead = expected_recovery / mtbf;
  return 1.0 / (1.0 + runtime_overhead) * (1.0 / (1.0 + recovery_overhead));
}

/* Sec. 3.6, dense checkpointing: 0 <= R <= interval * T_iter, E[R] ~ interval * T_iter / 2. */
void orc_recovery_dense(double ckpt_interval, double t_iter, double *expected, double *worst) {
  *worst = ckpt_interval * t_iter;
  *expected = 0.5 * ckpt_interval * t_iter;
}

/* Sec. 3.6, sparse checkpointing: replay W_sparse iterations to rebuild the dense checkpoint, then
 * re-execute up to W_sparse more: 0 <= R <= 2 * W * T_iter, E[R] ~ 3/2 * W * T_iter. */
void orc_recovery_sparse(double w_sparse, double t_iter, double *expected, double *worst) {
  *worst = 2.0 * w_sparse * t_iter;
  *expected = 1.5 * w_sparse * t_iter;
}

/* ===================================================================================
 * Snapshot layout, pack, unpack -- Sec. 3.2 (what a sparse snapshot holds), Sec. 3.3
 * (what loading one does).  The byte layout of a packed snapshot is this build's own
 * definition (the paper copies operator by operator and defines none):
 *
 *   [256-byte header][segment 0][zero pad][segment 1][zero pad] ...
 *
 *   segment order: walk O_Ordered; for each operator active in the slot, for each of its
 *   tensors in declared order: master, Adam m, Adam v; then walk O_Ordered again; for each
 *   operator active in a LATER slot, for each of its tensors: compute weights.
 *   dst_off[0] = roundup(256, align), dst_off[j+1] = dst_off[j] + roundup(nbytes[j], align);
 *   the snapshot ends at dst_off[last] + roundup(nbytes[last], align).
 *
 *   header (little endian): +0 u64 magic "MOEVSNAP", +8 u32 version (1), +12 u32 slot,
 *   +16 u64 plan hash, +24 u64 iteration, +32 u64 segment count, +40 u64 payload bytes
 *   (everything after the 256 header bytes), +48 u32 align, rest zero.
 * =================================================================================== */

static uint32_t width_of(const orc_model *mdl, uint32_t kind) {
  if (kind == ORC_MASTER) return mdl->width.master;
  if (kind == ORC_COMPUTE) return mdl->width.compute;
  if (kind == ORC_ADAM_M) return mdl->width.m;
  return mdl->width.v;
}

static uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) / a * a; }

static void put_le(uint8_t *dst, uint64_t value, int nbytes) {
  for (int i = 0; i < nbytes; ++i) dst[i] = (uint8_t)(value >> (8 * i));
}

static uint64_t get_le(const uint8_t *src, int nbytes) {
  uint64_t value = 0;
  for (int i = 0; i < nbytes; ++i) value |= (uint64_t)src[i] << (8 * i);
  return value;
}

static uint64_t fnv1a(uint64_t h, uint64_t value, int nbytes) {
  for (int i = 0; i < nbytes; ++i) {
    h ^= (value >> (8 * i)) & 0xffu;
    h *= 0x100000001b3ull;
  }
  return h;
}

/*
 * Storage format of a kind when the model names none: by element width, 4 bytes = FP32,
 * 2 bytes = FP16 (bfloat16 for the compute weights), 1 byte = E4M3, anything else = 0 (the kind
 * is only ever copied).
 */
static uint32_t storage_format_of_kind(const orc_model *mdl, int kind) {
  const uint32_t width[4] = {mdl->width.master, mdl->width.m, mdl->width.v, mdl->width.compute};
  if (mdl->fmt[kind]) return mdl->fmt[kind];
  if (width[kind] == 4) return ORC_FMT_F32;
  if (width[kind] == 2) return kind == ORC_COMPUTE ? ORC_FMT_BF16 : ORC_FMT_F16;
  if (width[kind] == 1) return ORC_FMT_E4M3;
  return 0;
}

/*
 * Identity of a plan, stored in every snapshot header so that a snapshot is never loaded
 * into a model, schedule or precision regime it was not taken from.  64-bit FNV-1a over the
 * little-endian stream: u32 n_ops, u32 n_tensors, u32 window, u32 align, u8 widths (master, m,
 * v, compute), u8 storage formats (master, m, v, compute), then per tensor (u32 op, u64 numel),
 * per operator u32 slot, per position u32 order.
 */
uint64_t orc_fnv1a64(const void *bytes, uint64_t n) {
  uint64_t h = 0xcbf29ce484222325ull;
  for (uint64_t i = 0; i < n; ++i) h = fnv1a(h, ((const uint8_t *)bytes)[i], 1);
  return h;
}

uint64_t orc_plan_hash(const orc_model *mdl) {
  uint64_t h = 0xcbf29ce484222325ull;
  h = fnv1a(h, mdl->n_ops, 4);
  h = fnv1a(h, mdl->n_tensors, 4);
  h = fnv1a(h, mdl->window, 4);
  h = fnv1a(h, mdl->align, 4);
  h = fnv1a(h, mdl->width.master, 1);
  h = fnv1a(h, mdl->width.m, 1);
  h = fnv1a(h, mdl->width.v, 1);
  h = fnv1a(h, mdl->width.compute, 1);
  for (int kind = 0; kind < 4; ++kind) h = fnv1a(h, storage_format_of_kind(mdl, kind), 1);
  for (uint32_t t = 0; t < mdl->n_tensors; ++t) {
    h = fnv1a(h, mdl->tensors[t].op, 4);
    h = fnv1a(h, mdl->tensors[t].numel, 8);
  }
  for (uint32_t e = 0; e < mdl->n_ops; ++e) h = fnv1a(h, mdl->slot_of_op[e], 4);
  for (uint32_t j = 0; j < mdl->n_ops; ++j) h = fnv1a(h, mdl->order[j], 4);
  return h;
}

/*
 * Segment list of one slot.  Sec. 3.2: the operators active in the slot contribute their
 * full training state (master weights and optimizer state, 12 bytes per parameter in the
 * default regime), the operators still waiting for their slot contribute only their
 * compute weights (2 bytes per parameter); operators whose slot has passed contribute
 * nothing (the worked example: the second snapshot holds FP32 state of E3,E4 and 2-byte
 * weights of NE,G only).  Returns the number of segments (also when segs == NULL or
 * seg_cap is too small, in which case nothing past seg_cap is stored).
 */
int64_t orc_layout(const orc_model *mdl, uint32_t slot, orc_segment *segs, uint64_t seg_cap,
                   uint64_t *packed_bytes) {
  if (!mdl || slot >= mdl->window || mdl->align == 0) return ORC_BAD_ARG;
  uint64_t n = 0, off = round_up(ORC_HEADER_BYTES, mdl->align);
  static const uint32_t full_state[3] = {ORC_MASTER, ORC_ADAM_M, ORC_ADAM_V};
  for (int pass = 0; pass < 2; ++pass) {
    for (uint32_t j = 0; j < mdl->n_ops; ++j) {
      uint32_t e = mdl->order[j];
      int is_active = mdl->slot_of_op[e] == slot;
      int is_frozen = mdl->slot_of_op[e] > slot;
      if (pass == 0 ? !is_active : !is_frozen) continue;
      for (uint32_t t = 0; t < mdl->n_tensors; ++t) {
        if (mdl->tensors[t].op != e) continue;
        int n_kinds = pass == 0 ? 3 : 1;
        for (int q = 0; q < n_kinds; ++q) {
          uint32_t kind = pass == 0 ? full_state[q] : ORC_COMPUTE;
          uint64_t nbytes = mdl->tensors[t].numel * width_of(mdl, kind);
          if (segs && n < seg_cap) {
            segs[n].kind = kind;
            segs[n].tensor = t;
            segs[n].nbytes = nbytes;
            segs[n].dst_off = off;
          }
          off += round_up(nbytes, mdl->align);
          ++n;
        }
      }
    }
  }
  if (packed_bytes) *packed_bytes = off;
  return (int64_t)n;
}

static void *state_ptr(const orc_state *st, uint32_t kind, uint32_t tensor) {
  if (kind == ORC_MASTER) return st->master[tensor];
  if (kind == ORC_ADAM_M) return st->m[tensor];
  if (kind == ORC_ADAM_V) return st->v[tensor];
  return st->compute[tensor];
}

/*
 * Sparse snapshot of slot `slot` taken from state `st` (Sec. 3.2): a byte-for-byte copy of
 * every listed segment to its offset, zero padding up to the alignment, header in front.
 */
int orc_pack(const orc_model *mdl, uint32_t slot, uint64_t iter, const orc_state *st,
             uint8_t *packed, uint64_t cap) {
  uint64_t total = 0;
  int64_t n = orc_layout(mdl, slot, NULL, 0, &total);
  if (n < 0) return (int)n;
  if (!st || !packed) return ORC_BAD_ARG;
  if (cap < total) return ORC_TOO_SMALL;
  orc_segment *segs = (orc_segment *)malloc((size_t)(n > 0 ? n : 1) * sizeof(orc_segment));
  if (!segs) return ORC_BAD_ARG;
  orc_layout(mdl, slot, segs, (uint64_t)n, NULL);

  memset(packed, 0, ORC_HEADER_BYTES);
  memcpy(packed, "MOEVSNAP", 8);
  put_le(packed + 8, 1, 4);
  put_le(packed + 12, slot, 4);
  put_le(packed + 16, orc_plan_hash(mdl), 8);
  put_le(packed + 24, iter, 8);
  put_le(packed + 32, (uint64_t)n, 8);
  put_le(packed + 40, total - ORC_HEADER_BYTES, 8);
  put_le(packed + 48, mdl->align, 4);
  /* with an alignment above 256 the first segment starts later than the header ends */
  memset(packed + ORC_HEADER_BYTES, 0, round_up(ORC_HEADER_BYTES, mdl->align) - ORC_HEADER_BYTES);

  for (int64_t j = 0; j < n; ++j) {
    uint64_t padded = round_up(segs[j].nbytes, mdl->align);
    memcpy(packed + segs[j].dst_off, state_ptr(st, segs[j].kind, segs[j].tensor), segs[j].nbytes);
    memset(packed + segs[j].dst_off + segs[j].nbytes, 0, padded - segs[j].nbytes);
  }
  free(segs);
  return ORC_OK;
}

/*
 * Round-to-nearest-even conversion of an FP32 master weight to a 2-byte bfloat16 compute
 * weight (the top 16 bits of the FP32 pattern).  NaN stays a (quiet) NaN; values above the
 * largest finite bfloat16 round to infinity as IEEE rounding prescribes (no saturation).
 * The paper names FP16 compute weights; this build's workloads use bfloat16.
 */
uint16_t orc_bf16_rne(float x) {
  uint32_t bits;
  memcpy(&bits, &x, 4);
  if ((bits & 0x7fffffffu) > 0x7f800000u) return (uint16_t)((bits >> 16) | 0x0040u);
  uint32_t lower = bits & 0xffffu;        /* the 16 bits that are dropped */
  uint32_t upper = bits >> 16;            /* the 16 bits that are kept   */
  if (lower > 0x8000u) upper += 1;        /* above the half-way point: round up */
  else if (lower == 0x8000u && (upper & 1u)) upper += 1; /* tie: to even */
  return (uint16_t)upper;
}

/*
 * Loading snapshot `slot` during sparse-to-dense conversion (Sec. 3.3; steps 1, 3, 5 of the
 * walk-through): every segment goes back into the dense tensor it came from.  Operators
 * whose FP32 state the snapshot carries become ACTIVE (mask 1); operators present only
 * with compute weights are FROZEN (mask 0); operators activated by an earlier snapshot are
 * not in the snapshot and are left alone.  A newly active operator's compute weights are
 * not stored (Sec. 3.2); reading taken: they are re-derived as bf16(master) so that the
 * dense state is complete (done only in the FP32-master / 2-byte-compute regime).
 * The header is checked first; a snapshot of another plan, slot or size is refused.
 */
int orc_unpack(const orc_model *mdl, uint32_t slot, const uint8_t *packed, uint64_t packed_len,
               const orc_state *st, uint8_t *active_mask, uint64_t *iter_out) {
  uint64_t total = 0;
  int64_t n = orc_layout(mdl, slot, NULL, 0, &total);
  if (n < 0) return (int)n;
  if (!st || !packed) return ORC_BAD_ARG;
  if (packed_len < total) return ORC_TOO_SMALL;
  if (memcmp(packed, "MOEVSNAP", 8) != 0 || get_le(packed + 8, 4) != 1 ||
      get_le(packed + 12, 4) != slot || get_le(packed + 16, 8) != orc_plan_hash(mdl) ||
      get_le(packed + 32, 8) != (uint64_t)n || get_le(packed + 40, 8) != total - ORC_HEADER_BYTES ||
      get_le(packed + 48, 4) != mdl->align)
    return ORC_BAD_SNAPSHOT;
  if (iter_out) *iter_out = get_le(packed + 24, 8);

  orc_segment *segs = (orc_segment *)malloc((size_t)(n > 0 ? n : 1) * sizeof(orc_segment));
  if (!segs) return ORC_BAD_ARG;
  orc_layout(mdl, slot, segs, (uint64_t)n, NULL);
  for (int64_t j = 0; j < n; ++j)
    memcpy(state_ptr(st, segs[j].kind, segs[j].tensor), packed + segs[j].dst_off, segs[j].nbytes);
  free(segs);

  for (uint32_t e = 0; e < mdl->n_ops; ++e) {
    if (mdl->slot_of_op[e] == slot) {
      if (active_mask) active_mask[e] = 1;
      if (mdl->width.master == 4 && mdl->width.compute == 2)
        for (uint32_t t = 0; t < mdl->n_tensors; ++t) {
          if (mdl->tensors[t].op != e) continue;
          const float *p = (const float *)st->master[t];
          uint16_t *c = (uint16_t *)st->compute[t];
          for (uint64_t i = 0; i < mdl->tensors[t].numel; ++i) c[i] = orc_bf16_rne(p[i]);
        }
    } else if (mdl->slot_of_op[e] > slot) {
      if (active_mask) active_mask[e] = 0;
    }
  }
  return ORC_OK;
}

/* ===================================================================================
 * Optimizer replay -- Sec. 3.3: active operators get their FP32 master weights and
 * optimizer state updated each optimizer step; frozen operators skip the update.
 * The paper names Adam (Sec. 3.2) / AdamW (App. D) and prints no formula.  Reading taken:
 * textbook Adam with bias correction, epsilon added after the square root, decoupled
 * weight decay applied first when non-zero.  All arithmetic in FP32 (the precision the
 * paper fixes for master weights and optimizer state), each product and sum rounded
 * separately, in exactly the order written below.
 * =================================================================================== */

/*
 * 1 - beta^t for both moments: beta^t by repeated multiplication in double, the
 * difference rounded to FP32 once.  All operators share the global iteration number t.
 */
void orc_bias_corrections(const orc_adam_hp *hp, uint64_t step, float *bc1, float *bc2) {
  double p1 = 1.0, p2 = 1.0;
  for (uint64_t i = 0; i < step; ++i) {
    p1 *= (double)hp->beta1;
    p2 *= (double)hp->beta2;
  }
  *bc1 = (float)(1.0 - p1);
  *bc2 = (float)(1.0 - p2);
}

void orc_adam_tensor(float *p, float *m, float *v, const float *g, uint16_t *c, uint64_t n,
                     const orc_adam_hp *hp, uint64_t step) {
  float bc1, bc2;
  orc_bias_corrections(hp, step, &bc1, &bc2);
  const float lr = hp->lr, beta1 = hp->beta1, beta2 = hp->beta2, eps = hp->eps;
  const float one_minus_beta1 = 1.0f - beta1;
  const float one_minus_beta2 = 1.0f - beta2;
  const float decay = lr * hp->weight_decay;
  for (uint64_t i = 0; i < n; ++i) {
    float grad = g[i];
    float param = p[i];
    if (hp->weight_decay != 0.0f) param = param - decay * param;
    float m_new = beta1 * m[i] + one_minus_beta1 * grad;
    float grad_sq = grad * grad;
    float v_new = beta2 * v[i] + one_minus_beta2 * grad_sq;
    float m_hat = m_new / bc1;
    float v_hat = v_new / bc2;
    float denom = sqrtf(v_hat) + eps;
    float update = lr * (m_hat / denom);
    param = param - update;
    p[i] = param;
    m[i] = m_new;
    v[i] = v_new;
    if (c) c[i] = orc_bf16_rne(param);
  }
}

/*
 * One replayed iteration of the conversion (steps 2, 4, 6 of the walk-through in
 * Sec. 3.3): every ACTIVE operator takes the optimizer step of global iteration `step`
 * with that iteration's gradients and refreshes its compute weights; FROZEN operators are
 * not touched at all (no moment decay, no step).
 */
int orc_replay_step(const orc_model *mdl, const orc_adam_hp *hp, uint64_t step,
                    const uint8_t *active_mask, const float *const *grads, const orc_state *st) {
  if (!mdl || !hp || !active_mask || !grads || !st || step == 0) return ORC_BAD_ARG;
  if (mdl->width.master != 4 || mdl->width.m != 4 || mdl->width.v != 4 || mdl->width.compute != 2) return ORC_BAD_ARG;
  for (uint32_t t = 0; t < mdl->n_tensors; ++t) {
    if (!active_mask[mdl->tensors[t].op]) continue;
    orc_adam_tensor((float *)st->master[t], (float *)st->m[t], (float *)st->v[t], grads[t],
                    (uint16_t *)st->compute[t], mdl->tensors[t].numel, hp, step);
  }
  return ORC_OK;
}

/* ===================================================================================
 * Low-precision training state -- Sec. 5.6 evaluates five regimes that store master
 * weights, optimizer state and compute weights in FP16 or 8-bit floating point instead of
 * FP32 / 2 bytes.  The paper only names the precisions; readings taken here:
 *   - FP16 is IEEE binary16 (overflow rounds to infinity); the 8-bit formats are the two
 *     of the Open Compute Project's 8-bit floating point specification: "E4M3" (bias 7, no
 *     infinities, one NaN pattern per sign, largest value 448) and "E5M2" (bias 15,
 *     IEEE-like, largest finite value 57344).  Conversions to them round to nearest even and
 *     SATURATE: what would exceed the largest finite value, infinities included, becomes
 *     that value; NaN stays NaN.
 *   - a stored value may carry a per-tensor scale s (the 8-bit training recipes the paper
 *     cites keep one per tensor together with its reciprocal): bits = encode(x * s),
 *     x = decode(bits) * (1 / s), every operation in FP32 (the reciprocal is rounded once).
 *     Kinds stored as FP32 ignore their scale.
 *   - the optimizer step widens the stored state to FP32, performs exactly the FP32 step of
 *     orc_adam_tensor, and narrows the results; compute weights are cast from the master
 *     weights AS STORED (after narrowing), not from the unrounded FP32 value.
 * =================================================================================== */

typedef struct {
  int exp_bits, man_bits, bias;
  int ieee_like;   /* 1: all-ones exponent = infinities and NaNs; 0: only all-ones exponent AND mantissa = NaN */
  int saturate;    /* 1: conversions clamp to the largest finite value */
} orc_format;

static int format_of(uint32_t fmt, orc_format *f) {
  switch (fmt) {
    case ORC_FMT_F16:  *f = (orc_format){5, 10, 15, 1, 0}; return 1;
    case ORC_FMT_BF16: *f = (orc_format){8, 7, 127, 1, 0}; return 1;
    case ORC_FMT_E4M3: *f = (orc_format){4, 3, 7, 0, 1}; return 1;
    case ORC_FMT_E5M2: *f = (orc_format){5, 2, 15, 1, 1}; return 1;
    default: return 0;
  }
}

uint32_t orc_fmt_bytes(uint32_t fmt) {
  switch (fmt) {
    case ORC_FMT_F32: return 4;
    case ORC_FMT_F16: case ORC_FMT_BF16: return 2;
    case ORC_FMT_E4M3: case ORC_FMT_E5M2: return 1;
    default: return 0;
  }
}

static double largest_finite(const orc_format *f) {
  int top_exp = (1 << f->exp_bits) - 1;          /* all-ones exponent field */
  if (f->ieee_like) {                             /* largest finite: exponent field top-1, mantissa all ones */
    return ldexp((double)((2 << f->man_bits) - 1), top_exp - 1 - f->bias - f->man_bits);
  }
  /* all-ones exponent is an ordinary binade; only its all-ones mantissa is NaN */
  return ldexp((double)((2 << f->man_bits) - 2), top_exp - f->bias - f->man_bits);
}

/* value of a bit pattern, by the definition of a binary floating-point format:
 * exponent field 0: mantissa * 2^(1 - bias - man_bits); otherwise (2^man_bits + mantissa) *
 * 2^(field - bias - man_bits) */
double orc_decode(uint32_t fmt, uint32_t bits) {
  if (fmt == ORC_FMT_F32) {
    float x;
    memcpy(&x, &bits, 4);
    return (double)x;
  }
  orc_format f;
  if (!format_of(fmt, &f)) return NAN;
  uint32_t man = bits & ((1u << f.man_bits) - 1u);
  uint32_t field = (bits >> f.man_bits) & ((1u << f.exp_bits) - 1u);
  int negative = (int)((bits >> (f.man_bits + f.exp_bits)) & 1u);
  uint32_t top = (1u << f.exp_bits) - 1u;
  double value;
  if (field == top && f.ieee_like) value = man ? NAN : INFINITY;
  else if (field == top && man == (1u << f.man_bits) - 1u) value = NAN;
  else if (field == 0) value = ldexp((double)man, 1 - f.bias - f.man_bits);
  else value = ldexp((double)((1u << f.man_bits) + man), (int)field - f.bias - f.man_bits);
  return negative ? -value : value;
}

/* nearest representable value, ties to the even mantissa; NaN becomes the quiet NaN with all
 * exponent bits and the top mantissa bit set (E4M3: its only NaN) -- except bfloat16, which keeps
 * orc_bf16_rne's convention (top 16 bits of the FP32 pattern with the quiet bit set) */
uint32_t orc_encode(uint32_t fmt, float x) {
  if (fmt == ORC_FMT_F32) {
    uint32_t bits;
    memcpy(&bits, &x, 4);
    return bits;
  }
  if (fmt == ORC_FMT_BF16) return orc_bf16_rne(x);
  orc_format f;
  if (!format_of(fmt, &f)) return 0;
  uint32_t sign = signbit(x) ? 1u << (f.man_bits + f.exp_bits) : 0u;
  uint32_t top = (1u << f.exp_bits) - 1u;
  if (isnan(x)) {
    if (f.ieee_like) return sign | (top << f.man_bits) | (1u << (f.man_bits - 1));
    return sign | (top << f.man_bits) | ((1u << f.man_bits) - 1u);
  }
  double a = fabs((double)x);
  double max_finite = largest_finite(&f);
  double q;  /* the rounded magnitude */
  if (isinf(x)) q = INFINITY;
  else if (a == 0.0) q = 0.0;
  else {
    int k;
    frexp(a, &k);                                   /* a = fraction * 2^k, fraction in [0.5, 1) */
    int binade = k - 1;                             /* 2^binade <= a < 2^(binade+1) */
    if (binade < 1 - f.bias) binade = 1 - f.bias;   /* subnormals share the spacing of the lowest binade */
    double spacing = ldexp(1.0, binade - f.man_bits);
    q = rint(a / spacing) * spacing;                /* default rounding mode: to nearest, ties to even */
  }
  if (q > max_finite) {
    if (f.saturate) q = max_finite;
    else return sign | (top << f.man_bits);         /* IEEE overflow: infinity */
  }
  if (q == 0.0) return sign;
  int k;
  frexp(q, &k);
  int binade = k - 1;
  if (binade < 1 - f.bias)                          /* subnormal: exponent field 0 */
    return sign | (uint32_t)ldexp(q, f.bias - 1 + f.man_bits);
  uint32_t man = (uint32_t)ldexp(q, f.man_bits - binade) - (1u << f.man_bits);
  return sign | ((uint32_t)(binade + f.bias) << f.man_bits) | man;
}

static float load_as_fp32(const void *base, uint64_t i, uint32_t fmt, float scale) {
  float reciprocal = 1.0f / scale;
  if (fmt == ORC_FMT_F32) return ((const float *)base)[i];
  uint32_t bits = orc_fmt_bytes(fmt) == 2 ? ((const uint16_t *)base)[i] : ((const uint8_t *)base)[i];
  float stored = (float)orc_decode(fmt, bits);      /* exact: every such value is an FP32 value */
  return stored * reciprocal;
}

static void store_from_fp32(void *base, uint64_t i, uint32_t fmt, float scale, float x) {
  if (fmt == ORC_FMT_F32) {
    ((float *)base)[i] = x;
    return;
  }
  float scaled = x * scale;
  uint32_t bits = orc_encode(fmt, scaled);
  if (orc_fmt_bytes(fmt) == 2) ((uint16_t *)base)[i] = (uint16_t)bits;
  else ((uint8_t *)base)[i] = (uint8_t)bits;
}

/*
 * One optimizer step on a tensor whose state is stored in the given formats
 * (fmt[kind], scale[kind] with kind = master, m, v, compute).  Gradients are FP32.
 */
int orc_adam_tensor_lp(void *p, void *m, void *v, const float *g, void *c, uint64_t n,
                       const orc_adam_hp *hp, uint64_t step, const uint32_t fmt[4], const float scale[4]) {
  for (int k = 0; k < 4; ++k)
    if (orc_fmt_bytes(fmt[k]) == 0) return ORC_BAD_ARG;
  for (uint64_t i = 0; i < n; ++i) {
    float param = load_as_fp32(p, i, fmt[ORC_MASTER], scale[ORC_MASTER]);
    float mom1 = load_as_fp32(m, i, fmt[ORC_ADAM_M], scale[ORC_ADAM_M]);
    float mom2 = load_as_fp32(v, i, fmt[ORC_ADAM_V], scale[ORC_ADAM_V]);
    orc_adam_tensor(&param, &mom1, &mom2, g + i, NULL, 1, hp, step);   /* the FP32 step itself */
    store_from_fp32(p, i, fmt[ORC_MASTER], scale[ORC_MASTER], param);
    store_from_fp32(m, i, fmt[ORC_ADAM_M], scale[ORC_ADAM_M], mom1);
    store_from_fp32(v, i, fmt[ORC_ADAM_V], scale[ORC_ADAM_V], mom2);
    if (c) {
      float as_stored = load_as_fp32(p, i, fmt[ORC_MASTER], scale[ORC_MASTER]);
      store_from_fp32(c, i, fmt[ORC_COMPUTE], scale[ORC_COMPUTE], as_stored);
    }
  }
  return ORC_OK;
}

/* replay step for a model whose state is stored in `fmt`; scales = [4][n_tensors] (kind-major)
 * or NULL for all ones */
int orc_replay_step_lp(const orc_model *mdl, const uint32_t fmt[4], const orc_adam_hp *hp, uint64_t step,
                       const uint8_t *active_mask, const float *const *grads, const orc_state *st,
                       const float *scales) {
  if (!mdl || !fmt || !hp || !active_mask || !grads || !st || step == 0) return ORC_BAD_ARG;
  if (orc_fmt_bytes(fmt[0]) != mdl->width.master || orc_fmt_bytes(fmt[1]) != mdl->width.m ||
      orc_fmt_bytes(fmt[2]) != mdl->width.v || orc_fmt_bytes(fmt[3]) != mdl->width.compute)
    return ORC_BAD_ARG;
  for (uint32_t t = 0; t < mdl->n_tensors; ++t) {
    if (!active_mask[mdl->tensors[t].op]) continue;
    float s[4] = {1.0f, 1.0f, 1.0f, 1.0f};
    if (scales)
      for (uint32_t k = 0; k < 4; ++k) s[k] = scales[(uint64_t)k * mdl->n_tensors + t];
    int rc = orc_adam_tensor_lp(st->master[t], st->m[t], st->v[t], grads[t], st->compute[t],
                                mdl->tensors[t].numel, hp, step, fmt, s);
    if (rc != ORC_OK) return rc;
  }
  return ORC_OK;
}
