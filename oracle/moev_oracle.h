/*
 * moev_oracle.h -- plain CPU oracle for sparse snapshot / sparse-to-dense conversion.
 *
 * TEST INFRASTRUCTURE ONLY.  This is the slow, obviously-correct statement of what the
 * GPU library computes, written from the paper (MoEvement, arXiv 2412.15411).  It shares
 * no code, header, table or helper with the HIP library and must never be linked, loaded
 * or called by it.  Only tests, the smoke check and the bench's cpu_baseline leg use it.
 *
 * Every function cites the passage of the paper it restates.  Where the paper is silent
 * (packed layout, header, alignment, Adam operation order) the reading taken is stated
 * next to the function.
 *
 * Single-threaded C99, built with -O2 -ffp-contract=off (no fused multiply-add, so the
 * fp32 operation order written in the source is the order executed).
 */
#ifndef MOEV_ORACLE_H
#define MOEV_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* kinds of state an operator holds per tensor (Sec. 3.2: master weights, optimizer
 * state = Adam first and second moment, compute weights) */
enum { ORC_MASTER = 0, ORC_ADAM_M = 1, ORC_ADAM_V = 2, ORC_COMPUTE = 3 };

enum { ORC_OK = 0, ORC_BAD_ARG = -1, ORC_NOT_A_SCHEDULE = -2, ORC_TOO_SMALL = -3, ORC_BAD_SNAPSHOT = -4 };

#define ORC_HEADER_BYTES 256u

/* one parameter tensor of operator `op`; tensors of one operator are listed together,
 * operators in ascending id */
typedef struct {
  uint32_t op;
  uint64_t numel;
} orc_tensor;

/* element width in bytes of each kind (FP32 master + FP32 Adam moments + 2-byte compute
 * weights is the paper's default regime: 12 vs 2 bytes per parameter, Sec. 3.2; the
 * low-precision regimes of Sec. 5.6 use other widths, e.g. FP8 master + FP8/FP16 moments) */
typedef struct {
  uint32_t master, m, v, compute;
} orc_widths;

typedef struct {
  uint32_t kind;   /* ORC_* */
  uint32_t tensor; /* index into the tensor list */
  uint64_t nbytes; /* numel * width(kind) */
  uint64_t dst_off;/* byte offset inside the packed snapshot */
} orc_segment;

/* the model and its checkpoint schedule */
typedef struct {
  uint32_t n_ops, n_tensors;
  const orc_tensor *tensors;
  const uint32_t *order;      /* O_Ordered of Algorithm 1: a permutation of the operators */
  const uint32_t *slot_of_op; /* window slot in which the operator is active */
  uint32_t window;            /* W_sparse */
  uint32_t align;             /* segment alignment in the packed snapshot */
  orc_widths width;
  uint32_t fmt[4];            /* ORC_FMT_* of master, m, v, compute; 0 = by element width */
} orc_model;

/* dense training state, one host pointer per tensor and kind */
typedef struct {
  void *const *master;
  void *const *m;
  void *const *v;
  void *const *compute;
} orc_state;

typedef struct {
  float lr, beta1, beta2, eps, weight_decay;
} orc_adam_hp;

/* ---- schedule (Algorithm 1) ------------------------------------------------------ */
int orc_find_window_size(uint32_t o_total, double t_iter, double s_compute, double s_master,
                         double s_optim, double b_pcie, uint32_t *w_sparse, uint32_t *o_active);
int orc_generate_schedule(uint32_t n_ops, const uint32_t *order, uint32_t o_active,
                          uint32_t *slot_of_op, uint32_t *w_sparse);
int orc_order_by_popularity(uint32_t n_ops, const double *popularity, uint32_t *order);
int orc_check_schedule(uint32_t n_ops, const uint32_t *order, const uint32_t *slot_of_op,
                       uint32_t window);

/* ---- alternative popularity estimates (App. B) and the efficiency model (Sec. 2.4, Sec. 3.6) --- */
void orc_popularity_time_decayed(uint32_t n_ops, double alpha, const double *previous, const double *batch_count,
                                 double *out);
void orc_popularity_capacity_aware(uint32_t n_ops, const double *popularity, const double *capacity, double *out);
double orc_ettr(double t_ckpt, double t_iter, double ckpt_interval, double expected_recovery, double mtbf);
void orc_recovery_dense(double ckpt_interval, double t_iter, double *expected, double *worst);
void orc_recovery_sparse(double w_sparse, double t_iter, double *expected, double *worst);

/* ---- snapshot layout, pack, unpack (Sec. 3.2, Sec. 3.3) ---------------------------- */
uint64_t orc_fnv1a64(const void *bytes, uint64_t n);   /* the hash function itself, over a byte string */
uint64_t orc_plan_hash(const orc_model *mdl);
int64_t orc_layout(const orc_model *mdl, uint32_t slot, orc_segment *segs, uint64_t seg_cap,
                   uint64_t *packed_bytes);
int orc_pack(const orc_model *mdl, uint32_t slot, uint64_t iter, const orc_state *st,
             uint8_t *packed, uint64_t cap);
int orc_unpack(const orc_model *mdl, uint32_t slot, const uint8_t *packed, uint64_t packed_len,
               const orc_state *st, uint8_t *active_mask, uint64_t *iter_out);

/* ---- optimizer replay (Sec. 3.3) --------------------------------------------------- */
uint16_t orc_bf16_rne(float x);
void orc_bias_corrections(const orc_adam_hp *hp, uint64_t step, float *bc1, float *bc2);
void orc_adam_tensor(float *p, float *m, float *v, const float *g, uint16_t *c, uint64_t n,
                     const orc_adam_hp *hp, uint64_t step);
int orc_replay_step(const orc_model *mdl, const orc_adam_hp *hp, uint64_t step,
                    const uint8_t *active_mask, const float *const *grads, const orc_state *st);

/* ---- low-precision training state (Sec. 5.6) ------------------------------------------- */
/* storage formats of master weights, Adam moments and compute weights in the regimes the paper
 * evaluates: FP32, FP16 (IEEE binary16), bfloat16 and the two 8-bit formats (4 exponent + 3
 * mantissa bits without infinities; 5 exponent + 2 mantissa bits, IEEE-like) */
enum { ORC_FMT_F32 = 1, ORC_FMT_F16 = 2, ORC_FMT_BF16 = 3, ORC_FMT_E4M3 = 4, ORC_FMT_E5M2 = 5 };

uint32_t orc_fmt_bytes(uint32_t fmt);
double orc_decode(uint32_t fmt, uint32_t bits);
uint32_t orc_encode(uint32_t fmt, float x);
int orc_adam_tensor_lp(void *p, void *m, void *v, const float *g, void *c, uint64_t n,
                       const orc_adam_hp *hp, uint64_t step, const uint32_t fmt[4], const float scale[4]);
int orc_replay_step_lp(const orc_model *mdl, const uint32_t fmt[4], const orc_adam_hp *hp, uint64_t step,
                       const uint8_t *active_mask, const float *const *grads, const orc_state *st,
                       const float *scales);

#ifdef __cplusplus
}
#endif
#endif
