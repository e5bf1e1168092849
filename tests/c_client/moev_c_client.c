/*
 * moev_c_client.c -- a plain C99 client of libmoev's C ABI (test infrastructure): no Python, no PyTorch.
 *
 * Reads a workload from a binary file, runs the hot path of Sec. 3.2 / 3.3 through the calls of moev.h with device
 * memory from hipMalloc and pinned host memory from hipHostMalloc, and writes what the path produced to another
 * file; tests/test_gpu_c_client.py generates the input, runs this program and compares the output with the oracle.
 *
 *   run in the program:  dense training run t0 .. t0+W: snapshot_pack + snapshot_drain of slot k after iteration
 *   t0+k (side stream, event-ordered), then convert_replay of iteration t0+k+1 on every operator; afterwards a
 *   conversion into a poisoned state: restore_unpack from the pinned host copies + convert_replay on the active
 *   operators (frozen operators get NULL gradients).
 *
 * input  (little endian): u32 magic 0x4d4f4556, u32 n_ops, u32 n_tensors, u32 window, u64 t0, f32 lr, beta1, beta2,
 *         eps, weight_decay; per tensor u32 op, u64 numel; per operator u32 slot; per operator u32 order;
 *         per tensor: master f32[n], m f32[n], v f32[n], compute u16[n]; per iteration 1..W, per tensor: gradient f32[n].
 * output: u32 magic; per slot u64 packed_bytes, then the drained snapshot; then the dense run's final state and the
 *         converted state, each per tensor master, m, v (f32[n]) and compute (u16[n]); then the final mask u8[n_ops].
 */
#define __HIP_PLATFORM_AMD__ 1
#include <hip/hip_runtime_api.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "moev.h"

#define MAGIC 0x4d4f4556u
#define HIP(call)                                                                         \
  do {                                                                                    \
    hipError_t e_ = (call);                                                               \
    if (e_ != hipSuccess) {                                                               \
      fprintf(stderr, "%s:%d: %s: %s\n", __FILE__, __LINE__, #call, hipGetErrorString(e_)); \
      return 2;                                                                           \
    }                                                                                     \
  } while (0)
#define MOEV(call)                                                                              \
  do {                                                                                          \
    int rc_ = (call);                                                                           \
    if (rc_ != MOEV_OK) {                                                                       \
      fprintf(stderr, "%s:%d: %s -> %d: %s\n", __FILE__, __LINE__, #call, rc_, moev_last_error()); \
      return 3;                                                                                 \
    }                                                                                           \
  } while (0)

static int read_exact(FILE *f, void *dst, size_t n) { return n == 0 || fread(dst, 1, n, f) == n ? 0 : -1; }
static int write_exact(FILE *f, const void *src, size_t n) { return n == 0 || fwrite(src, 1, n, f) == n ? 0 : -1; }

/* the four kinds of one copy of the state on the device */
typedef struct {
  void **ptr[4]; /* [kind][tensor] */
} dev_state;

static const size_t kWidth[4] = {4, 4, 4, 2};

static int alloc_state(dev_state *s, uint32_t n_tensors, const moev_tensor *tensors) {
  for (int k = 0; k < 4; ++k) {
    s->ptr[k] = (void **)calloc(n_tensors ? n_tensors : 1, sizeof(void *));
    if (!s->ptr[k]) return 1;
    for (uint32_t t = 0; t < n_tensors; ++t) {
      /* an empty tensor still needs a valid, aligned pointer */
      size_t bytes = (size_t)tensors[t].numel * kWidth[k];
      HIP(hipMalloc(&s->ptr[k][t], bytes ? bytes : 16));
    }
  }
  return 0;
}

int main(int argc, char **argv) {
  if (argc != 3) {
    fprintf(stderr, "usage: %s <input file> <output file>\n", argv[0]);
    return 1;
  }
  FILE *in = fopen(argv[1], "rb");
  if (!in) {
    perror(argv[1]);
    return 1;
  }
  uint32_t head[4];
  uint64_t t0;
  float hp[5];
  if (read_exact(in, head, sizeof head) || head[0] != MAGIC || read_exact(in, &t0, 8) || read_exact(in, hp, sizeof hp)) {
    fprintf(stderr, "bad input header\n");
    return 1;
  }
  const uint32_t n_ops = head[1], n_tensors = head[2], window = head[3];
  moev_tensor *tensors = (moev_tensor *)calloc(n_tensors, sizeof *tensors);
  uint32_t *slot_of_op = (uint32_t *)calloc(n_ops, 4), *order = (uint32_t *)calloc(n_ops, 4);
  if (!tensors || !slot_of_op || !order) return 1;
  for (uint32_t t = 0; t < n_tensors; ++t)
    if (read_exact(in, &tensors[t].op, 4) || read_exact(in, &tensors[t].numel, 8)) return 1;
  if (read_exact(in, slot_of_op, 4 * (size_t)n_ops) || read_exact(in, order, 4 * (size_t)n_ops)) return 1;

  HIP(hipSetDevice(0));
  hipStream_t main_stream, side_stream;
  HIP(hipStreamCreateWithFlags(&main_stream, hipStreamNonBlocking));
  HIP(hipStreamCreateWithFlags(&side_stream, hipStreamNonBlocking));

  /* state of the dense run, a second copy to convert into, gradients of every iteration */
  dev_state live, rebuilt;
  if (alloc_state(&live, n_tensors, tensors) || alloc_state(&rebuilt, n_tensors, tensors)) return 2;
  size_t max_bytes = 16;
  for (uint32_t t = 0; t < n_tensors; ++t)
    if ((size_t)tensors[t].numel * 4 > max_bytes) max_bytes = (size_t)tensors[t].numel * 4;
  void *staging = malloc(max_bytes);
  if (!staging) return 1;
  for (uint32_t t = 0; t < n_tensors; ++t)
    for (int k = 0; k < 4; ++k) {
      size_t bytes = (size_t)tensors[t].numel * kWidth[k];
      if (read_exact(in, staging, bytes)) return 1;
      HIP(hipMemcpy(live.ptr[k][t], staging, bytes, hipMemcpyHostToDevice));
      memset(staging, 0x7f, bytes); /* the conversion target starts from garbage */
      HIP(hipMemcpy(rebuilt.ptr[k][t], staging, bytes, hipMemcpyHostToDevice));
    }
  void ***grads = (void ***)calloc(window, sizeof *grads);
  if (!grads) return 1;
  for (uint32_t i = 0; i < window; ++i) {
    grads[i] = (void **)calloc(n_tensors ? n_tensors : 1, sizeof(void *));
    if (!grads[i]) return 1;
    for (uint32_t t = 0; t < n_tensors; ++t) {
      size_t bytes = (size_t)tensors[t].numel * 4;
      HIP(hipMalloc(&grads[i][t], bytes ? bytes : 16));
      if (read_exact(in, staging, bytes)) return 1;
      HIP(hipMemcpy(grads[i][t], staging, bytes, hipMemcpyHostToDevice));
    }
  }
  fclose(in);

  moev_plan_cfg cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_ops = n_ops;
  cfg.n_tensors = n_tensors;
  cfg.tensors = tensors;
  cfg.mode = MOEV_EXPLICIT;
  cfg.window = window;
  cfg.order = order;
  cfg.slot_of_op = slot_of_op;
  moev_plan *plan = NULL;
  MOEV(ckpt_plan(&cfg, &plan));
  MOEV(ckpt_plan_upload(plan, main_stream));

  const size_t cap = (size_t)ckpt_plan_max_packed_bytes(plan);
  void *d_packed = NULL;
  HIP(hipMalloc(&d_packed, cap));
  void **h_packed = (void **)calloc(window, sizeof(void *));
  hipEvent_t *packed_ev = (hipEvent_t *)calloc(window, sizeof(hipEvent_t)), *drained_ev = (hipEvent_t *)calloc(window, sizeof(hipEvent_t));
  uint8_t *d_mask = NULL, *d_everyone = NULL;
  HIP(hipMalloc((void **)&d_mask, n_ops ? n_ops : 1));
  HIP(hipMalloc((void **)&d_everyone, n_ops ? n_ops : 1));
  HIP(hipMemset(d_mask, 0, n_ops));
  HIP(hipMemset(d_everyone, 1, n_ops));

  const moev_state live_state = {live.ptr[0], live.ptr[1], live.ptr[2], live.ptr[3]};
  const moev_state rebuilt_state = {rebuilt.ptr[0], rebuilt.ptr[1], rebuilt.ptr[2], rebuilt.ptr[3]};
  moev_adam adam = {hp[0], hp[1], hp[2], hp[3], hp[4], 0, NULL};

  /* dense run with a sparse snapshot every iteration (Sec. 3.2): the pack of slot k takes the state after
   * iteration t0+k; its drain runs on the side stream while iteration t0+k+1 is replayed on the main stream.
   * One packed device buffer is reused, so the next pack waits for the previous drain. */
  for (uint32_t k = 0; k < window; ++k) {
    HIP(hipHostMalloc(&h_packed[k], cap, hipHostMallocDefault));
    HIP(hipEventCreateWithFlags(&packed_ev[k], hipEventDisableTiming));
    HIP(hipEventCreateWithFlags(&drained_ev[k], hipEventDisableTiming));
    if (k) HIP(hipStreamWaitEvent(main_stream, drained_ev[k - 1], 0));
    MOEV(snapshot_pack(plan, k, t0 + k, &live_state, d_packed, cap, main_stream));
    HIP(hipEventRecord(packed_ev[k], main_stream));
    MOEV(snapshot_drain(plan, k, d_packed, h_packed[k], cap, side_stream, packed_ev[k], drained_ev[k]));
    adam.step = t0 + k + 1;
    MOEV(convert_replay(plan, &adam, d_everyone, grads[k], &live_state, main_stream));
  }
  HIP(hipStreamSynchronize(side_stream));
  HIP(hipStreamSynchronize(main_stream));
  MOEV(ckpt_plan_device_status(plan, main_stream));

  /* sparse-to-dense conversion (Sec. 3.3) from the host copies into the garbage-filled state */
  void **active_grads = (void **)calloc(n_tensors ? n_tensors : 1, sizeof(void *));
  if (!active_grads) return 1;
  for (uint32_t i = 0; i < window; ++i) {
    moev_header hd;
    MOEV(snapshot_peek(plan, i, h_packed[i], &hd));
    if (hd.slot != i || hd.iter != t0 + i) {
      fprintf(stderr, "snapshot %u carries slot %u, iteration %llu\n", i, hd.slot, (unsigned long long)hd.iter);
      return 4;
    }
    MOEV(restore_unpack(plan, i, h_packed[i], d_packed, &rebuilt_state, d_mask, main_stream));
    for (uint32_t t = 0; t < n_tensors; ++t) active_grads[t] = slot_of_op[tensors[t].op] <= i ? grads[i][t] : NULL;
    adam.step = t0 + i + 1;
    MOEV(convert_replay(plan, &adam, d_mask, active_grads, &rebuilt_state, main_stream));
  }
  HIP(hipStreamSynchronize(main_stream));
  MOEV(ckpt_plan_device_status(plan, main_stream));

  FILE *out = fopen(argv[2], "wb");
  if (!out) {
    perror(argv[2]);
    return 1;
  }
  const uint32_t magic = MAGIC;
  if (write_exact(out, &magic, 4)) return 1;
  for (uint32_t k = 0; k < window; ++k) {
    const uint64_t n = ckpt_plan_packed_bytes(plan, k);
    if (write_exact(out, &n, 8) || write_exact(out, h_packed[k], (size_t)n)) return 1;
  }
  const dev_state *both[2] = {&live, &rebuilt};
  for (int w = 0; w < 2; ++w)
    for (uint32_t t = 0; t < n_tensors; ++t)
      for (int k = 0; k < 4; ++k) {
        size_t bytes = (size_t)tensors[t].numel * kWidth[k];
        HIP(hipMemcpy(staging, both[w]->ptr[k][t], bytes, hipMemcpyDeviceToHost));
        if (write_exact(out, staging, bytes)) return 1;
      }
  uint8_t *mask = (uint8_t *)malloc(n_ops ? n_ops : 1);
  if (!mask) return 1;
  HIP(hipMemcpy(mask, d_mask, n_ops, hipMemcpyDeviceToHost));
  if (write_exact(out, mask, n_ops) || fclose(out)) return 1;

  ckpt_plan_free(plan);
  /* process exit releases the device and pinned memory */
  printf("moev_c_client: %u operators, %u tensors, window %u: dense run and conversion written\n", n_ops, n_tensors, window);
  return 0;
}
