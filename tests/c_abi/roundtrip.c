/* Plain C user of the C ABI (no Python, no PyTorch): plan -> pack -> drain -> poison -> fused
 * conversion step -> compare.  Built and run by tests/test_c_abi.py. */
#include <hip/hip_runtime_api.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "moev.h"

#define CHECK_HIP(x) do { hipError_t e_ = (x); if (e_ != hipSuccess) { printf("HIP error %s line %d\n", hipGetErrorString(e_), __LINE__); return 2; } } while (0)
#define CHECK_MOEV(x) do { int r_ = (x); if (r_ != MOEV_OK) { printf("moev error %d (%s) line %d\n", r_, moev_last_error(), __LINE__); return 3; } } while (0)

enum { N_OPS = 4, N_TENSORS = 8 };

int main(void) {
  moev_tensor tensors[N_TENSORS];
  uint32_t slots[N_OPS] = {0, 0, 1, 1};
  size_t numel[N_TENSORS];
  for (int t = 0; t < N_TENSORS; ++t) {
    tensors[t].op = (uint32_t)(t / 2);
    tensors[t].numel = numel[t] = 5000u + 1237u * (unsigned)t;
  }
  moev_plan_cfg cfg;
  memset(&cfg, 0, sizeof cfg);
  cfg.n_ops = N_OPS;
  cfg.n_tensors = N_TENSORS;
  cfg.tensors = tensors;
  cfg.mode = MOEV_EXPLICIT;
  cfg.window = 2;
  cfg.slot_of_op = slots;
  moev_plan* plan = NULL;
  CHECK_MOEV(ckpt_plan(&cfg, &plan));

  void *master[N_TENSORS], *m[N_TENSORS], *v[N_TENSORS], *c[N_TENSORS], *g[N_TENSORS];
  float* h_ref[N_TENSORS];
  for (int t = 0; t < N_TENSORS; ++t) {
    size_t n = numel[t];
    h_ref[t] = (float*)malloc(n * 4);
    for (size_t i = 0; i < n; ++i) h_ref[t][i] = 0.001f * (float)((i * 7 + (size_t)t) % 1000) - 0.5f;
    CHECK_HIP(hipMalloc(&master[t], n * 4));
    CHECK_HIP(hipMalloc(&m[t], n * 4));
    CHECK_HIP(hipMalloc(&v[t], n * 4));
    CHECK_HIP(hipMalloc(&c[t], n * 2));
    CHECK_HIP(hipMalloc(&g[t], n * 4));
    CHECK_HIP(hipMemcpy(master[t], h_ref[t], n * 4, hipMemcpyHostToDevice));
    CHECK_HIP(hipMemset(m[t], 0, n * 4));
    CHECK_HIP(hipMemset(v[t], 0, n * 4));
    CHECK_HIP(hipMemset(c[t], 0, n * 2));
    CHECK_HIP(hipMemset(g[t], 0, n * 4));   /* zero gradients: the replayed step leaves the weights alone */
  }
  moev_state st = {master, m, v, c};
  size_t cap = ckpt_plan_max_packed_bytes(plan);
  void *d_packed, *h_packed[2];
  uint8_t* d_mask;
  CHECK_HIP(hipMalloc(&d_packed, cap));
  CHECK_HIP(hipMalloc((void**)&d_mask, N_OPS));
  CHECK_HIP(hipMemset(d_mask, 0, N_OPS));
  hipStream_t main_s, side_s;
  hipEvent_t packed_ev;
  CHECK_HIP(hipStreamCreate(&main_s));
  CHECK_HIP(hipStreamCreate(&side_s));
  CHECK_HIP(hipEventCreate(&packed_ev));
  for (uint32_t k = 0; k < 2; ++k) {
    CHECK_HIP(hipHostMalloc(&h_packed[k], cap, hipHostMallocDefault));
    CHECK_MOEV(snapshot_pack(plan, k, 10 + k, &st, d_packed, cap, main_s));
    CHECK_HIP(hipEventRecord(packed_ev, main_s));
    CHECK_MOEV(snapshot_drain(plan, k, d_packed, h_packed[k], cap, side_s, packed_ev, NULL));
    CHECK_HIP(hipStreamSynchronize(side_s));
    moev_header hd;
    CHECK_MOEV(snapshot_peek(plan, k, h_packed[k], &hd));
    if (hd.iter != 10 + k || hd.slot != k) return printf("bad header\n"), 4;
  }
  for (int t = 0; t < N_TENSORS; ++t) CHECK_HIP(hipMemset(master[t], 0xff, numel[t] * 4));   /* lose the state */
  moev_adam adam = {1e-4f, 0.9f, 0.95f, 1e-8f, 0.0f, 11};
  for (uint32_t k = 0; k < 2; ++k) {
    void* grads[N_TENSORS];
    for (int t = 0; t < N_TENSORS; ++t) grads[t] = slots[t / 2] <= k ? g[t] : NULL;
    adam.step = 11 + k;
    CHECK_MOEV(convert_window_step(plan, k, h_packed[k], d_packed, &adam, d_mask, grads, &st, main_s));
  }
  CHECK_HIP(hipStreamSynchronize(main_s));
  CHECK_MOEV(ckpt_plan_device_status(plan, main_s));
  for (int t = 0; t < N_TENSORS; ++t) {
    float* back = (float*)malloc(numel[t] * 4);
    CHECK_HIP(hipMemcpy(back, master[t], numel[t] * 4, hipMemcpyDeviceToHost));
    if (memcmp(back, h_ref[t], numel[t] * 4) != 0) return printf("tensor %d differs\n", t), 5;
    free(back);
  }
  uint8_t mask[N_OPS];
  CHECK_HIP(hipMemcpy(mask, d_mask, N_OPS, hipMemcpyDeviceToHost));
  for (int e = 0; e < N_OPS; ++e)
    if (mask[e] != 1) return printf("operator %d not active\n", e), 6;
  ckpt_plan_free(plan);

  /* The same operators with the state stored in a low-precision regime (Sec. 5.6): 8-bit master weights,
   * 8-bit first and 16-bit second moments, 8-bit compute weights, one scale per tensor and kind.  With zero
   * gradients and zero first moments the step leaves the stored master weights alone and casts the compute
   * weights from them (same format, same scale: the same codes). */
  memset(&cfg, 0, sizeof cfg);
  cfg.n_ops = N_OPS;
  cfg.n_tensors = N_TENSORS;
  cfg.tensors = tensors;
  cfg.mode = MOEV_EXPLICIT;
  cfg.window = 2;
  cfg.slot_of_op = slots;
  cfg.master_fmt = MOEV_FMT_E4M3;
  cfg.m_fmt = MOEV_FMT_E4M3;
  cfg.v_fmt = MOEV_FMT_F16;
  cfg.compute_fmt = MOEV_FMT_E4M3;
  CHECK_MOEV(ckpt_plan(&cfg, &plan));
  if (ckpt_plan_width(plan, MOEV_KIND_MASTER) != 1 || ckpt_plan_width(plan, MOEV_KIND_ADAM_V) != 2) return printf("bad widths\n"), 7;
  uint8_t* h_codes[N_TENSORS];
  for (int t = 0; t < N_TENSORS; ++t) {
    size_t n = numel[t];
    h_codes[t] = (uint8_t*)malloc(n);
    for (size_t i = 0; i < n; ++i) {
      uint8_t code = (uint8_t)((i * 13 + (size_t)t) & 0xff);
      if ((code & 0x7f) == 0x7f || (code & 0x7f) == 0) code = 0x38;   /* no NaN, no zero (a zero keeps its value, not its sign) */
      h_codes[t][i] = code;
    }
    CHECK_HIP(hipMemcpy(master[t], h_codes[t], n, hipMemcpyHostToDevice));   /* the FP32-sized allocations are large enough */
    CHECK_HIP(hipMemset(m[t], 0, n));
    CHECK_HIP(hipMemset(v[t], 0x3c, n * 2));    /* 0x3c3c: a positive FP16 value */
    CHECK_HIP(hipMemset(c[t], 0, n));
  }
  float h_scales[4 * N_TENSORS], *d_scales;
  for (int k = 0; k < 4; ++k)
    for (int t = 0; t < N_TENSORS; ++t) h_scales[k * N_TENSORS + t] = (k == 0 || k == 3) ? 1024.0f : 4096.0f;
  CHECK_HIP(hipMalloc((void**)&d_scales, sizeof h_scales));
  CHECK_HIP(hipMemcpy(d_scales, h_scales, sizeof h_scales, hipMemcpyHostToDevice));
  uint8_t ones[N_OPS] = {1, 1, 1, 1};
  CHECK_HIP(hipMemcpy(d_mask, ones, N_OPS, hipMemcpyHostToDevice));
  moev_adam lp = {1e-3f, 0.9f, 0.95f, 1e-8f, 0.0f, 12, NULL};
  lp.d_scales = d_scales;
  CHECK_MOEV(convert_replay(plan, &lp, d_mask, g, &st, main_s));
  CHECK_HIP(hipStreamSynchronize(main_s));
  CHECK_MOEV(ckpt_plan_device_status(plan, main_s));
  for (int t = 0; t < N_TENSORS; ++t) {
    uint8_t* back = (uint8_t*)malloc(numel[t]);
    CHECK_HIP(hipMemcpy(back, master[t], numel[t], hipMemcpyDeviceToHost));
    if (memcmp(back, h_codes[t], numel[t]) != 0) return printf("low-precision master %d changed\n", t), 8;
    CHECK_HIP(hipMemcpy(back, c[t], numel[t], hipMemcpyDeviceToHost));
    if (memcmp(back, h_codes[t], numel[t]) != 0) return printf("low-precision compute %d is not the cast of the master weights\n", t), 9;
    free(back);
  }
  ckpt_plan_free(plan);
  printf("ok\n");
  return 0;
}
