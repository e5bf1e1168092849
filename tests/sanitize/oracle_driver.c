/* Exercises the CPU oracle under AddressSanitizer / UBSan: exact-size heap buffers, so any access
 * past a tensor or a packed snapshot is reported. */
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "moev_oracle.h"

static uint64_t rng_state = 88172645463325252ull;
static uint64_t rnd(void) {
  rng_state ^= rng_state << 13;
  rng_state ^= rng_state >> 7;
  rng_state ^= rng_state << 17;
  return rng_state;
}

int main(void) {
  for (int iter = 0; iter < 300; ++iter) {
    uint32_t n_ops = 1 + rnd() % 9, n_tensors = 0;
    orc_tensor tensors[32];
    for (uint32_t e = 0; e < n_ops; ++e) {
      uint32_t k = 1 + rnd() % 3;
      for (uint32_t j = 0; j < k; ++j) {
        tensors[n_tensors].op = e;
        tensors[n_tensors].numel = rnd() % 300;
        ++n_tensors;
      }
    }
    uint32_t order[16], slots[16], window = 0, a = 1 + rnd() % n_ops;
    for (uint32_t e = 0; e < n_ops; ++e) order[e] = e;
    for (uint32_t e = n_ops - 1; e > 0; --e) {
      uint32_t j = rnd() % (e + 1), tmp = order[e];
      order[e] = order[j];
      order[j] = tmp;
    }
    if (orc_generate_schedule(n_ops, order, a, slots, &window) != ORC_OK) return 1;
    if (orc_check_schedule(n_ops, order, slots, window) != ORC_OK) return 2;
    const uint32_t aligns[] = {16, 64, 256, 1024};
    orc_model mdl = {n_ops, n_tensors, tensors, order, slots, window, aligns[rnd() % 4], {4, 4, 4, 2}};
    void *master[32], *m[32], *v[32], *c[32];
    float* grads[32];
    for (uint32_t t = 0; t < n_tensors; ++t) {
      size_t n = tensors[t].numel;
      master[t] = malloc(n * 4 + (n == 0));
      m[t] = malloc(n * 4 + (n == 0));
      v[t] = malloc(n * 4 + (n == 0));
      c[t] = malloc(n * 2 + (n == 0));
      grads[t] = (float*)malloc(n * 4 + (n == 0));
      for (size_t i = 0; i < n; ++i) {
        ((float*)master[t])[i] = (float)(rnd() % 2000) * 1e-5f - 0.01f;
        ((float*)m[t])[i] = (float)(rnd() % 2000) * 1e-6f - 0.001f;
        ((float*)v[t])[i] = (float)(rnd() % 2000) * 1e-9f;
        ((uint16_t*)c[t])[i] = (uint16_t)rnd();
        grads[t][i] = (float)(rnd() % 2000) * 1e-6f - 0.001f;
      }
    }
    orc_state st = {master, m, v, c};
    orc_adam_hp hp = {1e-4f, 0.9f, 0.95f, 1e-8f, (iter & 1) ? 0.01f : 0.0f};
    uint8_t mask[16];
    memset(mask, 0, sizeof mask);
    for (uint32_t k = 0; k < window; ++k) {
      uint64_t total = 0, it = 0;
      if (orc_layout(&mdl, k, NULL, 0, &total) < 0) return 3;
      uint8_t* packed = (uint8_t*)malloc(total);
      if (orc_pack(&mdl, k, 10 + k, &st, packed, total) != ORC_OK) return 4;
      if (orc_pack(&mdl, k, 10 + k, &st, packed, total - 1) != ORC_TOO_SMALL) return 5;
      if (orc_unpack(&mdl, k, packed, total, &st, mask, &it) != ORC_OK || it != 10 + k) return 6;
      if (orc_replay_step(&mdl, &hp, 11 + k, mask, (const float* const*)grads, &st) != ORC_OK) return 7;
      free(packed);
    }
    for (uint32_t e = 0; e < n_ops; ++e)
      if (!mask[e]) return 8;
    for (uint32_t t = 0; t < n_tensors; ++t) {
      free(master[t]);
      free(m[t]);
      free(v[t]);
      free(c[t]);
      free(grads[t]);
    }
  }
  printf("ok\n");
  return 0;
}
