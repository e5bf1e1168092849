// Exercises the library's host-side plan builder under AddressSanitizer / UBSan (host code only).
#include <cstdio>
#include <cstdlib>
#include <string>
#include <vector>

#include "plan.hpp"

static uint64_t rng_state = 0x9E3779B97F4A7C15ull;
static uint64_t rnd() {
  rng_state ^= rng_state << 13;
  rng_state ^= rng_state >> 7;
  rng_state ^= rng_state << 17;
  return rng_state;
}

int main() {
  int built = 0, rejected = 0;
  for (int iter = 0; iter < 3000; ++iter) {
    const uint32_t n_ops = 1 + rnd() % 40;
    std::vector<moev_tensor> tensors;
    for (uint32_t e = 0; e < n_ops; ++e) {
      const uint32_t k = 1 + rnd() % 3;
      for (uint32_t j = 0; j < k; ++j) tensors.push_back(moev_tensor{e, rnd() % 5000});
    }
    if (iter % 17 == 0 && tensors.size() > 2) tensors[1].op = n_ops + 3;      // malformed on purpose
    const uint32_t window = 1 + rnd() % 8;
    std::vector<uint32_t> slots(n_ops), order(n_ops);
    for (uint32_t e = 0; e < n_ops; ++e) {
      slots[e] = rnd() % window;
      order[e] = e;
    }
    for (uint32_t e = n_ops - 1; e > 0; --e) std::swap(order[e], order[rnd() % (e + 1)]);
    if (iter % 23 == 0) slots[0] = window + 1;                                // malformed on purpose
    moev_plan_cfg cfg{};
    cfg.n_ops = n_ops;
    cfg.n_tensors = static_cast<uint32_t>(tensors.size());
    cfg.tensors = tensors.data();
    cfg.mode = static_cast<int>(rnd() % 3);
    cfg.window = window;
    cfg.n_active = static_cast<uint32_t>(rnd() % (n_ops + 1));
    cfg.order = (rnd() & 1) ? order.data() : nullptr;
    cfg.slot_of_op = slots.data();
    cfg.t_iter_s = 1e-3 * static_cast<double>(rnd() % 3000);
    cfg.host_link_Bps = (iter % 29 == 0) ? 0.0 : 1e9 + static_cast<double>(rnd() % 1000) * 1e8;
    const uint32_t aligns[] = {0, 16, 64, 256, 4096, 48};
    cfg.align = aligns[rnd() % 6];
    if (cfg.mode == MOEV_EXPLICIT && cfg.order) cfg.order = nullptr;          // a random order rarely respects the slots
    moev::HostPlan plan;
    std::string err;
    const int rc = moev::build_plan(cfg, plan, err);
    if (rc != MOEV_OK) {
      ++rejected;
      continue;
    }
    ++built;
    // every operator active in exactly one slot; offsets aligned and disjoint
    std::vector<int> seen(n_ops, 0);
    for (uint32_t k = 0; k < plan.window; ++k) {
      uint64_t cursor = moev::round_up(MOEV_HEADER_BYTES, plan.align);
      for (uint32_t j = 0; j < plan.slots[k].n_segments; ++j) {
        const moev_segment& s = plan.segments[plan.slots[k].first_segment + j];
        if (s.dst_off != cursor || s.dst_off % plan.align) return std::printf("bad offset\n"), 1;
        cursor += moev::round_up(s.nbytes, plan.align);
        if (s.kind == MOEV_KIND_MASTER && s.tensor == plan.first_tensor_of_op[plan.tensors[s.tensor].op])
          ++seen[plan.tensors[s.tensor].op];
      }
      if (cursor != plan.slots[k].packed_bytes) return std::printf("bad total\n"), 1;
    }
    for (uint32_t e = 0; e < n_ops; ++e)
      if (seen[e] != 1) return std::printf("operator %u has %d full snapshots\n", e, seen[e]), 1;
  }
  std::printf("ok built=%d rejected=%d\n", built, rejected);
  return built > 500 && rejected > 50 ? 0 : 1;
}
