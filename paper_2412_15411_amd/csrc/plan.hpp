// plan.hpp -- host-side checkpoint plan: window schedule (Algorithm 1, Sec. 3.5) and the
// per-slot segment tables of the packed snapshot (Sec. 3.2).  Pure C++, no GPU calls.
#pragma once

#include <cstdint>
#include <string>
#include <vector>

#include "moev.h"

namespace moev {

struct HostSlot {
  uint32_t first_segment = 0;   // index of the slot's first segment in Plan::segments
  uint32_t n_segments = 0;
  uint64_t packed_bytes = 0;    // header + padded segments
};

struct HostPlan {
  uint32_t n_ops = 0, n_tensors = 0, window = 0, n_active = 0, align = 256;
  uint8_t width[4] = {4, 4, 4, 2};            // bytes per element, indexed by MOEV_KIND_*
  uint8_t fmt[4] = {MOEV_FMT_F32, MOEV_FMT_F32, MOEV_FMT_F32, MOEV_FMT_BF16};  // MOEV_FMT_*, 0 = copy only
  std::vector<moev_tensor> tensors;
  std::vector<uint32_t> order;                 // O_Ordered
  std::vector<uint32_t> slot_of_op;
  std::vector<uint32_t> first_tensor_of_op;    // [n_ops + 1]
  std::vector<moev_segment> segments;          // all slots, slot after slot (host-computed offsets)
  std::vector<HostSlot> slots;
  uint64_t hash = 0;
};

// Builds the plan from the caller's configuration.  Returns MOEV_OK or an error code and a
// message in `err`.
int build_plan(const moev_plan_cfg& cfg, HostPlan& plan, std::string& err);

int find_window_size(uint32_t n_ops, double t_iter, double s_compute, double s_master, double s_optim,
                     double link_bps, uint32_t* window, uint32_t* n_active);
void order_operators(uint32_t n_ops, const double* popularity, uint32_t* order);

inline uint64_t round_up(uint64_t x, uint64_t a) { return (x + a - 1) & ~(a - 1); }

}  // namespace moev
