// plan.cpp -- host-side checkpoint plan (Algorithm 1 and the snapshot layout).
#include "plan.hpp"

#include <algorithm>
#include <cmath>
#include <cstring>
#include <numeric>

namespace moev {

// FindWindowSize of Algorithm 1 (Sec. 3.5): the largest number of simultaneously
// checkpointed operators whose snapshot still drains within one iteration.  Candidates are
// tried from "all operators" downwards; the search stops at two (it never tries one, and does
// not test the fit at two).  W_sparse = ceil(O_Total / O_Active).
int find_window_size(uint32_t n_ops, double t_iter, double s_compute, double s_master, double s_optim,
                     double link_bps, uint32_t* window, uint32_t* n_active) {
  if (n_ops == 0 || !window || !n_active || !(link_bps > 0.0) || std::isnan(t_iter)) return MOEV_E_INVAL;
  uint32_t chosen = n_ops <= 2 ? n_ops : 2;
  for (uint32_t candidate = n_ops; candidate > 2; --candidate) {
    const double full = (s_master + s_optim) * static_cast<double>(candidate);
    const double light = s_compute * static_cast<double>(n_ops - candidate);
    if ((full + light) / link_bps <= t_iter) {
      chosen = candidate;
      break;
    }
  }
  *n_active = chosen;
  *window = (n_ops + chosen - 1) / chosen;
  return MOEV_OK;
}

// OrderOperators (Sec. 3.5): ascending popularity so that popular experts are checkpointed
// last and stay frozen longest during conversion; equal popularity keeps ascending id.
void order_operators(uint32_t n_ops, const double* popularity, uint32_t* order) {
  std::iota(order, order + n_ops, 0u);
  std::stable_sort(order, order + n_ops,
                   [&](uint32_t a, uint32_t b) { return popularity[a] < popularity[b]; });
}

namespace {

struct Fnv1a {
  uint64_t h = 0xcbf29ce484222325ull;
  template <typename T>
  void add(T value) {
    unsigned char raw[sizeof(T)];
    std::memcpy(raw, &value, sizeof(T));  // little-endian host
    for (unsigned char byte : raw) {
      h ^= byte;
      h *= 0x100000001b3ull;
    }
  }
};

bool is_pow2(uint64_t x) { return x && !(x & (x - 1)); }

}  // namespace

int build_plan(const moev_plan_cfg& cfg, HostPlan& p, std::string& err) {
  if (cfg.n_ops == 0 || cfg.n_tensors == 0 || !cfg.tensors) {
    err = "ckpt_plan: need at least one operator and one tensor";
    return MOEV_E_INVAL;
  }
  p.n_ops = cfg.n_ops;
  p.n_tensors = cfg.n_tensors;
  p.align = cfg.align ? cfg.align : 256;
  if (!is_pow2(p.align) || p.align < 16 || p.align > (1u << 24)) {
    err = "ckpt_plan: align must be a power of two in [16, 2^24]";
    return MOEV_E_INVAL;
  }
  // element widths and storage formats (Sec. 5.6 regimes); either may be left to the other
  const uint8_t widths_in[4] = {cfg.master_bytes, cfg.m_bytes, cfg.v_bytes, cfg.compute_bytes};
  const uint8_t fmts_in[4] = {cfg.master_fmt, cfg.m_fmt, cfg.v_fmt, cfg.compute_fmt};
  for (int k = 0; k < 4; ++k) {
    uint8_t w = widths_in[k], f = fmts_in[k];
    if (f > MOEV_FMT_E5M2) {
      err = "ckpt_plan: unknown storage format";
      return MOEV_E_INVAL;
    }
    const uint8_t w_of_f = f == MOEV_FMT_F32 ? 4 : (f == MOEV_FMT_F16 || f == MOEV_FMT_BF16) ? 2 : f ? 1 : 0;
    if (w == 0) w = w_of_f ? w_of_f : (k == MOEV_KIND_COMPUTE ? 2 : 4);
    if (w != 1 && w != 2 && w != 4 && w != 8) {
      err = "ckpt_plan: element widths must be 1, 2, 4 or 8 bytes";
      return MOEV_E_INVAL;
    }
    if (f == MOEV_FMT_DEFAULT)
      f = w == 4 ? MOEV_FMT_F32 : w == 2 ? (k == MOEV_KIND_COMPUTE ? MOEV_FMT_BF16 : MOEV_FMT_F16) : w == 1 ? MOEV_FMT_E4M3 : 0;
    else if (w_of_f != w) {
      err = "ckpt_plan: storage format does not have the given element width";
      return MOEV_E_INVAL;
    }
    p.width[k] = w;
    p.fmt[k] = f;
  }

  // tensors: grouped by operator, operators ascending from 0, every operator present
  p.tensors.assign(cfg.tensors, cfg.tensors + cfg.n_tensors);
  p.first_tensor_of_op.assign(p.n_ops + 1, 0);
  uint32_t expect_op = 0;
  for (uint32_t t = 0; t < p.n_tensors; ++t) {
    const uint32_t op = p.tensors[t].op;
    if (op >= p.n_ops || (t == 0 && op != 0) || (t > 0 && op != expect_op && op != expect_op + 1)) {
      err = "ckpt_plan: tensors must be grouped by operator in ascending operator id, no operator skipped";
      return MOEV_E_INVAL;
    }
    if (p.tensors[t].numel > (1ull << 40)) {
      err = "ckpt_plan: tensor too large";
      return MOEV_E_INVAL;
    }
    if (op != expect_op) {
      expect_op = op;
      p.first_tensor_of_op[op] = t;
    }
  }
  if (expect_op != p.n_ops - 1) {
    err = "ckpt_plan: an operator has no tensor";
    return MOEV_E_INVAL;
  }
  p.first_tensor_of_op[p.n_ops] = p.n_tensors;

  // ---- schedule ----
  p.slot_of_op.assign(p.n_ops, 0);
  p.order.resize(p.n_ops);
  auto is_permutation = [&](const uint32_t* o) {
    std::vector<uint8_t> seen(p.n_ops, 0);
    for (uint32_t j = 0; j < p.n_ops; ++j) {
      if (o[j] >= p.n_ops || seen[o[j]]) return false;
      seen[o[j]] = 1;
    }
    return true;
  };
  if (cfg.mode == MOEV_EXPLICIT) {
    if (!cfg.slot_of_op || cfg.window == 0) {
      err = "ckpt_plan: EXPLICIT mode needs slot_of_op and window";
      return MOEV_E_INVAL;
    }
    p.window = cfg.window;
    p.n_active = 0;
    for (uint32_t e = 0; e < p.n_ops; ++e) {
      if (cfg.slot_of_op[e] >= p.window) {
        err = "ckpt_plan: slot_of_op entry outside the window";
        return MOEV_E_INVAL;
      }
      p.slot_of_op[e] = cfg.slot_of_op[e];
    }
    if (cfg.order) {
      if (!is_permutation(cfg.order)) {
        err = "ckpt_plan: order is not a permutation of the operators";
        return MOEV_E_INVAL;
      }
      std::copy(cfg.order, cfg.order + p.n_ops, p.order.begin());
      for (uint32_t j = 1; j < p.n_ops; ++j)
        if (p.slot_of_op[p.order[j]] < p.slot_of_op[p.order[j - 1]]) {
          err = "ckpt_plan: slots must not decrease along the checkpoint order";
          return MOEV_E_INVAL;
        }
    } else {
      std::iota(p.order.begin(), p.order.end(), 0u);
      std::stable_sort(p.order.begin(), p.order.end(),
                       [&](uint32_t a, uint32_t b) { return p.slot_of_op[a] < p.slot_of_op[b]; });
    }
  } else if (cfg.mode == MOEV_FIXED || cfg.mode == MOEV_AUTO) {
    if (cfg.order) {
      if (!is_permutation(cfg.order)) {
        err = "ckpt_plan: order is not a permutation of the operators";
        return MOEV_E_INVAL;
      }
      std::copy(cfg.order, cfg.order + p.n_ops, p.order.begin());
    } else {
      std::iota(p.order.begin(), p.order.end(), 0u);
    }
    uint32_t per_slot = cfg.n_active;
    if (cfg.mode == MOEV_AUTO) {
      // Algorithm 1 works with one size per operator; operators of different size enter with
      // their mean (equal to the paper's quantities when operators are uniform).
      double params = 0;
      for (const auto& t : p.tensors) params += static_cast<double>(t.numel);
      const double per_op = params / p.n_ops;
      uint32_t w = 0;
      int rc = find_window_size(p.n_ops, cfg.t_iter_s, per_op * p.width[MOEV_KIND_COMPUTE],
                                per_op * p.width[MOEV_KIND_MASTER],
                                per_op * (p.width[MOEV_KIND_ADAM_M] + p.width[MOEV_KIND_ADAM_V]),
                                cfg.host_link_Bps, &w, &per_slot);
      if (rc != MOEV_OK) {
        err = "ckpt_plan: AUTO mode needs t_iter_s and a positive host_link_Bps";
        return rc;
      }
    }
    if (per_slot == 0) {
      err = "ckpt_plan: n_active must be positive";
      return MOEV_E_INVAL;
    }
    // GenerateSchedule: consecutive runs of n_active operators of the checkpoint order
    p.n_active = per_slot;
    p.window = (p.n_ops + per_slot - 1) / per_slot;
    for (uint32_t j = 0; j < p.n_ops; ++j) p.slot_of_op[p.order[j]] = j / per_slot;
  } else {
    err = "ckpt_plan: unknown mode";
    return MOEV_E_INVAL;
  }

  // ---- segment tables: full state of the slot's operators, then compute weights of later ones ----
  std::vector<std::vector<uint32_t>> ops_of_slot(p.window);
  for (uint32_t j = 0; j < p.n_ops; ++j) ops_of_slot[p.slot_of_op[p.order[j]]].push_back(p.order[j]);
  p.slots.assign(p.window, HostSlot{});
  p.segments.clear();
  const uint64_t first_offset = round_up(MOEV_HEADER_BYTES, p.align);
  for (uint32_t k = 0; k < p.window; ++k) {
    HostSlot& slot = p.slots[k];
    slot.first_segment = static_cast<uint32_t>(p.segments.size());
    uint64_t cursor = first_offset;
    auto emit = [&](uint32_t kind, uint32_t tensor) {
      const uint64_t nbytes = p.tensors[tensor].numel * p.width[kind];
      p.segments.push_back(moev_segment{kind, tensor, nbytes, cursor});
      cursor += round_up(nbytes, p.align);
    };
    for (uint32_t e : ops_of_slot[k])
      for (uint32_t t = p.first_tensor_of_op[e]; t < p.first_tensor_of_op[e + 1]; ++t) {
        emit(MOEV_KIND_MASTER, t);
        emit(MOEV_KIND_ADAM_M, t);
        emit(MOEV_KIND_ADAM_V, t);
      }
    for (uint32_t later = k + 1; later < p.window; ++later)
      for (uint32_t e : ops_of_slot[later])
        for (uint32_t t = p.first_tensor_of_op[e]; t < p.first_tensor_of_op[e + 1]; ++t)
          emit(MOEV_KIND_COMPUTE, t);
    slot.n_segments = static_cast<uint32_t>(p.segments.size()) - slot.first_segment;
    slot.packed_bytes = cursor;
    if (p.segments.size() > 0x7fffffffull) {
      err = "ckpt_plan: too many segments";
      return MOEV_E_INVAL;
    }
  }

  Fnv1a f;
  f.add<uint32_t>(p.n_ops);
  f.add<uint32_t>(p.n_tensors);
  f.add<uint32_t>(p.window);
  f.add<uint32_t>(p.align);
  f.add<uint8_t>(p.width[MOEV_KIND_MASTER]);
  f.add<uint8_t>(p.width[MOEV_KIND_ADAM_M]);
  f.add<uint8_t>(p.width[MOEV_KIND_ADAM_V]);
  f.add<uint8_t>(p.width[MOEV_KIND_COMPUTE]);
  // the storage formats too: an F16 snapshot must not load into a BF16 plan of the same widths
  for (uint8_t fmt : p.fmt) f.add<uint8_t>(fmt);
  for (const auto& t : p.tensors) {
    f.add<uint32_t>(t.op);
    f.add<uint64_t>(t.numel);
  }
  for (uint32_t s : p.slot_of_op) f.add<uint32_t>(s);
  for (uint32_t o : p.order) f.add<uint32_t>(o);
  p.hash = f.h;
  return MOEV_OK;
}

}  // namespace moev
