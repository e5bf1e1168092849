// api.hip -- extern "C" boundary of libmoev (declared in include/moev.h): argument checks,
// device tables of the plan, kernel launches, the side-stream drain.  No arithmetic of the
// method happens on the host: every byte moved and every Adam update runs in the kernels.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <mutex>
#include <new>
#include <string>
#include <vector>

#include "kernels.hpp"
#include "moev.h"
#include "plan.hpp"

static_assert(moev::kFmtF32 == MOEV_FMT_F32 && moev::kFmtF16 == MOEV_FMT_F16 && moev::kFmtBF16 == MOEV_FMT_BF16 &&
                  moev::kFmtE4M3 == MOEV_FMT_E4M3 && moev::kFmtE5M2 == MOEV_FMT_E5M2,
              "the kernels' format numbers are the interface's");

namespace {

thread_local std::string g_last_error;

int fail(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}

}  // namespace

namespace moev {
// for the library's other translation units: records the message behind moev_last_error()
int set_error(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}
}  // namespace moev

namespace {

#define MOEV_HIP(call)                                                                     \
  do {                                                                                     \
    hipError_t e_ = (call);                                                                \
    if (e_ != hipSuccess)                                                                  \
      return fail(MOEV_E_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

constexpr uint64_t kMagic = 0x50414e5356454f4dull;  // "MOEVSNAP" read as a little-endian u64
constexpr int kRing = 8;

struct StageSlot {
  void* pinned = nullptr;
  hipEvent_t done = nullptr;
  bool in_flight = false;
};

}  // namespace

// Scratch of convert_replay_static: the compacted tile list of one replay step ([n_tensors + 1] tile numbers),
// in device memory that exists from the moment the library is loaded, so that the call allocates nothing.
// Every GPU holds its own copy of the array at its own address.  In host code the array's name is only a
// handle for hipGetSymbolAddress: kernels and copies are always given the address that call returned.
static __device__ __align__(256) uint32_t scratch[MOEV_STATIC_MAX_TENSORS + 64];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
uint32_t* g_scratch_ptr[kMaxDevices] = {};  // per device: address of that device's `scratch`

// Address of the current device's scratch array (resolved once per device, with that device current).
int scratch_of_current_device(uint32_t** out) {
  int dev = -1;
  MOEV_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) return fail(MOEV_E_INVAL, "device %d is beyond the %d devices this library tracks", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    MOEV_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(MOEV_E_HIP, "hipGetSymbolAddress returned a null address for the scratch array");
    g_scratch_ptr[dev] = static_cast<uint32_t*>(ptr);
  }
  *out = g_scratch_ptr[dev];
  return MOEV_OK;
}

}  // namespace

struct moev_plan {
  moev::HostPlan host;
  std::mutex mu;

  // launch knobs
  int64_t persistent = 0;            // 0: one tile per workgroup, 1: fixed grid walking the tile list
  int64_t copy_threads = 256, copy_unroll = 1;   // one-tile-per-workgroup shape of the pack
  bool copy_unroll_auto = true;      // until MOEV_TUNE_COPY_UNROLL is set: chosen per slot, see pack_unroll()
  int64_t unpack_threads = 128, unpack_unroll = 2;  // ... of the unpack
  int64_t adam_threads = 64, adam_unroll = 1;
  int64_t copy_tile_bytes = 32768;   // fixed-grid shape
  int64_t copy_max_blocks = 0;
  int64_t adam_tile_elems = 8192;
  int64_t adam_max_blocks = 0;
  int64_t nontemporal = 1;
  int64_t xcd_regions = 1;           // replay, one tile per workgroup: 1 = contiguous eighth of the tiles per XCD, 0 = off,
                                     // G >= 2 (power of two) = chunks of G consecutive tiles dealt to the XCDs round robin
  int64_t copy_xcd_regions = 64;     // the same for pack and unpack (64 tiles of 4 KB: every XCD streams 256 KB runs)
  int64_t plain_divide_sqrt = 1;     // low-precision replay: plain division / square root sequences where in range
  int64_t paired_tiles = 32768;      // FP32 replay, 64 x 1 shape: two 512-byte pieces this many bytes apart per stream and
                                     // wavefront (a power of two); 0: consecutive tiles

  // Accesses per lane of the pack of one slot.  Measured: one 16-byte access per lane is best when the slot's
  // segments are large (117-235 MB: 6.55 vs 6.25 TB/s) or all FP32 state; slots that gather many small
  // compute-weight segments of later operators (5-17 MB each) gain 8% from two (6.35-6.53 vs 5.9-6.0 TB/s).
  int64_t pack_unroll(uint32_t slot) const {
    if (!copy_unroll_auto || persistent) return copy_unroll;
    uint64_t bytes = 0, n = 0;
    for (uint32_t j = 0; j < host.slots[slot].n_segments; ++j) {
      const moev_segment& sg = host.segments[host.slots[slot].first_segment + j];
      if (sg.kind == MOEV_KIND_COMPUTE && sg.nbytes) {
        bytes += sg.nbytes;
        ++n;
      }
    }
    return (n && bytes / n < (64ull << 20)) ? 2 : 1;
  }
  uint64_t eff_copy_tile(uint32_t slot) const {
    return persistent ? copy_tile_bytes : copy_threads * 16 * pack_unroll(slot);
  }
  uint64_t eff_unpack_tile() const { return persistent ? copy_tile_bytes : unpack_threads * 16 * unpack_unroll; }
  uint64_t eff_adam_tile() const { return persistent ? adam_tile_elems : adam_threads * 4 * adam_unroll; }

  // device side
  int device = -1;
  int n_cu = 0;
  bool uploaded = false;
  bool broken = false;
  void* pinned_tables = nullptr;  // staging of the static tables, kept until the plan is freed
  char* d_tables = nullptr;       // one allocation holding every static table
  moev::SegDesc* d_segs = nullptr;
  uint64_t* d_dst_off = nullptr;
  uint32_t* d_seg_tile_start = nullptr;     // per slot: n_segments + 1 entries (pack tiles)
  uint32_t* d_seg_tile_start_unpack = nullptr;  // same for the unpack's tile size
  uint64_t* d_slot_total = nullptr;
  uint64_t* d_numel = nullptr;
  uint32_t* d_op_of_tensor = nullptr;
  uint32_t* d_slot_of_op = nullptr;
  uint32_t* d_tensor_tile_start = nullptr;  // n_tensors + 1
  uint32_t* d_active_tile_start = nullptr;  // n_tensors + 1, rewritten by every replay step
  moev::ScanJob* d_jobs = nullptr;
  uint32_t* d_status = nullptr;
  void** d_state_ptrs = nullptr;            // [4 * n_tensors]
  void** d_grad_ptrs = nullptr;             // [n_tensors]
  std::vector<void*> state_cache, grad_cache;
  bool state_valid = false, grad_valid = false;
  StageSlot ring[kRing];
  int ring_next = 0;
  hipEvent_t tables_uploaded = nullptr;     // recorded after the copy out of pinned_tables
  // Cross-stream ordering of the device tables: each table is written on the stream of the call that
  // (re)builds it; a later call on another stream waits for that write before its kernel reads the table.
  struct Written {
    hipEvent_t event = nullptr;
    hipStream_t stream = nullptr;
    bool recorded = false;
  } scan_done, state_written, grads_written;
  std::vector<uint32_t> slot_tiles, slot_tiles_unpack;  // host-side tile counts (grid sizing only)
  std::vector<uint32_t> slot_first_compute_tile;        // unpack tiles in front of the first compute segment
  uint64_t* d_src_off = nullptr;            // [window][3][n_tensors] snapshot offsets of master, m, v (~0: absent)
  uint32_t tensor_tiles = 0;

  ~moev_plan() {
    if (device >= 0) {
      int cur = -1;
      if (hipGetDevice(&cur) == hipSuccess && cur != device) (void)hipSetDevice(device);
      for (auto& r : ring) {
        if (r.done) {
          (void)hipEventSynchronize(r.done);
          (void)hipEventDestroy(r.done);
        }
        if (r.pinned) (void)hipHostFree(r.pinned);
      }
      if (tables_uploaded) {
        (void)hipEventSynchronize(tables_uploaded);
        (void)hipEventDestroy(tables_uploaded);
      }
      for (Written* w : {&scan_done, &state_written, &grads_written})
        if (w->event) (void)hipEventDestroy(w->event);
      if (d_tables) (void)hipFree(d_tables);
      if (d_state_ptrs) (void)hipFree(d_state_ptrs);
      if (d_grad_ptrs) (void)hipFree(d_grad_ptrs);
      if (pinned_tables) (void)hipHostFree(pinned_tables);
      if (cur >= 0 && cur != device) (void)hipSetDevice(cur);
    }
  }
};

namespace {

using moev::round_up;

bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

uint32_t tiles_of(uint64_t padded, uint64_t tile) { return static_cast<uint32_t>((padded + tile - 1) / tile); }

void compute_host_tiles(moev_plan* pl) {
  const auto& h = pl->host;
  pl->slot_tiles.assign(h.window, 0);
  pl->slot_tiles_unpack.assign(h.window, 0);
  pl->slot_first_compute_tile.assign(h.window, 0);
  for (uint32_t k = 0; k < h.window; ++k) {
    uint64_t n = 0, nu = 0, nu_fp32 = 0;
    for (uint32_t j = 0; j < h.slots[k].n_segments; ++j) {
      const moev_segment& sg = h.segments[h.slots[k].first_segment + j];
      const uint64_t padded = round_up(sg.nbytes, h.align);
      n += tiles_of(padded, pl->eff_copy_tile(k));
      nu += tiles_of(padded, pl->eff_unpack_tile());
      if (sg.kind != MOEV_KIND_COMPUTE) nu_fp32 = nu;  // full-state segments come first in a slot
    }
    pl->slot_tiles[k] = static_cast<uint32_t>(n);
    pl->slot_tiles_unpack[k] = static_cast<uint32_t>(nu);
    pl->slot_first_compute_tile[k] = static_cast<uint32_t>(nu_fp32);
  }
  uint64_t n = 0;
  for (const auto& t : h.tensors) n += tiles_of(t.numel, pl->eff_adam_tile());
  pl->tensor_tiles = static_cast<uint32_t>(n);
}

// First use on the GPU: allocates the device tables and fills their pinned mirror.
int allocate_device_side(moev_plan* pl, int dev, hipStream_t s) {
  const auto& h = pl->host;
  hipDeviceProp_t prop;
  MOEV_HIP(hipGetDeviceProperties(&prop, dev));
  pl->n_cu = prop.multiProcessorCount;
  const size_t n_seg = h.segments.size();
  // carve one device allocation (and a pinned mirror for the inputs) into the tables
  size_t off = 0;
  auto carve = [&](size_t bytes) {
    size_t at = off;
    off = (off + bytes + 255) & ~size_t(255);
    return at;
  };
  const size_t o_segs = carve(n_seg * sizeof(moev::SegDesc));
  const size_t o_numel = carve(h.n_tensors * sizeof(uint64_t));
  const size_t o_opt = carve(h.n_tensors * sizeof(uint32_t));
  const size_t o_slot = carve(h.n_ops * sizeof(uint32_t));
  const size_t o_src = carve(3ull * h.window * h.n_tensors * sizeof(uint64_t));
  const size_t o_jobs = carve((2 * h.window + 1) * sizeof(moev::ScanJob));
  const size_t input_bytes = off;
  const size_t o_dst = carve(n_seg * sizeof(uint64_t));
  const size_t o_tile = carve((n_seg + h.window) * sizeof(uint32_t));
  const size_t o_utile = carve((n_seg + h.window) * sizeof(uint32_t));
  const size_t o_total = carve(h.window * sizeof(uint64_t));
  const size_t o_ttile = carve((h.n_tensors + 1) * sizeof(uint32_t));
  const size_t o_atile = carve((h.n_tensors + 1) * sizeof(uint32_t));
  const size_t o_status = carve(sizeof(uint32_t));
  pl->device = dev;  // from here on the destructor releases whatever was allocated
  MOEV_HIP(hipMalloc(reinterpret_cast<void**>(&pl->d_tables), off));
  MOEV_HIP(hipHostMalloc(&pl->pinned_tables, input_bytes, hipHostMallocDefault));
  MOEV_HIP(hipMalloc(reinterpret_cast<void**>(&pl->d_state_ptrs), 4ull * h.n_tensors * sizeof(void*)));
  MOEV_HIP(hipMalloc(reinterpret_cast<void**>(&pl->d_grad_ptrs), 1ull * h.n_tensors * sizeof(void*)));
  for (auto& r : pl->ring) {
    MOEV_HIP(hipHostMalloc(&r.pinned, 4ull * h.n_tensors * sizeof(void*), hipHostMallocDefault));
    MOEV_HIP(hipEventCreateWithFlags(&r.done, hipEventDisableTiming));
  }
  MOEV_HIP(hipEventCreateWithFlags(&pl->tables_uploaded, hipEventDisableTiming));
  for (moev_plan::Written* w : {&pl->scan_done, &pl->state_written, &pl->grads_written})
    MOEV_HIP(hipEventCreateWithFlags(&w->event, hipEventDisableTiming));
  char* d = pl->d_tables;
  pl->d_segs = reinterpret_cast<moev::SegDesc*>(d + o_segs);
  pl->d_numel = reinterpret_cast<uint64_t*>(d + o_numel);
  pl->d_op_of_tensor = reinterpret_cast<uint32_t*>(d + o_opt);
  pl->d_slot_of_op = reinterpret_cast<uint32_t*>(d + o_slot);
  pl->d_jobs = reinterpret_cast<moev::ScanJob*>(d + o_jobs);
  pl->d_src_off = reinterpret_cast<uint64_t*>(d + o_src);
  pl->d_dst_off = reinterpret_cast<uint64_t*>(d + o_dst);
  pl->d_seg_tile_start = reinterpret_cast<uint32_t*>(d + o_tile);
  pl->d_seg_tile_start_unpack = reinterpret_cast<uint32_t*>(d + o_utile);
  pl->d_slot_total = reinterpret_cast<uint64_t*>(d + o_total);
  pl->d_tensor_tile_start = reinterpret_cast<uint32_t*>(d + o_ttile);
  pl->d_active_tile_start = reinterpret_cast<uint32_t*>(d + o_atile);
  pl->d_status = reinterpret_cast<uint32_t*>(d + o_status);

  char* m = static_cast<char*>(pl->pinned_tables);
  std::memset(m, 0, input_bytes);
  auto* segs = reinterpret_cast<moev::SegDesc*>(m + o_segs);
  for (size_t j = 0; j < n_seg; ++j) segs[j] = moev::SegDesc{h.segments[j].tensor, h.segments[j].kind, h.segments[j].nbytes};
  auto* numel = reinterpret_cast<uint64_t*>(m + o_numel);
  auto* opt = reinterpret_cast<uint32_t*>(m + o_opt);
  for (uint32_t t = 0; t < h.n_tensors; ++t) {
    numel[t] = h.tensors[t].numel;
    opt[t] = h.tensors[t].op;
  }
  std::memcpy(m + o_slot, h.slot_of_op.data(), h.n_ops * sizeof(uint32_t));
  auto* src_off = reinterpret_cast<uint64_t*>(m + o_src);
  std::fill(src_off, src_off + 3ull * h.window * h.n_tensors, ~0ull);
  for (uint32_t k = 0; k < h.window; ++k)
    for (uint32_t j = 0; j < h.slots[k].n_segments; ++j) {
      const moev_segment& sg = h.segments[h.slots[k].first_segment + j];
      if (sg.kind != MOEV_KIND_COMPUTE)
        src_off[(3ull * k + sg.kind) * h.n_tensors + sg.tensor] = sg.dst_off;
    }
  MOEV_HIP(hipMemsetAsync(pl->d_status, 0, sizeof(uint32_t), s));
  return MOEV_OK;
}

// Table uploads allocate, copy out of reused pinned staging and wait on events: none of that may be
// recorded into a HIP graph.  Calls whose tables are already resident enqueue kernels only.
int refuse_under_capture(hipStream_t s, const char* what) {
  hipStreamCaptureStatus status = hipStreamCaptureStatusNone;
  MOEV_HIP(hipStreamIsCapturing(s, &status));
  if (status != hipStreamCaptureStatusNone)
    return fail(MOEV_E_INVAL, "%s while the stream is being captured into a graph: make one call with the same plan "
                "settings and the same state / gradient pointers before the capture", what);
  return MOEV_OK;
}

// Uploads the static tables and runs the on-device layout scan.  Caller holds pl->mu.
int upload_locked(moev_plan* pl, hipStream_t s) {
  const auto& h = pl->host;
  if (pl->broken) return fail(MOEV_E_HIP, "the plan's device side could not be set up earlier; create a new plan");
  int dev = -1;
  MOEV_HIP(hipGetDevice(&dev));
  if (pl->device >= 0 && pl->device != dev)
    return fail(MOEV_E_INVAL, "plan lives on device %d but device %d is current", pl->device, dev);
  if (pl->uploaded) return MOEV_OK;
  {
    int rc = refuse_under_capture(s, "the plan's device tables would have to be built");
    if (rc != MOEV_OK) return rc;
  }

  if (pl->device < 0) {
    int rc = allocate_device_side(pl, dev, s);
    if (rc != MOEV_OK) {
      pl->broken = true;
      return rc;
    }
  }
  {
    // set-up is also where this device's scratch array (convert_replay_static) gets its address resolved
    uint32_t* unused = nullptr;
    int rc = scratch_of_current_device(&unused);
    if (rc != MOEV_OK) return rc;
  }

  // (re)build the scan jobs: they depend on the tile sizes, which moev_tune() may change.  An earlier
  // upload may still be reading the pinned mirror: wait for it before rewriting the jobs.
  MOEV_HIP(hipEventSynchronize(pl->tables_uploaded));
  const size_t jobs_at = reinterpret_cast<char*>(pl->d_jobs) - pl->d_tables;
  auto* jobs = reinterpret_cast<moev::ScanJob*>(static_cast<char*>(pl->pinned_tables) + jobs_at);
  for (uint32_t k = 0; k < h.window; ++k) {
    const uint32_t first = h.slots[k].first_segment;
    jobs[k] = moev::ScanJob{&pl->d_segs[first].nbytes,
                            pl->d_dst_off + first,
                            pl->d_seg_tile_start + first + k,
                            pl->d_slot_total + k,
                            round_up(MOEV_HEADER_BYTES, h.align),
                            h.align,
                            pl->eff_copy_tile(k),
                            h.slots[k].n_segments,
                            static_cast<uint32_t>(sizeof(moev::SegDesc) / sizeof(uint64_t))};
  }
  // the unpack may use another tile size: same offsets (not written again), its own tile map
  for (uint32_t k = 0; k < h.window; ++k) {
    jobs[h.window + k] = jobs[k];
    jobs[h.window + k].prefix_out = nullptr;
    jobs[h.window + k].total_out = nullptr;
    jobs[h.window + k].tile_start_out = pl->d_seg_tile_start_unpack + h.slots[k].first_segment + k;
    jobs[h.window + k].tile = pl->eff_unpack_tile();
  }
  jobs[2 * h.window] = moev::ScanJob{pl->d_numel, nullptr, pl->d_tensor_tile_start, nullptr, 0, 1,
                                     pl->eff_adam_tile(), h.n_tensors, 1};
  const size_t input_bytes = jobs_at + (2 * h.window + 1) * sizeof(moev::ScanJob);
  MOEV_HIP(hipMemcpyAsync(pl->d_tables, pl->pinned_tables, input_bytes, hipMemcpyHostToDevice, s));
  MOEV_HIP(hipEventRecord(pl->tables_uploaded, s));
  MOEV_HIP(moev::launch_layout_scan(pl->d_jobs, 2 * h.window + 1, s));
  MOEV_HIP(hipEventRecord(pl->scan_done.event, s));
  pl->scan_done.stream = s;
  pl->scan_done.recorded = true;
  compute_host_tiles(pl);
  pl->uploaded = true;
  return MOEV_OK;
}

// Orders stream `s` after the writes of the device tables that happened on other streams.
int wait_for_tables(moev_plan* pl, hipStream_t s) {
  for (moev_plan::Written* w : {&pl->scan_done, &pl->state_written, &pl->grads_written}) {
    if (!w->recorded || w->stream == s) continue;
    if (hipEventQuery(w->event) == hipSuccess) {  // long finished: nothing to order, now or later
      w->recorded = false;
      continue;
    }
    MOEV_HIP(hipStreamWaitEvent(s, w->event, 0));
  }
  return MOEV_OK;
}

// Makes the device copy of a pointer table current.  Unchanged tables cost one memcmp.
int sync_ptr_table(moev_plan* pl, std::vector<void*>& cache, bool& valid, void** d_table,
                   const std::vector<void*>& wanted, hipStream_t s, moev_plan::Written& written) {
  if (valid && cache == wanted) return MOEV_OK;
  {
    int rc = refuse_under_capture(s, "a table of state or gradient pointers would have to be uploaded");
    if (rc != MOEV_OK) return rc;
  }
  StageSlot& slot = pl->ring[pl->ring_next];
  pl->ring_next = (pl->ring_next + 1) % kRing;
  if (slot.in_flight) MOEV_HIP(hipEventSynchronize(slot.done));
  std::memcpy(slot.pinned, wanted.data(), wanted.size() * sizeof(void*));
  MOEV_HIP(hipMemcpyAsync(d_table, slot.pinned, wanted.size() * sizeof(void*), hipMemcpyHostToDevice, s));
  MOEV_HIP(hipEventRecord(slot.done, s));
  slot.in_flight = true;
  MOEV_HIP(hipEventRecord(written.event, s));
  written.stream = s;
  written.recorded = true;
  cache = wanted;
  valid = true;
  return MOEV_OK;
}

int check_state(const moev_plan* pl, const moev_state* st, const char* who) {
  if (!st || !st->master || !st->m || !st->v || !st->compute)
    return fail(MOEV_E_INVAL, "%s: state and its four pointer arrays must be non-null", who);
  (void)pl;
  return MOEV_OK;
}

int bind_state(moev_plan* pl, const moev_state* st, hipStream_t s) {
  const uint32_t n = pl->host.n_tensors;
  std::vector<void*> wanted(4ull * n);
  for (uint32_t t = 0; t < n; ++t) {
    wanted[t] = st->master[t];
    wanted[1ull * n + t] = st->m[t];
    wanted[2ull * n + t] = st->v[t];
    wanted[3ull * n + t] = st->compute[t];
  }
  int rc = sync_ptr_table(pl, pl->state_cache, pl->state_valid, pl->d_state_ptrs, wanted, s, pl->state_written);
  if (rc != MOEV_OK) return rc;
  return wait_for_tables(pl, s);
}

uint32_t grid_for(const moev_plan* pl, uint32_t tiles, int64_t cap) {
  uint64_t limit = cap > 0 ? static_cast<uint64_t>(cap) : 8ull * static_cast<uint64_t>(pl->n_cu > 0 ? pl->n_cu : 256);
  uint64_t g = tiles < limit ? tiles : limit;
  return static_cast<uint32_t>(g ? g : 1);
}

// grid of a one-tile-per-workgroup launch: a multiple of the XCD count (the region mapping hands
// workgroup b the (b / 8)-th tile of XCD b % 8), at least one workgroup
uint32_t direct_grid(uint64_t tiles, int64_t xcd_regions = 1) {
  const uint64_t unit = xcd_regions > 1 ? 8ull * static_cast<uint64_t>(xcd_regions) : 8ull;  // chunked mapping: whole rounds of chunks
  const uint64_t g = (tiles + unit - 1) / unit * unit;
  return static_cast<uint32_t>(g ? g : unit);
}

void fill_header(const moev_plan* pl, uint32_t slot, uint64_t iter, uint64_t out[7]) {
  const auto& h = pl->host;
  out[0] = kMagic;
  out[1] = 1ull | (static_cast<uint64_t>(slot) << 32);
  out[2] = h.hash;
  out[3] = iter;
  out[4] = h.slots[slot].n_segments;
  out[5] = h.slots[slot].packed_bytes - MOEV_HEADER_BYTES;
  out[6] = h.align;
}

moev::CopyArgs copy_args(const moev_plan* pl, uint32_t slot, uint64_t iter, void* d_packed, bool unpack) {
  const auto& h = pl->host;
  const uint32_t first = h.slots[slot].first_segment;
  moev::CopyArgs a{};
  a.segs = pl->d_segs + first;
  a.dst_off = pl->d_dst_off + first;
  a.tile_start = (unpack ? pl->d_seg_tile_start_unpack : pl->d_seg_tile_start) + first + slot;
  a.ptrs = pl->d_state_ptrs;
  a.packed = static_cast<uint8_t*>(d_packed);
  fill_header(pl, slot, iter, a.header);
  a.n_seg = h.slots[slot].n_segments;
  a.n_tensors = h.n_tensors;
  a.tile_bytes = static_cast<uint32_t>(unpack ? pl->eff_unpack_tile() : pl->eff_copy_tile(slot));
  a.align = h.align;
  a.lds_entries = (pl->persistent && a.n_seg + 1 <= moev::kMaxLdsEntries) ? a.n_seg + 1 : 0;
  a.slot = slot;
  a.n_ops = h.n_ops;
  a.slot_of_op = pl->d_slot_of_op;
  a.status = pl->d_status;
  a.xcd_regions = static_cast<uint32_t>(pl->copy_xcd_regions);
  return a;
}

// every pointer the slot's segments touch must be present and 16-byte aligned
int check_slot_pointers(const moev_plan* pl, uint32_t slot, const moev_state* st, bool need_compute_of_active,
                        const char* who) {
  const auto& h = pl->host;
  void* const* table[4] = {st->master, st->m, st->v, st->compute};
  for (uint32_t j = 0; j < h.slots[slot].n_segments; ++j) {
    const moev_segment& sg = h.segments[h.slots[slot].first_segment + j];
    const void* p = table[sg.kind][sg.tensor];
    if (sg.nbytes == 0) continue;  // an empty tensor is never dereferenced
    if (!p || !aligned16(p))
      return fail(MOEV_E_INVAL, "%s: tensor %u kind %u pointer is null or not 16-byte aligned", who, sg.tensor, sg.kind);
    if (need_compute_of_active && sg.kind == MOEV_KIND_MASTER) {
      const void* c = st->compute[sg.tensor];
      if (!c || !aligned16(c))
        return fail(MOEV_E_INVAL, "%s: compute pointer of tensor %u is null or not 16-byte aligned", who, sg.tensor);
    }
  }
  return MOEV_OK;
}

// FP32 master weights and moments, bfloat16 compute weights: the regime of the specialised kernels
bool fp32_regime(const moev::HostPlan& h) {
  return h.fmt[MOEV_KIND_MASTER] == MOEV_FMT_F32 && h.fmt[MOEV_KIND_ADAM_M] == MOEV_FMT_F32 &&
         h.fmt[MOEV_KIND_ADAM_V] == MOEV_FMT_F32 && h.fmt[MOEV_KIND_COMPUTE] == MOEV_FMT_BF16;
}
// paired tiles apply to the default one-tile-per-workgroup shape only (master weights of 1, 2 or 4 bytes)
bool replay_paired(const moev_plan* p) {
  return p->paired_tiles && !p->persistent && p->adam_threads == 64 && p->adam_unroll == 1 && p->host.width[MOEV_KIND_MASTER] <= 4;
}
uint32_t master_wlog2(const moev_plan* p) {
  const uint32_t w = p->host.width[MOEV_KIND_MASTER];
  return w >= 4 ? 2u : w == 2 ? 1u : 0u;
}

// log2 of the piece distance in elements (the kernels' parameter; the knob is the distance in bytes of an FP32 stream, which
// the gradients always are), 0 when the replay is not paired
uint32_t pair_log2(const moev_plan* p) {
  return replay_paired(p) ? static_cast<uint32_t>(__builtin_ctzll(static_cast<uint64_t>(p->paired_tiles))) - 2u : 0u;
}
// tiles of one tensor under the paired shape; `master` locates the tensor inside its address block of 2^(L+1) elements
// of 2^wlog2 bytes
uint64_t paired_tiles_of(uint64_t numel, const void* master, uint32_t L, uint32_t wlog2) {
  if (numel == 0) return 0;
  const uint64_t shift = (reinterpret_cast<uintptr_t>(master) & (((2ull << L) << wlog2) - 1)) >> wlog2;
  return ((numel + shift + (2ull << L) - 1) >> (L + 1)) << (L - 7);
}
// ... when the pointer is not known to the host: the largest shift a 16-byte aligned pointer can have
uint64_t paired_tiles_bound(uint64_t numel, uint32_t L) {
  return numel ? ((numel + ((2ull << L) - 4) + (2ull << L) - 1) >> (L + 1)) << (L - 7) : 0;
}

// restore_unpack re-derives the compute weights of newly active operators in this case only; in the
// other regimes the replay step that follows the load writes them
bool derives_compute(const moev::HostPlan& h) {
  return h.fmt[MOEV_KIND_MASTER] == MOEV_FMT_F32 && h.fmt[MOEV_KIND_COMPUTE] == MOEV_FMT_BF16;
}

int check_unpack_args(moev_plan* p, uint32_t slot, const void* h_pinned, void* d_packed, const moev_state* state,
                      const char* who) {
  if (!p || !d_packed) return fail(MOEV_E_INVAL, "%s: null argument", who);
  if (slot >= p->host.window) return fail(MOEV_E_RANGE, "%s: slot %u outside window %u", who, slot, p->host.window);
  if (reinterpret_cast<uintptr_t>(d_packed) & 255u) return fail(MOEV_E_INVAL, "%s: d_packed must be 256-byte aligned", who);
  int rc = check_state(p, state, who);
  if (rc != MOEV_OK) return rc;
  const auto& h = p->host;
  const bool derive = derives_compute(h);
  rc = check_slot_pointers(p, slot, state, derive, who);
  if (rc != MOEV_OK) return rc;
  if (h_pinned) {
    rc = snapshot_peek(p, slot, h_pinned, nullptr);
    if (rc != MOEV_OK) return rc;
  }
  return MOEV_OK;
}

// (optional H2D copy and) the scatter kernel.  compute_only: scatter just the compute-weight segments
// (the tail of the slot's segment list); the FP32 segments are consumed in place by the fused replay.
int launch_unpack_locked(moev_plan* p, uint32_t slot, const void* h_pinned, void* d_packed, const moev_state* state,
                         uint8_t* d_active_mask, hipStream_t s, bool compute_only) {
  const auto& h = p->host;
  int rc = upload_locked(p, s);
  if (rc != MOEV_OK) return rc;
  rc = bind_state(p, state, s);
  if (rc != MOEV_OK) return rc;
  if (h_pinned)
    MOEV_HIP(hipMemcpyAsync(d_packed, h_pinned, h.slots[slot].packed_bytes, hipMemcpyHostToDevice, s));
  moev::CopyArgs a = copy_args(p, slot, 0, d_packed, true);
  a.mask = d_active_mask;
  a.derive_compute = derives_compute(h) ? 1u : 0u;
  if (p->persistent) {
    MOEV_HIP(moev::launch_unpack_persistent(a, grid_for(p, p->slot_tiles_unpack[slot], p->copy_max_blocks), p->nontemporal != 0, s));
  } else {
    a.tile_begin = compute_only ? p->slot_first_compute_tile[slot] : 0u;
    const uint32_t tiles = p->slot_tiles_unpack[slot] - a.tile_begin;
    MOEV_HIP(moev::launch_unpack_direct(a, direct_grid(tiles, p->copy_xcd_regions), static_cast<uint32_t>(p->unpack_threads),
                                        static_cast<uint32_t>(p->unpack_unroll), p->nontemporal != 0, s));
  }
  return MOEV_OK;
}

int check_replay_args(moev_plan* p, const moev_adam* adam, const uint8_t* d_active_mask, void* const* grads,
                      const moev_state* state, const char* who) {
  if (!p || !adam || !d_active_mask || !grads) return fail(MOEV_E_INVAL, "%s: null argument", who);
  const auto& h = p->host;
  if (!fp32_regime(h)) {
    if (!moev::lp_formats_supported(h.fmt))
      return fail(MOEV_E_INVAL, "%s: no replay kernel for storage formats %u, %u, %u, %u (master, m, v, compute)", who,
                  h.fmt[0], h.fmt[1], h.fmt[2], h.fmt[3]);
    if (!p->persistent && !moev::lp_shape_supported(static_cast<uint32_t>(p->adam_threads), static_cast<uint32_t>(p->adam_unroll)))
      return fail(MOEV_E_INVAL, "%s: the low-precision replay runs with 64, 128 or 256 threads and unroll 1 or 2", who);
    if (adam->d_scales && (reinterpret_cast<uintptr_t>(adam->d_scales) & 3u))
      return fail(MOEV_E_INVAL, "%s: d_scales is not 4-byte aligned", who);
  }
  if (adam->step == 0) return fail(MOEV_E_INVAL, "%s: step counts from 1", who);
  int rc = check_state(p, state, who);
  if (rc != MOEV_OK) return rc;
  void* const* table[4] = {state->master, state->m, state->v, state->compute};
  for (uint32_t t = 0; t < h.n_tensors; ++t) {
    if (h.tensors[t].numel == 0) continue;  // an empty tensor is never dereferenced
    for (int k = 0; k < 4; ++k)
      if (!table[k][t] || !aligned16(table[k][t]))
        return fail(MOEV_E_INVAL, "%s: tensor %u kind %d pointer is null or not 16-byte aligned", who, t, k);
    if (!aligned16(grads[t])) return fail(MOEV_E_INVAL, "%s: gradient %u is not 16-byte aligned", who, t);
  }
  return MOEV_OK;
}

// bias correction 1 - beta^step: in double, rounded to FP32 once
float bias_correction(float beta, uint64_t step) {
  return static_cast<float>(1.0 - std::pow(static_cast<double>(beta), static_cast<double>(step)));
}

// Argument block of one replay step, everything but the tables of state / gradient pointers and the tile list.
moev::AdamArgs adam_args(const moev_plan* p, const moev_adam* adam, const uint8_t* d_active_mask) {
  const auto& h = p->host;
  moev::AdamArgs a{};
  a.tile_start = p->d_tensor_tile_start;
  a.numel = p->d_numel;
  a.op_of_tensor = p->d_op_of_tensor;
  a.mask = d_active_mask;
  a.status = p->d_status;
  a.xcd_regions = static_cast<uint32_t>(p->xcd_regions);
  a.n_tensors = h.n_tensors;
  a.tile_elems = static_cast<uint32_t>(p->eff_adam_tile());
  a.paired = pair_log2(p);
  a.master_wlog2 = master_wlog2(p);
  a.lds_entries = (p->persistent && h.n_tensors + 1 <= moev::kMaxLdsEntries) ? h.n_tensors + 1 : 0;
  a.lr = adam->lr;
  a.beta1 = adam->beta1;
  a.beta2 = adam->beta2;
  a.eps = adam->eps;
  a.one_minus_beta1 = 1.0f - adam->beta1;
  a.one_minus_beta2 = 1.0f - adam->beta2;
  a.bc1 = bias_correction(adam->beta1, adam->step);
  a.bc2 = bias_correction(adam->beta2, adam->step);
  a.decay = adam->lr * adam->weight_decay;
  a.has_decay = adam->weight_decay != 0.0f ? 1u : 0u;
  // the plain division / square-root sequences hold for moments in [2^-60, 2^40) if the other operands are ordinary too
  const bool ordinary = a.bc1 >= 0x1p-20f && a.bc1 <= 1.0f && a.bc2 >= 0x1p-20f && a.bc2 <= 1.0f && a.eps >= 0.0f &&
                        a.eps <= 0x1p20f;
  a.plain_divide_sqrt = (p->plain_divide_sqrt && ordinary) ? 1u : 0u;
  return a;
}

// The two kernels of a one-tile-per-workgroup replay step: the device compacts the tile list to the tensors
// that are active (mask) and have gradients into d_active_tile_start ([n_tensors + 1], scratch of the step),
// then the Adam kernel runs over that list with a grid of `bound` workgroups (the host's upper bound on the
// number of tiles; surplus workgroups exit after one scalar load).
// fused_slot >= 0: the FP32 state of the tensors that slot activates is read from d_packed.
int launch_replay_direct(const moev_plan* p, moev::AdamArgs a, const moev_adam* adam, uint32_t* d_active_tile_start,
                         uint64_t bound, int fused_slot, const void* d_packed, hipStream_t s) {
  const auto& h = p->host;
  const bool low_precision = !fp32_regime(h);
  // (state in other formats than FP32 / FP32 / FP32 / BF16 has the one-tile-per-workgroup shape only)
  uint32_t threads = static_cast<uint32_t>(p->adam_threads), unroll = static_cast<uint32_t>(p->adam_unroll);
  if (p->persistent) {
    threads = 256;
    unroll = 1;
    a.lds_entries = 0;
  }
  MOEV_HIP(moev::launch_active_scan(a, d_active_tile_start, s));
  a.tile_start = d_active_tile_start;
  if (fused_slot >= 0) {
    a.src_off = p->d_src_off + 3ull * h.n_tensors * static_cast<uint32_t>(fused_slot);
    a.packed = static_cast<const uint8_t*>(d_packed);
    fill_header(p, static_cast<uint32_t>(fused_slot), 0, a.header);
    MOEV_HIP(moev::launch_adam_fused(a, static_cast<uint32_t>(bound), static_cast<uint32_t>(p->adam_threads),
                                     static_cast<uint32_t>(p->adam_unroll), p->nontemporal != 0, s));
  } else if (low_precision) {
    a.scales = adam->d_scales;
    for (int k = 0; k < 4; ++k) a.fmt[k] = h.fmt[k];
    MOEV_HIP(moev::launch_adam_lp(a, static_cast<uint32_t>(bound), threads, unroll, p->nontemporal != 0, s));
  } else {
    MOEV_HIP(moev::launch_adam_direct(a, static_cast<uint32_t>(bound), threads, unroll, p->nontemporal != 0, s));
  }
  return MOEV_OK;
}

// fused_slot >= 0: the FP32 state of the tensors that slot activates is read from d_packed
int launch_replay_locked(moev_plan* p, const moev_adam* adam, const uint8_t* d_active_mask, void* const* grads,
                         const moev_state* state, hipStream_t s, int fused_slot, const void* d_packed) {
  const auto& h = p->host;
  int rc = upload_locked(p, s);
  if (rc != MOEV_OK) return rc;
  rc = bind_state(p, state, s);
  if (rc != MOEV_OK) return rc;
  std::vector<void*> g(grads, grads + h.n_tensors);
  rc = sync_ptr_table(p, p->grad_cache, p->grad_valid, p->d_grad_ptrs, g, s, p->grads_written);
  if (rc != MOEV_OK) return rc;
  rc = wait_for_tables(p, s);
  if (rc != MOEV_OK) return rc;

  moev::AdamArgs a = adam_args(p, adam, d_active_mask);
  a.ptrs = p->d_state_ptrs;
  a.grads = p->d_grad_ptrs;
  if (p->persistent && fp32_regime(h)) {
    MOEV_HIP(moev::launch_adam_persistent(a, grid_for(p, p->tensor_tiles, p->adam_max_blocks), p->nontemporal != 0, s));
    return MOEV_OK;
  }
  if (p->persistent) a.tile_elems = 256 * 4;
  // the host only bounds the grid: tensors without a gradient pointer cannot contribute tiles
  uint64_t bound = 0;
  for (uint32_t t = 0; t < h.n_tensors; ++t)
    if (grads[t]) bound += a.paired ? paired_tiles_of(h.tensors[t].numel, state->master[t], a.paired, a.master_wlog2) : tiles_of(h.tensors[t].numel, a.tile_elems);
  if (bound + 8ull * 65536 >= (1ull << 31)) return fail(MOEV_E_RANGE, "replay: too many tiles for one launch");
  return launch_replay_direct(p, a, adam, p->d_active_tile_start, direct_grid(bound, p->xcd_regions), fused_slot, d_packed, s);
}

}  // namespace

// =====================================================================================
extern "C" {

const char* moev_last_error(void) { return g_last_error.c_str(); }

int ckpt_plan(const moev_plan_cfg* cfg, moev_plan** out) {
  if (!cfg || !out) return fail(MOEV_E_INVAL, "ckpt_plan: null argument");
  *out = nullptr;
  moev_plan* pl = new (std::nothrow) moev_plan();
  if (!pl) return fail(MOEV_E_NOMEM, "ckpt_plan: out of host memory");
  std::string err;
  int rc;
  try {
    rc = moev::build_plan(*cfg, pl->host, err);
  } catch (const std::bad_alloc&) {
    delete pl;
    return fail(MOEV_E_NOMEM, "ckpt_plan: out of host memory");
  }
  if (rc != MOEV_OK) {
    delete pl;
    return fail(rc, "%s", err.c_str());
  }
  // tile counts must fit 31 bits at the smallest tile size the knobs allow
  for (const auto& s : pl->host.slots)
    if (s.packed_bytes / 4096 + s.n_segments >= (1ull << 31)) {
      delete pl;
      return fail(MOEV_E_INVAL, "ckpt_plan: slot too large");
    }
  // Replay launch shape for state stored narrower than FP32 (measured on a Mixtral-shaped layer): 128 threads
  // for 6 bytes of master + moments per parameter or fewer, and two accesses per lane at 4 bytes (too few bytes
  // are in flight there with one 16-byte gradient access per lane).
  const auto& h = pl->host;
  const uint32_t state_bytes = h.width[MOEV_KIND_MASTER] + h.width[MOEV_KIND_ADAM_M] + h.width[MOEV_KIND_ADAM_V];
  if (!fp32_regime(h) && state_bytes <= 6) {
    pl->adam_threads = 128;
    pl->adam_unroll = state_bytes <= 4 ? 2 : 1;
  }
  compute_host_tiles(pl);
  *out = pl;
  return MOEV_OK;
}

void ckpt_plan_free(moev_plan* plan) { delete plan; }

int moev_find_window_size(uint32_t n_ops, double t_iter_s, double compute_bytes_per_op, double master_bytes_per_op,
                          double optim_bytes_per_op, double host_link_Bps, uint32_t* window, uint32_t* n_active) {
  int rc = moev::find_window_size(n_ops, t_iter_s, compute_bytes_per_op, master_bytes_per_op, optim_bytes_per_op,
                                  host_link_Bps, window, n_active);
  return rc == MOEV_OK ? rc : fail(rc, "moev_find_window_size: bad argument");
}

int moev_order_operators(uint32_t n_ops, const double* popularity, uint32_t* order) {
  if (!popularity || !order) return fail(MOEV_E_INVAL, "moev_order_operators: null argument");
  for (uint32_t e = 0; e < n_ops; ++e)
    if (std::isnan(popularity[e])) return fail(MOEV_E_INVAL, "moev_order_operators: popularity %u is NaN", e);
  moev::order_operators(n_ops, popularity, order);
  return MOEV_OK;
}

// Sec. 3.5: operators are re-ordered when the activation frequency changed by more than
// rel_change (relative to the old frequency) for at least min_fraction of the operators.
int moev_reorder_needed(uint32_t n_ops, const double* old_freq, const double* new_freq, double rel_change,
                        double min_fraction) {
  if (!old_freq || !new_freq || n_ops == 0) return fail(MOEV_E_INVAL, "moev_reorder_needed: bad argument");
  uint32_t moved = 0;
  for (uint32_t e = 0; e < n_ops; ++e) {
    const double base = std::fabs(old_freq[e]);
    const double delta = std::fabs(new_freq[e] - old_freq[e]);
    if (base > 0 ? delta > rel_change * base : delta > 0) ++moved;
  }
  return static_cast<double>(moved) >= min_fraction * static_cast<double>(n_ops) ? 1 : 0;
}

// App. B: exponential moving average of the per-batch activation counts.
int moev_popularity_time_decayed(uint32_t n_ops, double alpha, const double* previous, const double* batch_count,
                                 double* out) {
  if (!previous || !batch_count || !out || !(alpha >= 0.0 && alpha <= 1.0))
    return fail(MOEV_E_INVAL, "moev_popularity_time_decayed: null pointer or alpha outside [0, 1]");
  const double fresh = 1.0 - alpha;
  for (uint32_t e = 0; e < n_ops; ++e) out[e] = alpha * previous[e] + fresh * batch_count[e];
  return MOEV_OK;
}

// App. B: utilisation relative to capacity.
int moev_popularity_capacity_aware(uint32_t n_ops, const double* popularity, const double* capacity, double* out) {
  if (!popularity || !capacity || !out) return fail(MOEV_E_INVAL, "moev_popularity_capacity_aware: null pointer");
  for (uint32_t e = 0; e < n_ops; ++e)
    if (!(capacity[e] > 0.0)) return fail(MOEV_E_INVAL, "moev_popularity_capacity_aware: capacity %u is not positive", e);
  for (uint32_t e = 0; e < n_ops; ++e) out[e] = popularity[e] / capacity[e];
  return MOEV_OK;
}

// Sec. 2.4: product of the fault-free efficiency and the efficiency under failures.
double moev_ettr(double t_ckpt_s, double t_iter_s, double ckpt_interval_iters, double expected_recovery_s,
                 double mtbf_s) {
  if (!(t_iter_s > 0.0) || !(ckpt_interval_iters > 0.0) || !(mtbf_s > 0.0)) return std::nan("");
  const double useful_fault_free = (t_iter_s * ckpt_interval_iters) / (t_iter_s * ckpt_interval_iters + t_ckpt_s);
  const double useful_under_failures = mtbf_s / (mtbf_s + expected_recovery_s);
  return useful_fault_free * useful_under_failures;
}

// Sec. 3.6
int moev_recovery_time(int sparse, double interval_or_window, double t_iter_s, double* expected_s, double* worst_s) {
  if (!expected_s || !worst_s || !(interval_or_window > 0.0) || !(t_iter_s > 0.0))
    return fail(MOEV_E_INVAL, "moev_recovery_time: bad argument");
  const double span = interval_or_window * t_iter_s;
  *expected_s = sparse ? span + 0.5 * span : 0.5 * span;  // conversion replays W, then on average half a window more
  *worst_s = sparse ? span + span : span;
  return MOEV_OK;
}

int moev_bias_corrections(float beta1, float beta2, uint64_t step, float* bc1, float* bc2) {
  if (!bc1 || !bc2 || step == 0) return fail(MOEV_E_INVAL, "moev_bias_corrections: null pointer or step 0");
  *bc1 = bias_correction(beta1, step);
  *bc2 = bias_correction(beta2, step);
  return MOEV_OK;
}

uint32_t ckpt_plan_window(const moev_plan* p) { return p ? p->host.window : 0; }
uint32_t ckpt_plan_n_ops(const moev_plan* p) { return p ? p->host.n_ops : 0; }
uint32_t ckpt_plan_n_tensors(const moev_plan* p) { return p ? p->host.n_tensors : 0; }
uint32_t ckpt_plan_n_active(const moev_plan* p) { return p ? p->host.n_active : 0; }
uint64_t ckpt_plan_pack_tile_bytes(const moev_plan* p, uint32_t slot) {
  return (p && slot < p->host.window) ? p->eff_copy_tile(slot) : 0;
}
uint32_t ckpt_plan_width(const moev_plan* p, uint32_t kind) { return (p && kind < 4) ? p->host.width[kind] : 0; }
uint32_t ckpt_plan_format(const moev_plan* p, uint32_t kind) { return (p && kind < 4) ? p->host.fmt[kind] : 0; }
uint64_t ckpt_plan_hash(const moev_plan* p) { return p ? p->host.hash : 0; }

int ckpt_plan_slot_of_op(const moev_plan* p, uint32_t* out) {
  if (!p || !out) return fail(MOEV_E_INVAL, "ckpt_plan_slot_of_op: null argument");
  std::memcpy(out, p->host.slot_of_op.data(), p->host.n_ops * sizeof(uint32_t));
  return MOEV_OK;
}

int ckpt_plan_order(const moev_plan* p, uint32_t* out) {
  if (!p || !out) return fail(MOEV_E_INVAL, "ckpt_plan_order: null argument");
  std::memcpy(out, p->host.order.data(), p->host.n_ops * sizeof(uint32_t));
  return MOEV_OK;
}

uint64_t ckpt_plan_packed_bytes(const moev_plan* p, uint32_t slot) {
  return (p && slot < p->host.window) ? p->host.slots[slot].packed_bytes : 0;
}

uint64_t ckpt_plan_max_packed_bytes(const moev_plan* p) {
  uint64_t m = 0;
  if (p)
    for (const auto& s : p->host.slots) m = s.packed_bytes > m ? s.packed_bytes : m;
  return m;
}

uint32_t ckpt_plan_n_segments(const moev_plan* p, uint32_t slot) {
  return (p && slot < p->host.window) ? p->host.slots[slot].n_segments : 0;
}

int64_t ckpt_plan_segments(const moev_plan* p, uint32_t slot, moev_segment* out, uint64_t cap) {
  if (!p) return fail(MOEV_E_INVAL, "ckpt_plan_segments: null plan");
  if (slot >= p->host.window) return fail(MOEV_E_RANGE, "ckpt_plan_segments: slot %u outside window %u", slot, p->host.window);
  const auto& s = p->host.slots[slot];
  if (out)
    for (uint32_t j = 0; j < s.n_segments && j < cap; ++j) out[j] = p->host.segments[s.first_segment + j];
  return s.n_segments;
}

uint64_t ckpt_plan_active_params(const moev_plan* p, uint32_t i) {
  if (!p) return 0;
  uint64_t n = 0;
  for (const auto& t : p->host.tensors)
    if (p->host.slot_of_op[t.op] <= i) n += t.numel;
  return n;
}

int moev_tune(moev_plan* p, int knob, int64_t value) {
  if (!p) return fail(MOEV_E_INVAL, "moev_tune: null plan");
  std::lock_guard<std::mutex> lock(p->mu);
  switch (knob) {
    case MOEV_TUNE_COPY_TILE_BYTES:
      if (value < 4096 || value % 4096 || value > (1 << 26)) return fail(MOEV_E_INVAL, "copy tile must be a multiple of 4096 in [4096, 64 MiB]");
      p->copy_tile_bytes = value;
      break;
    case MOEV_TUNE_ADAM_TILE_ELEMS:
      if (value < 1024 || value % 1024 || value > (1 << 24)) return fail(MOEV_E_INVAL, "adam tile must be a multiple of 1024 in [1024, 16 Mi]");
      p->adam_tile_elems = value;
      break;
    case MOEV_TUNE_COPY_MAX_BLOCKS:
      if (value < 0 || value > (1 << 20)) return fail(MOEV_E_INVAL, "block cap out of range");
      p->copy_max_blocks = value;
      break;
    case MOEV_TUNE_ADAM_MAX_BLOCKS:
      if (value < 0 || value > (1 << 20)) return fail(MOEV_E_INVAL, "block cap out of range");
      p->adam_max_blocks = value;
      break;
    case MOEV_TUNE_NONTEMPORAL:
      p->nontemporal = value ? 1 : 0;
      break;
    case MOEV_TUNE_PERSISTENT:
      p->persistent = value ? 1 : 0;
      break;
    case MOEV_TUNE_XCD_REGIONS:
    case MOEV_TUNE_COPY_XCD_REGIONS:
      if (value < 0 || value > 65536 || (value & (value - 1)))
        return fail(MOEV_E_INVAL, "xcd regions: 0 (off), 1 (eighths) or a chunk of 2..65536 tiles, a power of two");
      (knob == MOEV_TUNE_XCD_REGIONS ? p->xcd_regions : p->copy_xcd_regions) = value;
      break;
    case MOEV_TUNE_PLAIN_DIVIDE_SQRT:
      p->plain_divide_sqrt = value ? 1 : 0;
      break;
    case MOEV_TUNE_PAIRED_TILES:
      if (value == 1) value = 32768;
      if (value != 0 && (value < 512 || value > (4 << 20) || (value & (value - 1))))
        return fail(MOEV_E_INVAL, "the piece distance of the paired tiles is 0 (off), 1 (default) or a power of two in [512, 4 MiB]");
      p->paired_tiles = value;
      break;
    case MOEV_TUNE_COPY_THREADS:
      if (!moev::direct_shape_supported(static_cast<uint32_t>(value), static_cast<uint32_t>(p->copy_unroll)))
        return fail(MOEV_E_INVAL, "unsupported (threads, unroll) launch shape");
      p->copy_threads = value;
      p->copy_unroll_auto = false;
      break;
    case MOEV_TUNE_COPY_UNROLL:
      if (!moev::direct_shape_supported(static_cast<uint32_t>(p->copy_threads), static_cast<uint32_t>(value)))
        return fail(MOEV_E_INVAL, "unsupported (threads, unroll) launch shape");
      p->copy_unroll = value;
      p->copy_unroll_auto = false;
      break;
    case MOEV_TUNE_UNPACK_THREADS:
      if (!moev::direct_shape_supported(static_cast<uint32_t>(value), static_cast<uint32_t>(p->unpack_unroll)))
        return fail(MOEV_E_INVAL, "unsupported (threads, unroll) launch shape");
      p->unpack_threads = value;
      break;
    case MOEV_TUNE_UNPACK_UNROLL:
      if (!moev::direct_shape_supported(static_cast<uint32_t>(p->unpack_threads), static_cast<uint32_t>(value)))
        return fail(MOEV_E_INVAL, "unsupported (threads, unroll) launch shape");
      p->unpack_unroll = value;
      break;
    case MOEV_TUNE_ADAM_THREADS:
      if (!moev::direct_shape_supported(static_cast<uint32_t>(value), static_cast<uint32_t>(p->adam_unroll)))
        return fail(MOEV_E_INVAL, "unsupported (threads, unroll) launch shape");
      p->adam_threads = value;
      break;
    case MOEV_TUNE_ADAM_UNROLL:
      if (!moev::direct_shape_supported(static_cast<uint32_t>(p->adam_threads), static_cast<uint32_t>(value)))
        return fail(MOEV_E_INVAL, "unsupported (threads, unroll) launch shape");
      p->adam_unroll = value;
      break;
    default:
      return fail(MOEV_E_INVAL, "moev_tune: unknown knob %d", knob);
  }
  p->uploaded = false;  // the tile tables are rebuilt by the next GPU call
  compute_host_tiles(p);
  return MOEV_OK;
}

int64_t moev_tune_get(const moev_plan* p, int knob) {
  if (!p) return -1;
  switch (knob) {
    case MOEV_TUNE_COPY_TILE_BYTES: return p->copy_tile_bytes;
    case MOEV_TUNE_COPY_MAX_BLOCKS: return p->copy_max_blocks;
    case MOEV_TUNE_ADAM_TILE_ELEMS: return p->adam_tile_elems;
    case MOEV_TUNE_ADAM_MAX_BLOCKS: return p->adam_max_blocks;
    case MOEV_TUNE_NONTEMPORAL: return p->nontemporal;
    case MOEV_TUNE_PERSISTENT: return p->persistent;
    case MOEV_TUNE_XCD_REGIONS: return p->xcd_regions;
    case MOEV_TUNE_COPY_XCD_REGIONS: return p->copy_xcd_regions;
    case MOEV_TUNE_PLAIN_DIVIDE_SQRT: return p->plain_divide_sqrt;
    case MOEV_TUNE_PAIRED_TILES: return p->paired_tiles;
    case MOEV_TUNE_COPY_THREADS: return p->copy_threads;
    case MOEV_TUNE_COPY_UNROLL: return p->copy_unroll_auto ? 0 : p->copy_unroll;
    case MOEV_TUNE_UNPACK_THREADS: return p->unpack_threads;
    case MOEV_TUNE_UNPACK_UNROLL: return p->unpack_unroll;
    case MOEV_TUNE_ADAM_THREADS: return p->adam_threads;
    case MOEV_TUNE_ADAM_UNROLL: return p->adam_unroll;
    default: return -1;
  }
}

int ckpt_plan_upload(moev_plan* p, void* stream) {
  if (!p) return fail(MOEV_E_INVAL, "ckpt_plan_upload: null plan");
  std::lock_guard<std::mutex> lock(p->mu);
  return upload_locked(p, static_cast<hipStream_t>(stream));
}

int ckpt_plan_device_layout(moev_plan* p, uint32_t slot, uint64_t* dst_off_out, uint32_t* tile_start_out,
                            uint64_t* packed_bytes_out, void* stream) {
  if (!p) return fail(MOEV_E_INVAL, "ckpt_plan_device_layout: null plan");
  if (slot >= p->host.window) return fail(MOEV_E_RANGE, "ckpt_plan_device_layout: slot outside window");
  std::lock_guard<std::mutex> lock(p->mu);
  hipStream_t s = static_cast<hipStream_t>(stream);
  int rc = upload_locked(p, s);
  if (rc != MOEV_OK) return rc;
  rc = wait_for_tables(p, s);
  if (rc != MOEV_OK) return rc;
  const auto& sl = p->host.slots[slot];
  if (dst_off_out && sl.n_segments)
    MOEV_HIP(hipMemcpyAsync(dst_off_out, p->d_dst_off + sl.first_segment, sl.n_segments * sizeof(uint64_t),
                            hipMemcpyDeviceToHost, s));
  if (tile_start_out)
    MOEV_HIP(hipMemcpyAsync(tile_start_out, p->d_seg_tile_start + sl.first_segment + slot,
                            (sl.n_segments + 1) * sizeof(uint32_t), hipMemcpyDeviceToHost, s));
  if (packed_bytes_out)
    MOEV_HIP(hipMemcpyAsync(packed_bytes_out, p->d_slot_total + slot, sizeof(uint64_t), hipMemcpyDeviceToHost, s));
  MOEV_HIP(hipStreamSynchronize(s));
  return MOEV_OK;
}

int ckpt_plan_device_status(moev_plan* p, void* stream) {
  if (!p) return fail(MOEV_E_INVAL, "ckpt_plan_device_status: null plan");
  std::lock_guard<std::mutex> lock(p->mu);
  if (!p->uploaded && p->device < 0) return MOEV_OK;
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint32_t status = 0;
  MOEV_HIP(hipMemcpyAsync(&status, p->d_status, sizeof(status), hipMemcpyDeviceToHost, s));
  MOEV_HIP(hipStreamSynchronize(s));
  if (status) {
    MOEV_HIP(hipMemsetAsync(p->d_status, 0, sizeof(uint32_t), s));
    MOEV_HIP(hipStreamSynchronize(s));
    if (status == 2u) return fail(MOEV_E_INVAL, "convert_replay skipped an active operator whose gradient pointer was null");
    return fail(MOEV_E_MISMATCH, "a device-resident snapshot was refused by restore_unpack (foreign header)");
  }
  return MOEV_OK;
}

int moev_arith_selfcheck(int what, float divisor, uint32_t first_bits, uint64_t count, uint64_t seed, uint64_t* mismatches,
                         void* stream) {
  if (what < 0 || what > 2 || !mismatches) return fail(MOEV_E_INVAL, "moev_arith_selfcheck: bad argument");
  if (what != 2 && static_cast<uint64_t>(first_bits) + count > 0x7f800000ull)
    return fail(MOEV_E_RANGE, "moev_arith_selfcheck: the patterns must be finite positive values");
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned long long* d_count = nullptr;
  MOEV_HIP(hipMalloc(reinterpret_cast<void**>(&d_count), sizeof(unsigned long long)));
  unsigned long long host_count = 0;
  hipError_t e = hipMemcpyAsync(d_count, &host_count, sizeof host_count, hipMemcpyHostToDevice, s);
  if (e == hipSuccess) e = moev::launch_arith_check(static_cast<uint32_t>(what), divisor, first_bits, count, seed, d_count, s);
  if (e == hipSuccess) e = hipMemcpyAsync(&host_count, d_count, sizeof host_count, hipMemcpyDeviceToHost, s);
  if (e == hipSuccess) e = hipStreamSynchronize(s);
  (void)hipFree(d_count);
  if (e != hipSuccess) return fail(MOEV_E_HIP, "moev_arith_selfcheck: %s", hipGetErrorString(e));
  *mismatches = host_count;
  return MOEV_OK;
}

int moev_copy_probe(void* d_dst, const void* d_src, size_t nbytes, uint32_t blocks, int nontemporal, void* stream) {
  // blocks == 0: one 4 KB tile per workgroup (the default gather shape); otherwise a fixed grid, 32 KB per step
  if (!d_dst || !d_src || nbytes == 0 || (nbytes & 15u)) return fail(MOEV_E_INVAL, "moev_copy_probe: null pointer or size not a multiple of 16");
  if (!aligned16(d_dst) || !aligned16(d_src)) return fail(MOEV_E_INVAL, "moev_copy_probe: pointers must be 16-byte aligned");
  uint32_t unroll = 8;
  if (blocks == 0) {
    unroll = 1;
    const uint64_t tiles = (nbytes + 4095) / 4096;
    if (tiles >= (1ull << 31)) return fail(MOEV_E_RANGE, "moev_copy_probe: too large");
    blocks = static_cast<uint32_t>(tiles);
  } else {
    const uint64_t chunks = (nbytes + 32767) / 32768;
    if (blocks > chunks) blocks = static_cast<uint32_t>(chunks);
  }
  MOEV_HIP(moev::launch_copy_probe(d_src, d_dst, nbytes, blocks, unroll, nontemporal != 0, static_cast<hipStream_t>(stream)));
  return MOEV_OK;
}

int moev_stream_probe(int mode, void* d_dst, const void* d_src, size_t nbytes, uint32_t value, int nontemporal, void* stream) {
  if (mode < 1 || mode > 3) return fail(MOEV_E_INVAL, "moev_stream_probe: mode must be 1 (read only), 2 (write only) or 3 (paired copy)");
  if (!d_dst || (mode != 2 && !d_src) || nbytes == 0 || (nbytes & 15u))
    return fail(MOEV_E_INVAL, "moev_stream_probe: null pointer or size not a multiple of 16");
  if (!aligned16(d_dst) || (mode != 2 && !aligned16(d_src))) return fail(MOEV_E_INVAL, "moev_stream_probe: pointers must be 16-byte aligned");
  if (mode == 3) {  // value = distance between the two pieces of a wavefront, a power of two in [512, 2^30]
    if (value < 512 || value > (1u << 30) || (value & (value - 1)))
      return fail(MOEV_E_INVAL, "moev_stream_probe: the piece distance must be a power of two in [512, 2^30]");
    const uint64_t block = 2ull * value;
    if (nbytes % block || reinterpret_cast<uintptr_t>(d_dst) % block || reinterpret_cast<uintptr_t>(d_src) % block)
      return fail(MOEV_E_INVAL, "moev_stream_probe: paired copy needs size and pointers aligned to twice the piece distance");
    value = static_cast<uint32_t>(__builtin_ctz(value));
  }
  if ((nbytes + 4095) / 4096 >= (1ull << 31)) return fail(MOEV_E_RANGE, "moev_stream_probe: too large");
  MOEV_HIP(moev::launch_stream_probe(mode, d_src, d_dst, nbytes, value, nontemporal != 0, static_cast<hipStream_t>(stream)));
  return MOEV_OK;
}

int snapshot_pack(moev_plan* p, uint32_t slot, uint64_t iter, const moev_state* state, void* d_packed, size_t cap,
                  void* stream) {
  if (!p || !d_packed) return fail(MOEV_E_INVAL, "snapshot_pack: null argument");
  if (slot >= p->host.window) return fail(MOEV_E_RANGE, "snapshot_pack: slot %u outside window %u", slot, p->host.window);
  if (cap < p->host.slots[slot].packed_bytes)
    return fail(MOEV_E_RANGE, "snapshot_pack: buffer of %zu bytes, slot needs %llu", cap,
                static_cast<unsigned long long>(p->host.slots[slot].packed_bytes));
  if (reinterpret_cast<uintptr_t>(d_packed) & 255u) return fail(MOEV_E_INVAL, "snapshot_pack: d_packed must be 256-byte aligned");
  int rc = check_state(p, state, "snapshot_pack");
  if (rc != MOEV_OK) return rc;
  rc = check_slot_pointers(p, slot, state, false, "snapshot_pack");
  if (rc != MOEV_OK) return rc;
  std::lock_guard<std::mutex> lock(p->mu);
  hipStream_t s = static_cast<hipStream_t>(stream);
  rc = upload_locked(p, s);
  if (rc != MOEV_OK) return rc;
  rc = bind_state(p, state, s);
  if (rc != MOEV_OK) return rc;
  const moev::CopyArgs a = copy_args(p, slot, iter, d_packed, false);
  if (p->persistent)
    MOEV_HIP(moev::launch_pack_persistent(a, grid_for(p, p->slot_tiles[slot], p->copy_max_blocks), p->nontemporal != 0, s));
  else
    MOEV_HIP(moev::launch_pack_direct(a, direct_grid(p->slot_tiles[slot], p->copy_xcd_regions), static_cast<uint32_t>(p->copy_threads),
                                      static_cast<uint32_t>(p->pack_unroll(slot)), p->nontemporal != 0, s));
  return MOEV_OK;
}

int snapshot_drain(moev_plan* p, uint32_t slot, const void* d_packed, void* h_pinned, size_t cap, void* side_stream,
                   void* pack_done, void* drained) {
  if (!p || !d_packed || !h_pinned) return fail(MOEV_E_INVAL, "snapshot_drain: null argument");
  if (slot >= p->host.window) return fail(MOEV_E_RANGE, "snapshot_drain: slot %u outside window %u", slot, p->host.window);
  const uint64_t nbytes = p->host.slots[slot].packed_bytes;
  if (cap < nbytes) return fail(MOEV_E_RANGE, "snapshot_drain: host buffer too small");
  hipStream_t s = static_cast<hipStream_t>(side_stream);
  if (pack_done) MOEV_HIP(hipStreamWaitEvent(s, static_cast<hipEvent_t>(pack_done), 0));
  MOEV_HIP(hipMemcpyAsync(h_pinned, d_packed, nbytes, hipMemcpyDeviceToHost, s));
  if (drained) MOEV_HIP(hipEventRecord(static_cast<hipEvent_t>(drained), s));
  return MOEV_OK;
}

int snapshot_drain_range(moev_plan* p, uint32_t slot, const void* d_packed, uint64_t offset, void* h_pinned, size_t nbytes,
                         void* side_stream, void* pack_done, void* drained) {
  if (!p || !d_packed || (!h_pinned && nbytes)) return fail(MOEV_E_INVAL, "snapshot_drain_range: null argument");
  if (slot >= p->host.window)
    return fail(MOEV_E_RANGE, "snapshot_drain_range: slot %u outside window %u", slot, p->host.window);
  const uint64_t total = p->host.slots[slot].packed_bytes;
  if (offset > total || nbytes > total - offset)
    return fail(MOEV_E_RANGE, "snapshot_drain_range: bytes [%llu, %llu) are outside the slot's %llu packed bytes",
                static_cast<unsigned long long>(offset), static_cast<unsigned long long>(offset + nbytes),
                static_cast<unsigned long long>(total));
  hipStream_t s = static_cast<hipStream_t>(side_stream);
  if (pack_done) MOEV_HIP(hipStreamWaitEvent(s, static_cast<hipEvent_t>(pack_done), 0));
  if (nbytes)
    MOEV_HIP(hipMemcpyAsync(h_pinned, static_cast<const uint8_t*>(d_packed) + offset, nbytes, hipMemcpyDeviceToHost, s));
  if (drained) MOEV_HIP(hipEventRecord(static_cast<hipEvent_t>(drained), s));
  return MOEV_OK;
}

int snapshot_peek(const moev_plan* p, uint32_t slot, const void* h_packed, moev_header* out) {
  if (!p || !h_packed) return fail(MOEV_E_INVAL, "snapshot_peek: null argument");
  if (slot >= p->host.window) return fail(MOEV_E_RANGE, "snapshot_peek: slot outside window");
  uint64_t w[7];
  std::memcpy(w, h_packed, sizeof(w));
  moev_header hd;
  hd.magic = w[0];
  hd.version = static_cast<uint32_t>(w[1]);
  hd.slot = static_cast<uint32_t>(w[1] >> 32);
  hd.plan_hash = w[2];
  hd.iter = w[3];
  hd.n_segments = w[4];
  hd.payload_bytes = w[5];
  hd.align = static_cast<uint32_t>(w[6]);
  if (out) *out = hd;
  uint64_t want[7];
  fill_header(p, slot, hd.iter, want);
  if (std::memcmp(w, want, sizeof(w)) != 0)
    return fail(MOEV_E_MISMATCH, "snapshot header does not match plan %016llx slot %u",
                static_cast<unsigned long long>(p->host.hash), slot);
  return MOEV_OK;
}

int restore_unpack(moev_plan* p, uint32_t slot, const void* h_pinned, void* d_packed, const moev_state* state,
                   uint8_t* d_active_mask, void* stream) {
  int rc = check_unpack_args(p, slot, h_pinned, d_packed, state, "restore_unpack");
  if (rc != MOEV_OK) return rc;
  std::lock_guard<std::mutex> lock(p->mu);
  return launch_unpack_locked(p, slot, h_pinned, d_packed, state, d_active_mask, static_cast<hipStream_t>(stream), false);
}

int convert_replay(moev_plan* p, const moev_adam* adam, const uint8_t* d_active_mask, void* const* grads,
                   const moev_state* state, void* stream) {
  int rc = check_replay_args(p, adam, d_active_mask, grads, state, "convert_replay");
  if (rc != MOEV_OK) return rc;
  std::lock_guard<std::mutex> lock(p->mu);
  return launch_replay_locked(p, adam, d_active_mask, grads, state, static_cast<hipStream_t>(stream), -1, nullptr);
}

int convert_replay_static(moev_plan* p, const moev_adam* adam, const uint8_t* d_active_mask, void* const* d_grad_table,
                          void* const* d_state_table, void* stream) {
  if (!p || !adam || !d_active_mask || !d_grad_table || !d_state_table)
    return fail(MOEV_E_INVAL, "convert_replay_static: null argument");
  const auto& h = p->host;
  if (h.n_tensors > MOEV_STATIC_MAX_TENSORS)
    return fail(MOEV_E_RANGE, "convert_replay_static: %u tensors, the static scratch holds the tile list of at most %u",
                h.n_tensors, static_cast<unsigned>(MOEV_STATIC_MAX_TENSORS));
  if ((reinterpret_cast<uintptr_t>(d_grad_table) | reinterpret_cast<uintptr_t>(d_state_table)) & 7u)
    return fail(MOEV_E_INVAL, "convert_replay_static: the pointer tables must be 8-byte aligned");
  if (adam->step == 0) return fail(MOEV_E_INVAL, "convert_replay_static: step counts from 1");
  if (!fp32_regime(h)) {
    if (!moev::lp_formats_supported(h.fmt))
      return fail(MOEV_E_INVAL, "convert_replay_static: no replay kernel for storage formats %u, %u, %u, %u", h.fmt[0],
                  h.fmt[1], h.fmt[2], h.fmt[3]);
    if (!moev::lp_shape_supported(static_cast<uint32_t>(p->adam_threads), static_cast<uint32_t>(p->adam_unroll)))
      return fail(MOEV_E_INVAL, "convert_replay_static: the low-precision replay runs with 64, 128 or 256 threads and unroll 1 or 2");
    if (adam->d_scales && (reinterpret_cast<uintptr_t>(adam->d_scales) & 3u))
      return fail(MOEV_E_INVAL, "convert_replay_static: d_scales is not 4-byte aligned");
  }
  std::lock_guard<std::mutex> lock(p->mu);
  if (p->persistent)
    return fail(MOEV_E_INVAL, "convert_replay_static: one-tile-per-workgroup launch shape only (MOEV_TUNE_PERSISTENT is set)");
  if (!p->uploaded || p->broken)
    return fail(MOEV_E_INVAL, "convert_replay_static: the plan's device tables are not resident; call ckpt_plan_upload "
                "first (this call allocates and uploads nothing)");
  int dev = -1;
  MOEV_HIP(hipGetDevice(&dev));
  if (dev != p->device) return fail(MOEV_E_INVAL, "plan lives on device %d but device %d is current", p->device, dev);
  hipStream_t s = static_cast<hipStream_t>(stream);
  uint32_t* d_scratch = nullptr;
  int rc = scratch_of_current_device(&d_scratch);  // resolved by ckpt_plan_upload already: a table lookup
  if (rc != MOEV_OK) return rc;
  rc = wait_for_tables(p, s);  // the layout scan may have run on another stream
  if (rc != MOEV_OK) return rc;

  moev::AdamArgs a = adam_args(p, adam, d_active_mask);
  a.ptrs = d_state_table;
  a.grads = d_grad_table;
  // the gradient table lives on the device, so the host cannot tell which entries are null: the grid covers
  // the tiles of every tensor, and workgroups beyond the step's compacted list exit at once
  uint64_t bound = p->tensor_tiles;
  if (a.paired) {
    bound = 0;
    for (const auto& t : h.tensors) bound += paired_tiles_bound(t.numel, a.paired);
    if (bound + 8ull * 65536 >= (1ull << 31)) return fail(MOEV_E_RANGE, "convert_replay_static: too many tiles for one launch");
  }
  return launch_replay_direct(p, a, adam, d_scratch, direct_grid(bound, p->xcd_regions), -1, nullptr, s);
}

int convert_window_step(moev_plan* p, uint32_t slot, const void* h_pinned, void* d_packed, const moev_adam* adam,
                        uint8_t* d_active_mask, void* const* grads, const moev_state* state, void* stream) {
  int rc = check_unpack_args(p, slot, h_pinned, d_packed, state, "convert_window_step");
  if (rc != MOEV_OK) return rc;
  rc = check_replay_args(p, adam, d_active_mask, grads, state, "convert_window_step");
  if (rc != MOEV_OK) return rc;
  const auto& h = p->host;
  // the operators this snapshot activates take their first replayed step right away: they need gradients
  for (uint32_t t = 0; t < h.n_tensors; ++t)
    if (h.slot_of_op[h.tensors[t].op] == slot && h.tensors[t].numel && !grads[t])
      return fail(MOEV_E_INVAL, "convert_window_step: tensor %u becomes active in slot %u but has no gradient", t, slot);
  std::lock_guard<std::mutex> lock(p->mu);
  hipStream_t s = static_cast<hipStream_t>(stream);
  const bool fused = !p->persistent && fp32_regime(h);
  rc = launch_unpack_locked(p, slot, h_pinned, d_packed, state, d_active_mask, s, fused);
  if (rc != MOEV_OK) return rc;
  return launch_replay_locked(p, adam, d_active_mask, grads, state, s, fused ? static_cast<int>(slot) : -1, d_packed);
}

}  // extern "C"
