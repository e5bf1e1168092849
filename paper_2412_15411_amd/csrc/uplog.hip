// uplog.hip -- upstream logging ring (Sec. 3.4): stage-boundary tensors (activations sent
// downstream, gradients sent upstream) are copied device -> pinned host memory on a side stream,
// tagged with (iteration, micro-batch, kind), kept until the sparse checkpoint that makes them
// obsolete has persisted ("Stale Log Cleanup"), and copied back for localized recovery.
//
// The ring is host bookkeeping around hipMemcpyAsync: entries are laid out in arrival order in
// one caller-owned pinned buffer; garbage collection frees from the oldest end.
#include <hip/hip_runtime.h>

#include <cstdarg>
#include <cstdio>
#include <deque>
#include <mutex>
#include <new>
#include <string>

#include "moev.h"

namespace moev {
int set_error(int code, const char* fmt, ...);  // defined in api.hip: fills moev_last_error()
}

namespace {

struct Entry {
  uint64_t iter;
  uint32_t micro_batch, kind;
  uint64_t offset, nbytes, reserved;  // reserved = nbytes rounded up to the ring's alignment
};

constexpr uint64_t kAlign = 256;

#define UPLOG_HIP(call)                                                                            \
  do {                                                                                             \
    hipError_t e_ = (call);                                                                        \
    if (e_ != hipSuccess)                                                                          \
      return moev::set_error(MOEV_E_HIP, "%s failed: %s (%s:%d)", #call, hipGetErrorString(e_), __FILE__, __LINE__); \
  } while (0)

}  // namespace

struct moev_uplog {
  uint8_t* base = nullptr;
  uint64_t capacity = 0;
  uint64_t head = 0;        // offset where the next entry starts
  uint64_t used = 0;        // bytes between the oldest entry's start and head, including skipped tails
  std::deque<Entry> entries;  // oldest first
  uint32_t max_entries = 0;
  std::mutex mu;
};

namespace {

// Finds room for `nbytes` at the head of the ring (entries never wrap: if the tail of the buffer
// is too short it is skipped).  Returns false when the ring is full.
bool reserve_locked(moev_uplog* log, uint64_t nbytes, uint64_t* offset, uint64_t* reserved) {
  uint64_t need = (nbytes + kAlign - 1) / kAlign * kAlign;
  if (need == 0) need = kAlign;  // an empty tensor still gets a slot of its own
  if (need > log->capacity || log->entries.size() >= log->max_entries) return false;
  if (log->entries.empty()) {
    log->head = 0;
    log->used = 0;
  }
  uint64_t at = log->head, skipped = 0;
  bool restart = false;
  if (at + need > log->capacity) {  // does not fit before the end: start again at 0
    skipped = log->capacity - at;
    at = 0;
    restart = true;
  }
  // The live entries occupy [tail, head) going forward, tail = start of the oldest entry; the head
  // never catches up with the tail (head == tail only when the ring is empty).
  if (!log->entries.empty()) {
    const uint64_t tail = log->entries.front().offset;
    if (log->head > tail) {          // not wrapped: free = [head, capacity) and [0, tail)
      if (restart && need >= tail) return false;
    } else {                          // wrapped: free = [head, tail)
      if (restart || at + need >= tail) return false;
    }
  }
  *offset = at;
  *reserved = need + skipped;
  log->head = at + need;
  log->used += need + skipped;
  return true;
}

const Entry* find_locked(const moev_uplog* log, uint64_t iter, uint32_t mb, uint32_t kind) {
  for (auto it = log->entries.rbegin(); it != log->entries.rend(); ++it)
    if (it->iter == iter && it->micro_batch == mb && it->kind == kind) return &*it;
  return nullptr;
}

}  // namespace

extern "C" {

int uplog_create(void* h_pinned_ring, size_t ring_bytes, uint32_t max_entries, moev_uplog** out) {
  if (!h_pinned_ring || !out || ring_bytes < kAlign || max_entries == 0)
    return moev::set_error(MOEV_E_INVAL, "uplog_create: null ring, ring below 256 bytes or no entries");
  if (reinterpret_cast<uintptr_t>(h_pinned_ring) % 16)
    return moev::set_error(MOEV_E_INVAL, "uplog_create: ring must be 16-byte aligned");
  moev_uplog* log = new (std::nothrow) moev_uplog();
  if (!log) return moev::set_error(MOEV_E_NOMEM, "uplog_create: out of host memory");
  log->base = static_cast<uint8_t*>(h_pinned_ring);
  log->capacity = ring_bytes / kAlign * kAlign;
  log->max_entries = max_entries;
  *out = log;
  return MOEV_OK;
}

void uplog_free(moev_uplog* log) { delete log; }

int uplog_reserve(moev_uplog* log, uint64_t iter, uint32_t micro_batch, uint32_t kind, size_t nbytes,
                  uint64_t* offset_out) {
  if (!log || kind > 1) return moev::set_error(MOEV_E_INVAL, "uplog_reserve: null log or kind not 0/1");
  std::lock_guard<std::mutex> lock(log->mu);
  if (!log->entries.empty() && iter < log->entries.back().iter)
    return moev::set_error(MOEV_E_INVAL, "uplog_reserve: iterations must not go backwards");
  if (find_locked(log, iter, micro_batch, kind))
    return moev::set_error(MOEV_E_INVAL, "uplog_reserve: (%llu, %u, %u) is already logged",
                           static_cast<unsigned long long>(iter), micro_batch, kind);
  uint64_t offset = 0, reserved = 0;
  if (!reserve_locked(log, nbytes, &offset, &reserved))
    return moev::set_error(MOEV_E_NOMEM, "uplog: ring full (%zu bytes asked, %llu of %llu in use, %zu entries)", nbytes,
                           static_cast<unsigned long long>(log->used), static_cast<unsigned long long>(log->capacity),
                           log->entries.size());
  log->entries.push_back(Entry{iter, micro_batch, kind, offset, nbytes, reserved});
  if (offset_out) *offset_out = offset;
  return MOEV_OK;
}

int uplog_append(moev_uplog* log, uint64_t iter, uint32_t micro_batch, uint32_t kind, const void* d_tensor,
                 size_t nbytes, void* side_stream, void* ready) {
  if (!d_tensor && nbytes) return moev::set_error(MOEV_E_INVAL, "uplog_append: null tensor");
  uint64_t offset = 0;
  int rc = uplog_reserve(log, iter, micro_batch, kind, nbytes, &offset);
  if (rc != MOEV_OK) return rc;
  hipStream_t s = static_cast<hipStream_t>(side_stream);
  if (ready) UPLOG_HIP(hipStreamWaitEvent(s, static_cast<hipEvent_t>(ready), 0));
  if (nbytes) UPLOG_HIP(hipMemcpyAsync(log->base + offset, d_tensor, nbytes, hipMemcpyDeviceToHost, s));
  return MOEV_OK;
}

int uplog_find(moev_uplog* log, uint64_t iter, uint32_t micro_batch, uint32_t kind, const void** h_ptr, size_t* nbytes) {
  if (!log) return moev::set_error(MOEV_E_INVAL, "uplog_find: null log");
  std::lock_guard<std::mutex> lock(log->mu);
  const Entry* e = find_locked(log, iter, micro_batch, kind);
  if (!e)
    return moev::set_error(MOEV_E_RANGE, "uplog: nothing logged for iteration %llu micro-batch %u kind %u",
                           static_cast<unsigned long long>(iter), micro_batch, kind);
  if (h_ptr) *h_ptr = log->base + e->offset;
  if (nbytes) *nbytes = e->nbytes;
  return MOEV_OK;
}

int uplog_replay(moev_uplog* log, uint64_t iter, uint32_t micro_batch, uint32_t kind, void* d_dst, size_t cap,
                 void* stream) {
  const void* src = nullptr;
  size_t nbytes = 0;
  int rc = uplog_find(log, iter, micro_batch, kind, &src, &nbytes);
  if (rc != MOEV_OK) return rc;
  if (cap < nbytes) return moev::set_error(MOEV_E_RANGE, "uplog_replay: destination too small");
  if (!d_dst && nbytes) return moev::set_error(MOEV_E_INVAL, "uplog_replay: null destination");
  if (nbytes) UPLOG_HIP(hipMemcpyAsync(d_dst, src, nbytes, hipMemcpyHostToDevice, static_cast<hipStream_t>(stream)));
  return MOEV_OK;
}

int64_t uplog_gc(moev_uplog* log, uint64_t first_kept_iter) {
  if (!log) return moev::set_error(MOEV_E_INVAL, "uplog_gc: null log");
  std::lock_guard<std::mutex> lock(log->mu);
  int64_t dropped = 0;
  while (!log->entries.empty() && log->entries.front().iter < first_kept_iter) {
    log->used -= log->entries.front().reserved;
    log->entries.pop_front();
    ++dropped;
  }
  if (log->entries.empty()) {
    log->head = 0;
    log->used = 0;
  }
  return dropped;
}

int uplog_stats(moev_uplog* log, uint64_t* entries, uint64_t* bytes_in_use, uint64_t* capacity) {
  if (!log) return moev::set_error(MOEV_E_INVAL, "uplog_stats: null log");
  std::lock_guard<std::mutex> lock(log->mu);
  if (entries) *entries = log->entries.size();
  if (bytes_in_use) *bytes_in_use = log->used;
  if (capacity) *capacity = log->capacity;
  return MOEV_OK;
}

}  // extern "C"
