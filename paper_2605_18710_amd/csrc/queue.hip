// Host side of the persistent kernels' work queues: which 64-byte block of counters a stream
// uses, and how many workgroups a launch needs.  The counters live in an array that is part of
// the library's device code (zero when the code object is loaded, set back to zero by the last
// workgroup of every launch), so no call here allocates or clears device memory, and launches
// can be captured into HIP graphs (replay a captured launch on the stream it was captured on:
// the queue belongs to that stream).
#include <stdlib.h>
#include <mutex>
#include <unordered_map>
#include <vector>
#include "tile_queue.h"

namespace {

constexpr int kQueueSlots = 2048;            // streams per device that can hold a queue at once
constexpr int kMaxDevices = 64;
__device__ __align__(256) unsigned tile_queue_counters[kQueueSlots * kTileQueueWords];   // 4 MiB

struct DeviceQueues {
  unsigned* base = nullptr;                  // device address of tile_queue_counters on this GPU
  std::unordered_map<hipStream_t, int> slot; // stream -> block index
  std::vector<int> free_slots;               // blocks given back by destroyed streams
  int next = 0;
};

std::mutex g_mu;
DeviceQueues g_dev[kMaxDevices];

}  // namespace

static mosaic_status tile_queue_for_stream(hipStream_t s, unsigned** ctr_out) {
  int dev = 0;
  MOSAIC_HIP(hipGetDevice(&dev));
  if (dev < 0 || dev >= kMaxDevices) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "device index %d beyond the %d this table holds", dev, kMaxDevices);
  std::lock_guard<std::mutex> lk(g_mu);
  DeviceQueues& d = g_dev[dev];
  if (!d.base) {
    void* p = nullptr;
    MOSAIC_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(tile_queue_counters)));
    if (!p) MOSAIC_FAIL(MOSAIC_EHIP, "hipGetSymbolAddress returned a null address");
    d.base = (unsigned*)p;
  }
  auto it = d.slot.find(s);
  if (it == d.slot.end()) {
    int idx;
    if (!d.free_slots.empty()) { idx = d.free_slots.back(); d.free_slots.pop_back(); }
    else if (d.next < kQueueSlots) idx = d.next++;
    else MOSAIC_FAIL(MOSAIC_ENOMEM, "more than %d live streams have launched persistent kernels on device %d", kQueueSlots, dev);
    it = d.slot.emplace(s, idx).first;
  }
  *ctr_out = d.base + (size_t)it->second * kTileQueueWords;
  return MOSAIC_OK;
}

// Called with the stream idle (its owner synchronises it first), before it is destroyed: a new
// stream may be handed the same handle value, or the block.
void tile_queue_release(hipStream_t s) {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return;
  std::lock_guard<std::mutex> lk(g_mu);
  DeviceQueues& d = g_dev[dev];
  auto it = d.slot.find(s);
  if (it == d.slot.end()) return;
  d.free_slots.push_back(it->second);
  d.slot.erase(it);
}

// A quota that is a multiple of 32 CUs gives every shader engine of every XCD the same number
// of CUs and `quota * wg_per_cu` workgroups fill them exactly.  Any other quota of 32 CUs or
// more holds fewer workgroups at once than it has room for (tile_queue.h); the launch is then
// sized for the next multiple of 32, so that whatever room the dispatcher does use is used.
// Workgroups that find no room start when others leave, find the queue empty and leave at once.
mosaic_status tile_queue_plan(hipStream_t s, int quota, int wg_per_cu, int64_t n_items, int unit, bool prefer_queue,
                              TileQueueArgs* q, int* grid) {
  if (n_items <= 0 || n_items > INT32_MAX / 2) MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "work list of %lld items", (long long)n_items);
  bool even = quota % 32 == 0 || quota < 32;
#ifdef MOSAIC_TUNING
  // A/B timing only: MOSAIC_TQ_FORCE=1 sends every launch through the queue
  static const int force = getenv("MOSAIC_TQ_FORCE") ? atoi(getenv("MOSAIC_TQ_FORCE")) : 0;
  if (force == 1) { prefer_queue = true; }
#endif
  const int64_t resident = (int64_t)tile_queue_sure_cus(quota) * wg_per_cu;
  q->n_items = (int)n_items;
  q->ctr = nullptr;
  q->chunk = 1; q->n_full = 0; q->tail_per = 0;
  if (even && (n_items <= resident || !prefer_queue)) {
    // every workgroup resident at once: static rounds, no queue
    q->mode = TQ_ROUNDS;
    int64_t g = resident;
    if (g > n_items) g = (resident & 7) == 0 ? (n_items + 7) / 8 * 8 : n_items;   // XCD x takes the x-th eighth
    *grid = (int)g;
    return MOSAIC_OK;
  }
  q->mode = n_items <= resident ? TQ_ONCE : TQ_QUEUE;
  const int64_t chunk = unit > 0 ? unit : (resident + 7) / 8;
  q->chunk = (int)chunk;
  q->n_full = (int)(n_items / (8 * chunk) * (8 * chunk));
  q->tail_per = (int)((n_items - q->n_full + 7) / 8);
  int64_t g = resident;
  if (!even) {
    g = (int64_t)(quota / 32 + 1) * 32 * wg_per_cu;
    const int64_t cap = ((n_items + 31) / 32 + 1) * 32;      // a launch of few items needs no more than this
    if (g > cap) g = cap;
  } else if (g > n_items) {
    g = n_items;
  }
  *grid = (int)g;
  return tile_queue_for_stream(s, &q->ctr);
}
