// Work queue of the persistent kernels.
//
// A persistent kernel's grid is sized to its stream's CU quota, but how many of its workgroups
// are resident at once, and on which XCD each of them runs, is the dispatcher's business: under a
// CU mask that gives the shader engines of an XCD unequal numbers of CUs some workgroups only
// start when others have left.  A static deal of work items to blockIdx then makes the late
// workgroups run their whole share alone at the end.  Here every workgroup draws its next item
// from a queue instead; a workgroup that starts late finds the queue empty and leaves.  Which
// workgroup computes an item never changes how it is computed, so results stay bit-identical
// for every quota, mask and dispatch order.
//
// The queue is eight lists, one per XCD, so that the workgroups that run on one XCD at the
// same time work on neighbouring items and meet in that XCD's L2: the flat item list
// [0, n_items) is cut into chunks of `chunk` consecutive items and chunk c belongs to list
// c % 8; what is left after the last whole round of eight chunks is cut into eight equal
// pieces.  With the chunk as long as an XCD has resident workgroups, the workgroups of an XCD
// walk one contiguous patch of items per round, and the last, partial round is spread evenly.
// A workgroup reads the id of the XCD it really runs on from the hardware register, draws
// from that list, and moves on to the other lists when its own is used up.
//
// Three modes, chosen on the host from the item count and the quota:
//   TQ_ROUNDS  a quota whose workgroups are all resident at once (a multiple of 32 CUs, or fewer
//              than 32) and items of equal cost: no queue.  Round r hands out items
//              [r*G, (r+1)*G) to the G workgroups; workgroup b is taken to run on XCD b % 8 and
//              XCD x takes the x-th eighth of the round.  No atomics, nothing to wait for.
//   TQ_ONCE    at most one item per workgroup under any other quota: one claim per workgroup.
//   TQ_QUEUE   several items per workgroup: claims until the queue is empty.
//
// Device memory per queue: sixteen counters, each on a cache line of its own (workgroups of
// one XCD then contend only with each other; hundreds of workgroups adding to one address
// cost tens of microseconds): [32*x] the cursor of list x, [32*(8+x)] the number of workgroups
// that have left from XCD x.  A workgroup that sees all of the launch gone sets the counters
// back to zero, so a queue is ready for the next launch on the same stream without a memset
// (kernels of one stream run one after another; every stream has its own queue).
#pragma once
#include "common.h"

constexpr int kTileQueueStride = 32;                       // counters (uint32) between two cursors: 128 bytes
constexpr int kTileQueueWords = 16 * kTileQueueStride;     // per queue: 2 KB

enum { TQ_ROUNDS = 0, TQ_ONCE = 1, TQ_QUEUE = 2 };

struct TileQueueArgs {
  unsigned* ctr;     // the queue's counters
  int n_items;       // length of the flat item list
  int chunk;         // consecutive items per chunk (>= 1)
  int n_full;        // items covered by whole rounds of eight chunks (a multiple of 8 * chunk)
  int tail_per;      // the remaining n_items - n_full items go to the lists in pieces of this many
  int mode;
};

// Host side (queue.hip).  Fills `q` for a launch of n_items items on the stream's queue of the
// current device, with chunks of `unit` items (0: as many as an XCD has resident workgroups;
// prefer_queue: use the queue even where static rounds would do, for items of unequal cost),
// and returns the number of workgroups to launch: every CU of the quota
// receives wg_per_cu workgroups whatever the mask's share of each shader engine.  Queues live
// in an array built into the library's device code; nothing is allocated.
mosaic_status tile_queue_plan(hipStream_t s, int quota, int wg_per_cu, int64_t n_items, int unit, bool prefer_queue,
                              TileQueueArgs* q, int* grid);
// CUs of a quota that are certain to hold a workgroup at the same time.  The dispatcher deals
// the workgroups of a launch round-robin over the XCDs and, inside an XCD, over its four shader
// engines, and stalls at the first shader engine that is full although others have room
// (measured with a probe that records where and when every workgroup starts: 232 CUs start
// 224 to 228 workgroups at once, 248 start 225, 216 start 200, 40 start 32; multiples of 32
// and quotas below 32 start all).  Launch plans count rounds with this number; the launch
// itself is sized for every CU, and the work queue hands the stragglers nothing.
static inline int tile_queue_sure_cus(int quota) { return quota >= 32 ? quota / 32 * 32 : quota; }
// Gives a stream's queue back; the stream must be idle.
void tile_queue_release(hipStream_t s);

#ifdef __HIPCC__
// flat index of entry e of list x, or -1 past the end of that list (monotone in e)
__device__ __forceinline__ int tq_item(const TileQueueArgs& q, int x, unsigned e) {
  const unsigned full_e = (unsigned)q.n_full >> 3;        // entries of a list inside the whole rounds
  if (e < full_e) return (int)((e / (unsigned)q.chunk) * 8u * (unsigned)q.chunk + (unsigned)(x * q.chunk) + e % (unsigned)q.chunk);
  const unsigned t = e - full_e;
  if (t >= (unsigned)q.tail_per) return -1;
  const int64_t idx = (int64_t)q.n_full + (int64_t)x * q.tail_per + t;
  return idx < q.n_items ? (int)idx : -1;
}

__device__ __forceinline__ int tq_xcc_id() {
  return (int)(__builtin_amdgcn_s_getreg((31 << 11) | 20) & 7u);   // XCC_ID, bits 3:0 (eight XCDs)
}

// State of a workgroup's draws: the list thread 0 currently draws from, or the round.
struct TileQueueCursor {
  int list;
  int round;
  __device__ __forceinline__ void init() { list = tq_xcc_id(); round = 0; }
};

// TQ_ROUNDS: this workgroup's item of round r, or -1 when it has none (nor in any later round)
__device__ __forceinline__ int tq_rounds_item(const TileQueueArgs& q, int r) {
  const int G = gridDim.x, b = blockIdx.x;
  const int64_t base = (int64_t)r * G;
  if (base >= q.n_items) return -1;
  const int cnt = (int)min((int64_t)G, q.n_items - base);
  int local = b;
  if ((G & 7) == 0) {
    const int per = (cnt + 7) >> 3, slot = b >> 3;
    if (slot >= per) return -1;
    local = (b & 7) * per + slot;
  }
  return local < cnt ? (int)base + local : -1;
}

// Claims the next entry of the current list; the returned entry number is turned into an item by
// tq_resolve.  Issued early (its latency then hides under other work), resolved late.
__device__ __forceinline__ unsigned tq_claim(const TileQueueArgs& q, const TileQueueCursor& c) {
  return __hip_atomic_fetch_add(q.ctr + c.list * kTileQueueStride, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// number of entries of list x
__device__ __forceinline__ int tq_list_len(const TileQueueArgs& q, int x) {
  const int tail = q.n_items - q.n_full, mine = tail - x * q.tail_per;
  return (q.n_full >> 3) + (mine <= 0 ? 0 : (mine < q.tail_per ? mine : q.tail_per));
}

// Item of a claimed entry; when the current list is used up, looks at all cursors for the
// nearest list that still has entries and claims from it.  -1: every list is used up.
// *left (may be null) receives the number of entries left in the list the item came from.
__device__ __forceinline__ int tq_resolve(const TileQueueArgs& q, TileQueueCursor& c, unsigned e, int* left = nullptr) {
  int it = tq_item(q, c.list, e);
  while (it < 0) {
    int found = -1;
#pragma unroll
    for (int d = 1; d < 8; ++d) {
      const int x = (c.list + d) & 7;
      const unsigned cx = __hip_atomic_load(q.ctr + x * kTileQueueStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      if (found < 0 && tq_item(q, x, cx) >= 0) found = x;
    }
    if (found < 0) return -1;
    c.list = found;
    e = tq_claim(q, c);
    it = tq_item(q, c.list, e);
  }
  if (left) *left = tq_list_len(q, c.list) - (int)e - 1;
  return it;
}

// The first item of a workgroup: computed by every thread in TQ_ROUNDS mode, a claim by thread 0
// otherwise (other threads then get garbage).
__device__ __forceinline__ int tq_first_item(const TileQueueArgs& q, TileQueueCursor& c) {
  c.init();
  if (q.mode == TQ_ROUNDS) return tq_rounds_item(q, 0);
  return tq_resolve(q, c, tq_claim(q, c));
}

// Called once by every workgroup, after its last claim has returned.  The workgroup counts
// itself out on its XCD's counter, then adds up all eight: the one that finds the whole launch
// gone zeroes the counters for the next launch (the addition is complete before the eight
// counters are read, so of two workgroups leaving at the same time at least one sees the
// other; both zeroing is harmless).
__device__ __forceinline__ void tq_leave(const TileQueueArgs& q) {
  if (q.mode == TQ_ROUNDS) return;             // no counter was touched
  unsigned* gone = q.ctr + 8 * kTileQueueStride;
  // sequentially consistent: the addition has been performed before the loads below are issued
  __hip_atomic_fetch_add(gone + tq_xcc_id() * kTileQueueStride, 1u, __ATOMIC_SEQ_CST, __HIP_MEMORY_SCOPE_AGENT);
  unsigned v[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) v[i] = __hip_atomic_load(gone + i * kTileQueueStride, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  unsigned sum = 0;
#pragma unroll
  for (int i = 0; i < 8; ++i) sum += v[i];
  if (sum == gridDim.x) {
#pragma unroll
    for (int i = 0; i < 16; ++i) __hip_atomic_store(q.ctr + i * kTileQueueStride, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  }
}

// Draw loop for kernels with four spare bytes of LDS (`mail`):
//   int item = tq_first(q, c, mail);
//   while (item >= 0) {
//     ...work on item; shortly before its end:  const unsigned e = tq_claim_ahead(q, c);
//     item = tq_next(q, c, e, mail);
//   }
//   tq_done(q);
// Thread 0 claims the following item when the current one is nearly done (claimed earlier, a
// workgroup that started first would take items from workgroups that have not started yet)
// and resolves the claim after the item's last stores, so most of the round trip to memory
// hides under the item's tail.  All threads call every function.
__device__ __forceinline__ int tq_first(const TileQueueArgs& q, TileQueueCursor& c, int* mail) {
  if (q.mode == TQ_ROUNDS) return tq_first_item(q, c);
  if (threadIdx.x == 0) *mail = tq_first_item(q, c);
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(*(volatile int*)mail);
}
__device__ __forceinline__ unsigned tq_claim_ahead(const TileQueueArgs& q, const TileQueueCursor& c) {
  return (threadIdx.x == 0 && q.mode == TQ_QUEUE) ? tq_claim(q, c) : 0u;
}
__device__ __forceinline__ int tq_next(const TileQueueArgs& q, TileQueueCursor& c, unsigned e, int* mail) {
  if (q.mode == TQ_ROUNDS) return tq_rounds_item(q, ++c.round);
  if (q.mode != TQ_QUEUE) return -1;
  __syncthreads();                 // everybody has read the previous item
  if (threadIdx.x == 0) *mail = tq_resolve(q, c, e);
  __syncthreads();
  return __builtin_amdgcn_readfirstlane(*(volatile int*)mail);
}
__device__ __forceinline__ void tq_done(const TileQueueArgs& q) {
  if (threadIdx.x == 0) tq_leave(q);
}
#endif
