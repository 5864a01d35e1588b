// Launcher: CU-mask construction, quota'd streams and their pool (Sec. 3.2), plan
// validation (Eq. 5), quota choice from measured curves (Eq. 4-5), and stage execution in
// colocated, time-sliced (Eq. 1) and chained modes.
#include <stdlib.h>
#include <string.h>
#include <atomic>
#include <mutex>
#include <new>
#include <string>
#include <thread>
#include <vector>
#include "kernels.h"
#include "tile_queue.h"

// ------------------------------------------------------------------------------ errors
static thread_local char g_err[512] = "";

void mosaic_set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof(g_err), fmt, ap);
  va_end(ap);
}

extern "C" const char* mosaic_last_error(void) { return g_err; }

// ------------------------------------------------------------------------------ device
mosaic_status mosaic_device_info(DeviceInfo* out) {
  static DeviceInfo cached = {0, 0, false};
  static std::mutex mu;
  std::lock_guard<std::mutex> lk(mu);
  if (!cached.ok) {
    int dev = 0;
    MOSAIC_HIP(hipGetDevice(&dev));
    hipDeviceProp_t prop;
    MOSAIC_HIP(hipGetDeviceProperties(&prop, dev));
    cached.cu_count = prop.multiProcessorCount;
    // gfx942 / gfx950 parts expose 8 accelerator dies in the default partition mode;
    // the probe kernel is the check that this matches the device at hand.
    cached.xcd_count = (cached.cu_count % 8 == 0) ? 8 : 1;
    cached.ok = true;
  }
  *out = cached;
  return MOSAIC_OK;
}

extern "C" int32_t mosaic_device_cu_count(void) {
  DeviceInfo di;
  mosaic_status s = mosaic_device_info(&di);
  return s == MOSAIC_OK ? di.cu_count : s;
}

extern "C" int32_t mosaic_device_xcd_count(void) {
  DeviceInfo di;
  mosaic_status s = mosaic_device_info(&di);
  return s == MOSAIC_OK ? di.xcd_count : s;
}

// ------------------------------------------------------------------------------- masks
extern "C" mosaic_status mosaic_cu_mask_build(int32_t cu_total, int32_t n_xcd, int32_t cu_quota, int32_t cu_offset,
                                              int32_t layout, uint32_t* words, int32_t n_words) {
  if (!words) MOSAIC_FAIL(MOSAIC_EINVAL, "null mask buffer");
  if (cu_total <= 0 || n_xcd <= 0 || cu_total % n_xcd) MOSAIC_FAIL(MOSAIC_EINVAL, "bad device shape %d CUs / %d XCDs", cu_total, n_xcd);
  if (n_words < (cu_total + 31) / 32) MOSAIC_FAIL(MOSAIC_EINVAL, "mask buffer of %d words is too short", n_words);
  if (cu_quota <= 0) MOSAIC_FAIL(MOSAIC_EQUOTA, "quota %d must be positive", cu_quota);
  if (cu_offset < 0 || cu_offset + cu_quota > cu_total)
    MOSAIC_FAIL(MOSAIC_EQUOTA, "CU range [%d, %d) leaves the device's %d CUs", cu_offset, cu_offset + cu_quota, cu_total);
  const int per = cu_total / n_xcd;
  if (layout == MOSAIC_XCD_ALIGNED) {
    if (cu_quota % per || cu_offset % per)
      MOSAIC_FAIL(MOSAIC_EQUOTA, "XCD-aligned quota and offset must be multiples of %d CUs", per);
  } else if (layout != MOSAIC_STRIPED) {
    MOSAIC_FAIL(MOSAIC_EINVAL, "bad mask layout %d", layout);
  }
  for (int i = 0; i < n_words; ++i) words[i] = 0;
  for (int c = cu_offset; c < cu_offset + cu_quota; ++c) {
    // mask bit i addresses slot i / n_xcd of XCD i % n_xcd
    const int bit = (layout == MOSAIC_STRIPED) ? c : (c % per) * n_xcd + c / per;
    words[bit >> 5] |= 1u << (bit & 31);
  }
  return MOSAIC_OK;
}

// ----------------------------------------------------------------------------- streams
struct mosaic_stream {
  hipStream_t s = nullptr;
  int quota = 0, offset = 0, layout = 0;
  bool pooled = false;
  std::vector<uint32_t> mask;
};

static std::atomic<int64_t> g_creations{0};

hipStream_t mosaic_stream_hip(const mosaic_stream* s) { return s ? s->s : nullptr; }
int mosaic_stream_quota_or(const mosaic_stream* s, int fallback) { return s ? s->quota : fallback; }

extern "C" mosaic_status mosaic_stream_create(int32_t cu_quota, int32_t cu_offset, int32_t layout, mosaic_stream** out) {
  if (!out) MOSAIC_FAIL(MOSAIC_EINVAL, "null output");
  *out = nullptr;
  DeviceInfo di;
  MOSAIC_TRY(mosaic_device_info(&di));
  std::vector<uint32_t> mask((di.cu_count + 31) / 32);
  MOSAIC_TRY(mosaic_cu_mask_build(di.cu_count, di.xcd_count, cu_quota, cu_offset, layout, mask.data(), (int)mask.size()));
  // One queue spans every XCD and its workgroups are dealt round-robin over them, so the
  // driver refuses a mask that leaves an XCD without a CU (and the runtime's failure path
  // is not safe to enter): reject such masks here.
  for (int x = 0; x < di.xcd_count; ++x) {
    bool any = false;
    for (int i = x; i < di.cu_count; i += di.xcd_count) any |= (mask[i >> 5] >> (i & 31)) & 1u;
    if (!any) {
      if (layout == MOSAIC_XCD_ALIGNED)
        MOSAIC_FAIL(MOSAIC_EUNSUPPORTED, "XCD-aligned quota %d at offset %d leaves XCD %d without CUs; this device "
                    "spreads every queue over all %d XCDs, use MOSAIC_STRIPED", cu_quota, cu_offset, x, di.xcd_count);
      MOSAIC_FAIL(MOSAIC_EQUOTA, "quota %d leaves XCD %d without CUs; the smallest quota is %d", cu_quota, x, di.xcd_count);
    }
  }
  mosaic_stream* st = new (std::nothrow) mosaic_stream();
  if (!st) MOSAIC_FAIL(MOSAIC_ENOMEM, "host allocation failed");
  hipError_t e;
  if (cu_quota == di.cu_count) e = hipStreamCreate(&st->s);
  else e = hipExtStreamCreateWithCUMask(&st->s, (uint32_t)mask.size(), mask.data());
  if (e != hipSuccess) {
    delete st;
    MOSAIC_FAIL(MOSAIC_EHIP, "stream creation failed: %s", hipGetErrorString(e));
  }
  st->quota = cu_quota; st->offset = cu_offset; st->layout = layout; st->mask = mask;
  g_creations.fetch_add(1);
  *out = st;
  return MOSAIC_OK;
}

extern "C" void* mosaic_stream_native(const mosaic_stream* s) { return s ? (void*)s->s : nullptr; }
extern "C" int32_t mosaic_stream_quota(const mosaic_stream* s) { return s ? s->quota : 0; }
extern "C" int32_t mosaic_stream_offset(const mosaic_stream* s) { return s ? s->offset : 0; }

extern "C" mosaic_status mosaic_stream_destroy(mosaic_stream* s) {
  if (!s) return MOSAIC_OK;
  if (s->pooled) MOSAIC_FAIL(MOSAIC_EINVAL, "a pooled stream is released with mosaic_pool_clear");
  // the stream's work queue goes back to the table once nothing can be using it
  (void)hipStreamSynchronize(s->s);
  tile_queue_release(s->s);
  hipError_t e = hipStreamDestroy(s->s);
  delete s;
  if (e != hipSuccess) MOSAIC_FAIL(MOSAIC_EHIP, "hipStreamDestroy failed: %s", hipGetErrorString(e));
  return MOSAIC_OK;
}

// -------------------------------------------------------------------------------- pool
static std::mutex g_pool_mu;
static std::vector<mosaic_stream*> g_pool;

static mosaic_stream* pool_find(int quota, int offset, int layout) {
  for (mosaic_stream* s : g_pool)
    if (s->quota == quota && s->offset == offset && s->layout == layout) return s;
  return nullptr;
}

extern "C" mosaic_status mosaic_pool_reserve(int32_t cu_quota, int32_t cu_offset, int32_t layout) {
  std::lock_guard<std::mutex> lk(g_pool_mu);
  if (pool_find(cu_quota, cu_offset, layout)) return MOSAIC_OK;
  mosaic_stream* s = nullptr;
  MOSAIC_TRY(mosaic_stream_create(cu_quota, cu_offset, layout, &s));
  s->pooled = true;
  g_pool.push_back(s);
  return MOSAIC_OK;
}

extern "C" mosaic_status mosaic_pool_get(int32_t cu_quota, int32_t cu_offset, int32_t layout, mosaic_stream** out) {
  if (!out) MOSAIC_FAIL(MOSAIC_EINVAL, "null output");
  std::lock_guard<std::mutex> lk(g_pool_mu);
  *out = pool_find(cu_quota, cu_offset, layout);
  if (!*out)
    MOSAIC_FAIL(MOSAIC_EQUOTA, "no pooled stream for quota %d at offset %d (layout %d): reserve it before the stage runs",
                cu_quota, cu_offset, layout);
  return MOSAIC_OK;
}

extern "C" int64_t mosaic_pool_creations(void) { return g_creations.load(); }

extern "C" mosaic_status mosaic_pool_clear(void) {
  std::lock_guard<std::mutex> lk(g_pool_mu);
  mosaic_status rc = MOSAIC_OK;
  for (mosaic_stream* s : g_pool) {
    (void)hipStreamSynchronize(s->s);
    tile_queue_release(s->s);
    if (hipStreamDestroy(s->s) != hipSuccess) rc = MOSAIC_EHIP;
    delete s;
  }
  g_pool.clear();
  if (rc != MOSAIC_OK) mosaic_set_error("hipStreamDestroy failed while clearing the pool");
  return rc;
}

// ------------------------------------------------------------------------------- probe
__global__ void placement_probe_kernel(int32_t* out, int n) {
  if (threadIdx.x == 0 && (int)blockIdx.x < n) {
    // HW_ID (register 4): CU_ID bits 11:8, SH_ID bit 12, SE_ID bits 15:13.  XCC_ID (register 20): bits 3:0.
    const uint32_t hw = __builtin_amdgcn_s_getreg((31 << 11) | 4);
    const uint32_t xcc = __builtin_amdgcn_s_getreg((31 << 11) | 20);
    out[3 * blockIdx.x + 0] = (int32_t)(xcc & 0xF);
    out[3 * blockIdx.x + 1] = (int32_t)((hw >> 13) & 0x7);
    out[3 * blockIdx.x + 2] = (int32_t)(((hw >> 12) & 0x1) * 16 + ((hw >> 8) & 0xF));
  }
  // keep the workgroup resident for a moment so that later workgroups spread out
  __builtin_amdgcn_s_sleep(64);
}

extern "C" mosaic_status mosaic_probe_placement(const mosaic_stream* stream, int32_t n, int32_t* out) {
  if (!out || n <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "bad probe arguments");
  placement_probe_kernel<<<n, 64, 0, mosaic_stream_hip(stream)>>>(out, n);
  MOSAIC_LAUNCH_CHECK();
  return MOSAIC_OK;
}

// ------------------------------------------------------------------------------- plans
extern "C" int32_t mosaic_device_hw_queues(void) {
  // the runtime's limit on hardware queues per process: its default unless the environment says otherwise
  const char* e = getenv("GPU_MAX_HW_QUEUES");
  const int v = e ? atoi(e) : 0;
  return v > 0 ? v : 4;
}

extern "C" int32_t mosaic_plan_stream_count(const mosaic_plan* p) {
  if (!p || !p->cu_quota || !p->cu_offset || p->n <= 0) return 0;
  if (p->mode != MOSAIC_COLOCATED) return 1;
  int distinct = 0;
  for (int i = 0; i < p->n; ++i) {
    bool first = true;
    for (int j = 0; j < i; ++j)
      if (p->cu_quota[j] == p->cu_quota[i] && p->cu_offset[j] == p->cu_offset[i]) first = false;
    distinct += first;
  }
  return distinct;
}

extern "C" mosaic_status mosaic_plan_validate(const mosaic_plan* p, int32_t cu_total, int32_t n_xcd) {
  if (!p || !p->cu_quota || !p->cu_offset) MOSAIC_FAIL(MOSAIC_EINVAL, "null plan");
  if (p->n <= 0 || p->n > MOSAIC_MAX_STAGE_MODULES) MOSAIC_FAIL(MOSAIC_EINVAL, "plan holds %d modules (1..%d allowed)", p->n, MOSAIC_MAX_STAGE_MODULES);
  if (p->mode != MOSAIC_COLOCATED && p->mode != MOSAIC_TIME_SLICED && p->mode != MOSAIC_CHAINED)
    MOSAIC_FAIL(MOSAIC_EINVAL, "bad plan mode %d", p->mode);
  std::vector<uint32_t> words((cu_total + 31) / 32);
  const int n_checked = (p->mode == MOSAIC_COLOCATED) ? p->n : 1;
  for (int i = 0; i < n_checked; ++i)
    MOSAIC_TRY(mosaic_cu_mask_build(cu_total, n_xcd, p->cu_quota[i], p->cu_offset[i], p->layout, words.data(), (int)words.size()));
  if (p->mode == MOSAIC_COLOCATED) {
    // Eq. 5: the quotas of the distinct streams fit on the GPU together, i.e. their CU ranges are disjoint
    int64_t total = 0;
    for (int i = 0; i < p->n; ++i) {
      bool first = true;
      for (int j = 0; j < i; ++j)
        if (p->cu_quota[j] == p->cu_quota[i] && p->cu_offset[j] == p->cu_offset[i]) first = false;
      if (!first) continue;
      total += p->cu_quota[i];
      for (int j = 0; j < i; ++j) {
        if (p->cu_quota[j] == p->cu_quota[i] && p->cu_offset[j] == p->cu_offset[i]) continue;
        const int a0 = p->cu_offset[i], a1 = a0 + p->cu_quota[i], b0 = p->cu_offset[j], b1 = b0 + p->cu_quota[j];
        if (a0 < b1 && b0 < a1)
          MOSAIC_FAIL(MOSAIC_EQUOTA, "modules %d and %d overlap: CU ranges [%d,%d) and [%d,%d)", j, i, b0, b1, a0, a1);
      }
    }
    if (total > cu_total) MOSAIC_FAIL(MOSAIC_EQUOTA, "quotas sum to %lld CUs, the device has %d", (long long)total, cu_total);
    // Every masked stream needs a hardware queue of its own to run beside the others; streams
    // that end up sharing one run one after the other, which silently turns a colocated stage
    // into a time-sliced one.
    const int distinct = mosaic_plan_stream_count(p);
    const int queues = mosaic_device_hw_queues();
    if (distinct > queues)
      MOSAIC_FAIL(MOSAIC_EQUOTA, "the plan needs %d streams side by side, the process has %d hardware queues "
                  "(GPU_MAX_HW_QUEUES): let modules share quotas, or split the stage", distinct, queues);
  }
  return MOSAIC_OK;
}

extern "C" mosaic_status mosaic_plan_choose(int32_t n_modules, int32_t n_points, const int32_t* cu_points,
                                            const float* times, int32_t cu_total, int32_t* quota_out, float* time_out) {
  if (!cu_points || !times || !quota_out) MOSAIC_FAIL(MOSAIC_EINVAL, "null argument");
  if (n_modules <= 0 || n_modules > MOSAIC_MAX_STAGE_MODULES || n_points <= 0) MOSAIC_FAIL(MOSAIC_EINVAL, "bad sizes");
  // order the candidate quotas ascending so that ties go to the smallest tuple
  std::vector<int> order(n_points);
  for (int i = 0; i < n_points; ++i) order[i] = i;
  for (int i = 1; i < n_points; ++i)
    for (int j = i; j > 0 && cu_points[order[j]] < cu_points[order[j - 1]]; --j) std::swap(order[j], order[j - 1]);
  std::vector<int> pick(n_modules, 0), best(n_modules, -1);
  float best_t = 0.f;
  bool found = false;
  // odometer over all n_points^n_modules assignments, most significant digit = module 0
  while (true) {
    int used = 0;
    float t = 0.f;
    for (int m = 0; m < n_modules; ++m) {
      used += cu_points[order[pick[m]]];
      const float tm = times[m * n_points + order[pick[m]]];
      if (tm > t) t = tm;
    }
    if (used <= cu_total && (!found || t < best_t)) { found = true; best_t = t; best = pick; }
    int m = n_modules - 1;
    while (m >= 0 && ++pick[m] == n_points) { pick[m] = 0; --m; }
    if (m < 0) break;
  }
  if (!found) MOSAIC_FAIL(MOSAIC_EQUOTA, "no combination of the offered quotas fits in %d CUs", cu_total);
  for (int m = 0; m < n_modules; ++m) quota_out[m] = cu_points[order[best[m]]];
  if (time_out) *time_out = best_t;
  return MOSAIC_OK;
}

// -------------------------------------------------------------------------- stage run
namespace {

// Events of one mosaic_stage_run call.  Calls may come from several host threads at once, so
// every call takes a set of its own from a free list (sets are created on first use and kept:
// event creation is not on the stage's critical path after the first iterations).
struct EventSet {
  hipEvent_t start = nullptr;
  hipEvent_t ms[MOSAIC_MAX_STAGE_MODULES] = {};
  hipEvent_t me[MOSAIC_MAX_STAGE_MODULES] = {};
};

std::mutex g_ev_mu;
std::vector<EventSet*> g_ev_free;

mosaic_status acquire_events(EventSet** out) {
  {
    std::lock_guard<std::mutex> lk(g_ev_mu);
    if (!g_ev_free.empty()) { *out = g_ev_free.back(); g_ev_free.pop_back(); return MOSAIC_OK; }
  }
  EventSet* ev = new (std::nothrow) EventSet();
  if (!ev) MOSAIC_FAIL(MOSAIC_ENOMEM, "host allocation failed");
  hipError_t e = hipEventCreate(&ev->start);
  for (int i = 0; i < MOSAIC_MAX_STAGE_MODULES && e == hipSuccess; ++i) {
    e = hipEventCreate(&ev->ms[i]);
    if (e == hipSuccess) e = hipEventCreate(&ev->me[i]);
  }
  if (e != hipSuccess) {
    if (ev->start) (void)hipEventDestroy(ev->start);
    for (int i = 0; i < MOSAIC_MAX_STAGE_MODULES; ++i) {
      if (ev->ms[i]) (void)hipEventDestroy(ev->ms[i]);
      if (ev->me[i]) (void)hipEventDestroy(ev->me[i]);
    }
    delete ev;
    MOSAIC_FAIL(MOSAIC_EHIP, "hipEventCreate failed: %s", hipGetErrorString(e));
  }
  *out = ev;
  return MOSAIC_OK;
}

struct EventLease {           // gives the set back when the call returns, on every path
  EventSet* ev = nullptr;
  ~EventLease() {
    if (!ev) return;
    std::lock_guard<std::mutex> lk(g_ev_mu);
    g_ev_free.push_back(ev);
  }
};

mosaic_status step_one(const mosaic_stage* st, int i, int quota, const mosaic_stream* s) {
  return mosaic_module_step(st->modules[i], quota, s, st->x[i], st->dy ? st->dy[i] : nullptr,
                            st->target ? st->target[i] : nullptr, st->y[i], st->dx ? st->dx[i] : nullptr,
                            st->loss ? st->loss[i] : nullptr);
}

}  // namespace

extern "C" mosaic_status mosaic_stage_run(const mosaic_stage* st, const mosaic_plan* plan, mosaic_timing* out) {
  if (!st || !plan) MOSAIC_FAIL(MOSAIC_EINVAL, "null stage or plan");
  if (!st->modules || !st->x || !st->y) MOSAIC_FAIL(MOSAIC_EINVAL, "stage arrays missing");
  if (st->n != plan->n) MOSAIC_FAIL(MOSAIC_EINVAL, "stage has %d modules, plan has %d", st->n, plan->n);
  DeviceInfo di;
  MOSAIC_TRY(mosaic_device_info(&di));
  MOSAIC_TRY(mosaic_plan_validate(plan, di.cu_count, di.xcd_count));
  const int n = st->n;
  for (int i = 0; i < n; ++i)
    if (!st->modules[i] || !st->x[i] || !st->y[i]) MOSAIC_FAIL(MOSAIC_EINVAL, "module %d: null module or buffer", i);
  // streams come from the pool only
  mosaic_stream* streams[MOSAIC_MAX_STAGE_MODULES];
  for (int i = 0; i < n; ++i) {
    const int k = (plan->mode == MOSAIC_COLOCATED) ? i : 0;
    MOSAIC_TRY(mosaic_pool_get(plan->cu_quota[k], plan->cu_offset[k], plan->layout, &streams[i]));
  }
  EventLease lease;
  MOSAIC_TRY(acquire_events(&lease.ev));
  EventSet* ev = lease.ev;
  mosaic_timing tm;
  memset(&tm, 0, sizeof(tm));

  if (plan->mode == MOSAIC_CHAINED) {
    for (int i = 0; i + 1 < n; ++i) {
      if (st->x[i + 1] != st->y[i]) MOSAIC_FAIL(MOSAIC_EINVAL, "chained stage: x[%d] must be y[%d]", i + 1, i);
      if (!st->dy || !st->dx || st->dy[i] != st->dx[i + 1]) MOSAIC_FAIL(MOSAIC_EINVAL, "chained stage: dy[%d] must be dx[%d]", i, i + 1);
    }
    if (!st->target || !st->target[n - 1] || !st->loss || !st->loss[n - 1])
      MOSAIC_FAIL(MOSAIC_EINVAL, "chained stage: the last module needs a target and a loss");
    const mosaic_stream* s = streams[0];
    const int q = s->quota;
    MOSAIC_HIP(hipEventRecord(ev->start, s->s));
    for (int i = 0; i + 1 < n; ++i) MOSAIC_TRY(mosaic_module_forward(st->modules[i], q, s, st->x[i], st->y[i]));
    MOSAIC_TRY(mosaic_module_step(st->modules[n - 1], q, s, st->x[n - 1], nullptr, st->target[n - 1], st->y[n - 1],
                                  st->dx[n - 1], st->loss[n - 1]));
    for (int i = n - 2; i >= 0; --i) MOSAIC_TRY(mosaic_module_backward(st->modules[i], q, s, st->dy[i], st->dx[i]));
    MOSAIC_HIP(hipEventRecord(ev->me[0], s->s));
    MOSAIC_HIP(hipEventSynchronize(ev->me[0]));
    MOSAIC_HIP(hipEventElapsedTime(&tm.stage_ms, ev->start, ev->me[0]));
    if (out) *out = tm;
    return MOSAIC_OK;
  }

  if (plan->mode == MOSAIC_TIME_SLICED) {
    const mosaic_stream* s = streams[0];
    MOSAIC_HIP(hipEventRecord(ev->start, s->s));
    for (int i = 0; i < n; ++i) {
      MOSAIC_HIP(hipEventRecord(ev->ms[i], s->s));
      MOSAIC_TRY(step_one(st, i, s->quota, s));
      MOSAIC_HIP(hipEventRecord(ev->me[i], s->s));
    }
    MOSAIC_HIP(hipEventSynchronize(ev->me[n - 1]));
    for (int i = 0; i < n; ++i) MOSAIC_HIP(hipEventElapsedTime(&tm.module_ms[i], ev->ms[i], ev->me[i]));
    MOSAIC_HIP(hipEventElapsedTime(&tm.stage_ms, ev->start, ev->me[n - 1]));
    if (out) *out = tm;
    return MOSAIC_OK;
  }

  // COLOCATED: modules that share a stream run back to back on it; distinct streams are
  // fed by one host thread each so that their kernels are enqueued side by side.  All
  // streams wait on a common start event.
  std::vector<mosaic_stream*> uniq;
  for (int i = 0; i < n; ++i) {
    bool seen = false;
    for (mosaic_stream* u : uniq) seen |= (u == streams[i]);
    if (!seen) uniq.push_back(streams[i]);
  }
  MOSAIC_HIP(hipEventRecord(ev->start, uniq[0]->s));
  for (size_t u = 1; u < uniq.size(); ++u) MOSAIC_HIP(hipStreamWaitEvent(uniq[u]->s, ev->start, 0));
  int dev = 0;
  MOSAIC_HIP(hipGetDevice(&dev));
  std::vector<mosaic_status> rc(uniq.size(), MOSAIC_OK);
  std::vector<std::string> msg(uniq.size());
  auto feed = [&](size_t u) {
    if (hipSetDevice(dev) != hipSuccess) { rc[u] = MOSAIC_EHIP; msg[u] = "hipSetDevice failed"; return; }
    for (int i = 0; i < n; ++i) {
      if (streams[i] != uniq[u]) continue;
      mosaic_status s1 = MOSAIC_OK;
      if (hipEventRecord(ev->ms[i], uniq[u]->s) != hipSuccess) s1 = MOSAIC_EHIP;
      if (s1 == MOSAIC_OK) s1 = step_one(st, i, uniq[u]->quota, uniq[u]);
      if (s1 == MOSAIC_OK && hipEventRecord(ev->me[i], uniq[u]->s) != hipSuccess) s1 = MOSAIC_EHIP;
      if (s1 != MOSAIC_OK) { rc[u] = s1; msg[u] = mosaic_last_error(); return; }
    }
  };
  std::vector<std::thread> workers;
  for (size_t u = 1; u < uniq.size(); ++u) workers.emplace_back(feed, u);
  feed(0);
  for (std::thread& w : workers) w.join();
  // whatever was enqueued must drain before returning, error or not
  for (mosaic_stream* u : uniq) MOSAIC_HIP(hipStreamSynchronize(u->s));
  for (size_t u = 0; u < uniq.size(); ++u)
    if (rc[u] != MOSAIC_OK) MOSAIC_FAIL(rc[u], "%s", msg[u].c_str());
  for (int i = 0; i < n; ++i) {
    MOSAIC_HIP(hipEventElapsedTime(&tm.module_ms[i], ev->ms[i], ev->me[i]));
    float t_end = 0.f;
    MOSAIC_HIP(hipEventElapsedTime(&t_end, ev->start, ev->me[i]));
    if (t_end > tm.stage_ms) tm.stage_ms = t_end;     // Eq. 4: the stage ends with its slowest module
  }
  if (out) *out = tm;
  return MOSAIC_OK;
}
