// Host side of the C ABI declared in swift_undo.h: argument validation, derived scalars in
// binary64, the planner that turns a tensor list into a device-resident chunk table (cached per
// distinct list), and the kernel launches.  One translation unit, built with hipcc for gfx950.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <exception>
#include <list>
#include <memory>
#include <mutex>
#include <new>
#include <string>
#include <unordered_map>
#include <vector>

#include "swift_undo.h"
#include "opt_kernels.hpp"
#include "digest_kernels.hpp"
#include "lamb_kernels.hpp"
#include "fused_kernels.hpp"
#include "logging_groups.hpp"

namespace swift {
namespace {

thread_local std::string g_last_error;

int fail(int code, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}

// No C++ exception may cross the C boundary: an entry point's body runs inside guarded().
template <typename F>
int guarded(F &&body) {
  try {
    return body();
  } catch (const std::bad_alloc &) {
    return fail(SWIFT_EHIP, "out of host memory");
  } catch (const std::exception &e) {
    return fail(SWIFT_EHIP, "internal error: %s", e.what());
  }
}

#define SWIFT_HIP(call)                                                                       \
  do {                                                                                        \
    hipError_t e_ = (call);                                                                   \
    if (e_ != hipSuccess)                                                                     \
      return fail(SWIFT_EHIP, "%s failed: %s (%s)", #call, hipGetErrorName(e_), hipGetErrorString(e_)); \
  } while (0)

long env_long(const char *name, long dflt) {
  const char *s = getenv(name);
  if (!s || !*s) return dflt;
  char *end = nullptr;
  long v = strtol(s, &end, 10);
  return (end && *end == 0) ? v : dflt;
}

// Tuning knobs.  They exist for sweeps: the defaults are the measured best.  The environment is read
// once, when the first call needs a knob; only a process started with SWIFT_TUNE=1 reads it again on
// every call (a sweep that changes the variables between calls).  kUnset = "use the built-in default".
constexpr long kUnset = -1;
struct Knobs {
  long tile_u, tile_block, waves_per_cu, chunk_elems, dmask_wgs_per_cu, dmask_queue, dmask_counters, dmask_queue_waves;
  long digest_chunk_elems, digest_waves_per_cu, copy_u, copy_waves_per_cu;
  long lamb_u1, lamb_u3, lamb_waves_p1, lamb_waves_p3, fused_u, fused_waves_per_cu;
  long max_grid;   // 0: none.  Tests set it to drive the kernels' strided loops, which only lists beyond 2^32 work-items reach
};

Knobs read_knobs() {
  Knobs k;
  k.tile_u = env_long("SWIFT_TILE_U", SWIFT_DEFAULT_U);
  k.tile_block = env_long("SWIFT_TILE_BLOCK", SWIFT_DEFAULT_BLOCK);
  k.waves_per_cu = env_long("SWIFT_WAVES_PER_CU", kUnset);
  k.chunk_elems = env_long("SWIFT_CHUNK_ELEMS", 0);
  k.dmask_wgs_per_cu = env_long("SWIFT_DMASK_WGS_PER_CU", SWIFT_DEFAULT_DMASK_WGS_PER_CU);
  k.dmask_queue = env_long("SWIFT_DMASK_QUEUE", SWIFT_DMASK_QUEUE);
  k.dmask_counters = env_long("SWIFT_DMASK_COUNTERS", SWIFT_DMASK_COUNTERS);
  k.dmask_queue_waves = env_long("SWIFT_DMASK_QUEUE_WAVES_PER_CU", SWIFT_DMASK_QUEUE_WAVES_PER_CU);
  k.digest_chunk_elems = env_long("SWIFT_DIGEST_CHUNK_ELEMS", 0);
  k.digest_waves_per_cu = env_long("SWIFT_DIGEST_WAVES_PER_CU", SWIFT_DIGEST_WAVES_PER_CU);
  k.copy_u = env_long("SWIFT_COPY_U", SWIFT_COPY_U);
  k.copy_waves_per_cu = env_long("SWIFT_COPY_WAVES_PER_CU", SWIFT_COPY_WAVES_PER_CU);
  k.lamb_u1 = env_long("SWIFT_LAMB_U1", SWIFT_LAMB_U1);
  k.lamb_u3 = env_long("SWIFT_LAMB_U3", SWIFT_LAMB_U3);
  k.lamb_waves_p1 = env_long("SWIFT_LAMB_WAVES_P1", SWIFT_LAMB_WAVES_P1);
  k.lamb_waves_p3 = env_long("SWIFT_LAMB_WAVES_P3", SWIFT_LAMB_WAVES_P3);
  k.fused_u = env_long("SWIFT_FUSED_U", SWIFT_FUSED_U);
  k.fused_waves_per_cu = env_long("SWIFT_FUSED_WAVES_PER_CU", SWIFT_FUSED_WAVES_PER_CU);
  k.max_grid = env_long("SWIFT_MAX_GRID", 0);
  return k;
}

Knobs knobs() {
  static const bool live = env_long("SWIFT_TUNE", 0) != 0;
  static const Knobs at_start = read_knobs();
  return live ? read_knobs() : at_start;
}

// ------------------------------------------------------------------------------------------
// Device facts, queried once per device.
struct DeviceInfo {
  int cus = 0;
  int lds_per_cu = 0;   // bytes
};

int device_info(int dev, DeviceInfo *out) {
  static std::mutex mu;
  static std::vector<DeviceInfo> cache;
  std::lock_guard<std::mutex> lock(mu);
  if ((int)cache.size() <= dev) cache.resize(dev + 1);
  if (cache[dev].cus == 0) {
    int cus = 0;
    SWIFT_HIP(hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev));
    if (cus <= 0) return fail(SWIFT_EHIP, "device %d reports %d compute units", dev, cus);
    int lds = 0;
    SWIFT_HIP(hipDeviceGetAttribute(&lds, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev));
    cache[dev].cus = cus;
    cache[dev].lds_per_cu = lds > 0 ? lds : 64 * 1024;
  }
  *out = cache[dev];
  return SWIFT_OK;
}

// ------------------------------------------------------------------------------------------
// Plans: descriptor table + chunk table in one device allocation, cached by the exact
// contents of the host arrays that produced them.
struct Plan {
  std::string key;
  int device = -1;
  void *dev_mem = nullptr;       // [descs | chunks]
  size_t desc_bytes = 0;
  uint32_t n_chunks = 0;
  uint32_t chunk_elems = 0;
  uint64_t n_out = 0;            // digest plans: number of outputs
  size_t dev_bytes = 0;          // device memory held by this plan (tables and scratch)
  bool pinned = false;           // used while a stream was capturing: a graph may replay it, never trimmed
  const void *probe_ptr = nullptr;   // first buffer of the list and the allocation it was found in when the
  const void *probe_base = nullptr;  // plan was built: looked up again on every later use (guarded by g_plan_mu)
  size_t probe_size = 0;
  // optimizer plans: where each tensor of the caller's list sits in the chunk table
  std::vector<uint64_t> t_first_chunk, t_numel;   // t_numel[i] = 0 for empty or unmarked tensors
  std::vector<uint8_t> t_active;
  // LAMB only, created on first use (guarded by lamb_mu): tensor spans and per-tile partial sums
  std::mutex lamb_mu;
  void *lamb_spans = nullptr;
  void *lamb_partial = nullptr;
  uint32_t lamb_tile_elems = 0;
  // fused step/undo + digest only, created on first use (guarded by lamb_mu): chunk spans, chunk sums, tile sums
  void *fused_spans = nullptr;
  void *fused_slots = nullptr;
  void *fused_tiles = nullptr;
  uint32_t fused_tile_elems = 0;
  // digest plans whose shards span several chunks: per-output spans and per-chunk sums (built with the plan)
  void *digest_spans = nullptr;
  void *digest_partial = nullptr;
  bool digest_has_empty = false;   // some output belongs to an empty buffer (its digest, 0, is written by a fill)
  // device-mask calls only, created on first use (guarded by lamb_mu): [tensor spans | packed chunk table | slot count]
  void *packed_mem = nullptr;
  size_t packed_table_off = 0, packed_count_off = 0;
  const void *descs() const { return dev_mem; }
  const void *chunks() const { return static_cast<const char *>(dev_mem) + desc_bytes; }
  ~Plan() {
    if (dev_mem) {
      int cur = -1;
      if (hipGetDevice(&cur) == hipSuccess && cur != device) (void)hipSetDevice(device);
      (void)hipFree(dev_mem);    // synchronises the device: no kernel still reads the table
      if (lamb_spans) (void)hipFree(lamb_spans);
      if (lamb_partial) (void)hipFree(lamb_partial);
      if (fused_spans) (void)hipFree(fused_spans);
      if (fused_slots) (void)hipFree(fused_slots);
      if (fused_tiles) (void)hipFree(fused_tiles);
      if (digest_spans) (void)hipFree(digest_spans);
      if (digest_partial) (void)hipFree(digest_partial);
      if (packed_mem) (void)hipFree(packed_mem);
      if (cur >= 0 && cur != device) (void)hipSetDevice(cur);
    }
  }
};

// The cache only grows: tables are freed by swift_cache_trim (the caller's decision) and by
// swift_shutdown, never as a side effect of another call.  A captured graph holds raw pointers into a
// plan's tables and scratch, so a plan that was used while its stream was capturing is pinned and
// survives every trim.
std::mutex g_plan_mu;
// Keys are the caller's pointer and size arrays verbatim (hundreds of kilobytes for a list of ten thousand
// tensors), compared in full on a hit.  Hashing all of that on every call would cost more than the comparison,
// so the hash looks at the length, both ends and 32 evenly spaced words: lists that differ elsewhere only share
// a bucket and are told apart by the comparison.
struct KeyHash {
  size_t operator()(const std::string &k) const noexcept {
    const size_t n = k.size();
    uint64_t h = 0x9E3779B97F4A7C15ull ^ (uint64_t)n;
    auto mix = [&h](uint64_t v) {
      h ^= v;
      h *= 0xD6E8FEB86659FD93ull;
      h ^= h >> 32;
    };
    auto word = [&k, n](size_t off) {
      uint64_t v = 0;
      memcpy(&v, k.data() + off, std::min<size_t>(8, n - off));
      return v;
    };
    if (n <= 512) {
      for (size_t off = 0; off < n; off += 8) mix(word(off));
    } else {
      for (size_t off = 0; off < 128; off += 8) mix(word(off));
      for (size_t off = n - 128; off < n; off += 8) mix(word(off));
      const size_t stride = (n / 32) & ~size_t(7);
      for (size_t j = 1; j < 32; ++j) mix(word(j * stride));
    }
    return (size_t)h;
  }
};
struct PlanCache {
  std::list<std::shared_ptr<Plan>> lru;                                               // most recently used first
  std::unordered_map<std::string, std::list<std::shared_ptr<Plan>>::iterator, KeyHash> index;  // key -> position in lru
};
PlanCache *g_plans = nullptr;   // leaked at exit on purpose: the HIP runtime may already be gone by then

std::shared_ptr<Plan> find_plan(const std::string &key) {
  std::lock_guard<std::mutex> lock(g_plan_mu);
  if (!g_plans) g_plans = new PlanCache();
  auto hit = g_plans->index.find(key);
  if (hit == g_plans->index.end()) return nullptr;
  g_plans->lru.splice(g_plans->lru.begin(), g_plans->lru, hit->second);   // iterators stay valid
  return *hit->second;
}

void keep_plan(const std::shared_ptr<Plan> &p) {
  std::shared_ptr<Plan> dropped;   // destroyed (hipFree) outside the lock
  std::lock_guard<std::mutex> lock(g_plan_mu);
  if (!g_plans) g_plans = new PlanCache();
  auto hit = g_plans->index.find(p->key);
  if (hit != g_plans->index.end()) {            // another thread built the same plan meanwhile: replace it
    dropped = *hit->second;
    g_plans->lru.erase(hit->second);
    g_plans->index.erase(hit);
  }
  g_plans->lru.push_front(p);
  g_plans->index[p->key] = g_plans->lru.begin();
}

// Takes one plan out of the cache (its tables are freed when the last reference goes).
void drop_plan(const std::shared_ptr<Plan> &p) {
  std::lock_guard<std::mutex> lock(g_plan_mu);
  if (!g_plans) return;
  auto hit = g_plans->index.find(p->key);
  if (hit == g_plans->index.end() || *hit->second != p) return;
  g_plans->lru.erase(hit->second);
  g_plans->index.erase(hit);
}

// Is `stream` recording a graph right now?  (The legacy default stream cannot.)
int stream_is_capturing(hipStream_t stream, bool *capturing) {
  *capturing = false;
  if (!stream) return SWIFT_OK;
  hipStreamCaptureStatus st = hipStreamCaptureStatusNone;
  SWIFT_HIP(hipStreamIsCapturing(stream, &st));
  *capturing = st != hipStreamCaptureStatusNone;
  return SWIFT_OK;
}

// The library may not allocate or copy synchronously while the caller's stream records a graph:
// whatever a call needs must exist before the capture begins.
int refuse_under_capture(hipStream_t stream, const char *what) {
  bool capturing = false;
  int rc = stream_is_capturing(stream, &capturing);
  if (rc) return rc;
  if (capturing)
    return fail(SWIFT_EINVAL, "the stream is capturing a graph and %s: make the same call once before the capture begins, "
                              "so that the library's tables for this tensor list exist", what);
  return SWIFT_OK;
}

// A cached plan is about to be used on `stream`.  It is pinned if the stream is capturing.  The first
// buffer of the list is looked up again: if the runtime no longer knows it, or finds it in another
// allocation than when the plan was built, the caller has freed and re-allocated its tensors, the
// cached validation is void and the plan is dropped (*stale = true; the caller rebuilds it).
int reuse_plan(const std::shared_ptr<Plan> &plan, hipStream_t stream, bool *stale) {
  *stale = false;
  if (plan->probe_ptr) {
    hipDeviceptr_t base = nullptr;
    size_t size = 0;
    const hipError_t e = hipMemGetAddressRange(&base, &size, const_cast<void *>(plan->probe_ptr));
    if (e != hipSuccess) (void)hipGetLastError();
    if (e != hipSuccess || base != plan->probe_base || size != plan->probe_size) {
      if (plan->pinned)
        return fail(SWIFT_EINVAL, "the tensors of a list that a captured graph uses were re-allocated");
      int rc = refuse_under_capture(stream, "the cached tables of this list are stale (its tensors were re-allocated)");
      if (rc) return rc;
      drop_plan(plan);
      *stale = true;
      return SWIFT_OK;
    }
  }
  if (!plan->pinned) {
    bool capturing = false;
    int rc = stream_is_capturing(stream, &capturing);
    if (rc) return rc;
    if (capturing) {
      std::lock_guard<std::mutex> lock(g_plan_mu);
      plan->pinned = true;
    }
  }
  return SWIFT_OK;
}

void set_probe(Plan &plan, const void *p) {
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  if (p && hipMemGetAddressRange(&base, &size, const_cast<void *>(p)) == hipSuccess) {
    plan.probe_ptr = p;
    plan.probe_base = base;
    plan.probe_size = size;
  } else {
    (void)hipGetLastError();
  }
}

template <typename T>
void key_add(std::string &k, const T &v) { k.append(reinterpret_cast<const char *>(&v), sizeof v); }

// No buffer of this library's callers can be longer (4 TiB of binary32); the bound keeps byte counts
// and chunk counts derived from a corrupt numel far away from integer overflow.
constexpr int64_t kMaxNumel = (int64_t)1 << 40;
constexpr int64_t kMaxTensors = ((int64_t)1 << 24) - 1;

// A device range [p, p + bytes) must lie inside one allocation of the current device.
int check_device_range(const void *p, size_t bytes, int dev, const char *what, int64_t idx) {
  hipPointerAttribute_t attr;
  hipError_t e = hipPointerGetAttributes(&attr, p);
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(SWIFT_EINVAL, "%s[%lld] = %p is not known to the HIP runtime (%s)", what, (long long)idx, p,
                hipGetErrorName(e));
  }
  if (attr.type != hipMemoryTypeDevice && attr.type != hipMemoryTypeManaged)
    return fail(SWIFT_EINVAL, "%s[%lld] = %p is not device memory", what, (long long)idx, p);
  if (attr.type == hipMemoryTypeDevice && attr.device != dev)
    return fail(SWIFT_EINVAL, "%s[%lld] = %p lives on device %d, current device is %d", what, (long long)idx, p,
                attr.device, dev);
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  e = hipMemGetAddressRange(&base, &size, const_cast<void *>(p));
  if (e != hipSuccess) {
    (void)hipGetLastError();
    return fail(SWIFT_EINVAL, "%s[%lld] = %p: cannot find its allocation (%s)", what, (long long)idx, p,
                hipGetErrorName(e));
  }
  const char *b = static_cast<const char *>(base), *q = static_cast<const char *>(p);
  if (q < b || q + bytes > b + size)
    return fail(SWIFT_EINVAL, "%s[%lld]: %zu bytes at %p run past the end of its allocation (%zu bytes at %p)", what,
                (long long)idx, bytes, p, size, base);
  return SWIFT_OK;
}

// Launch shape of the streaming kernels: U 16-byte vectors per lane, BLOCK lanes per workgroup,
// at most `waves_per_cu` wavefronts resident on a compute unit (0 = no cap).  The defaults come
// from sweeps on MI355X; the environment variables exist for such sweeps.
struct Tuning {
  int u, block, waves_per_cu;
};

// Which state streams an optimizer kind has: plain SGD (App. A) none, SGD with momentum m, the Adam family m and v.
bool kind_has_m(int kind) { return kind != SWIFT_SGD; }
bool kind_has_v(int kind) { return kind == SWIFT_ADAM || kind == SWIFT_ADAMW || kind == SWIFT_LAMB; }

Tuning opt_tuning(int kind, bool bf16, bool undo) {
  // Measured optima: the fewer bytes a wavefront moves (SGDM has 3 streams in and 2 out instead of
  // 4 and 3; bf16 gradients halve one stream), the more wavefronts a compute unit wants.
  (void)undo;      // step and undo want the same residency once every load of a tile is issued up front
  const int base = kind == SWIFT_SGD ? SWIFT_DEFAULT_WAVES_PER_CU_SGD
                 : kind == SWIFT_SGDM ? SWIFT_DEFAULT_WAVES_PER_CU_SGDM : SWIFT_DEFAULT_WAVES_PER_CU;
  // bf16 gradients: one more (plain SGD, where the gradient is half of what is read: four more, 6.72 TB/s at 28 against 6.60 at 24)
  const int waves = base + (bf16 ? (kind == SWIFT_SGD ? 4 : 1) : 0);
  const Knobs k = knobs();
  return Tuning{(int)k.tile_u, (int)k.tile_block, k.waves_per_cu == kUnset ? waves : (int)k.waves_per_cu};
}

// Dynamic LDS bytes per workgroup that make at most waves_per_cu wavefronts fit on one CU.
uint32_t lds_cap_bytes(const DeviceInfo &info, const Tuning &t) {
  const int wgs = t.waves_per_cu / (t.block / 64);
  if (t.waves_per_cu <= 0 || wgs >= 32) return 0;
  const int w = wgs < 3 ? 3 : wgs;                      // stay within the 64 KiB a launch may ask for
  uint32_t bytes = (uint32_t)(info.lds_per_cu / w) & ~511u;
  return bytes > 65536u ? 65536u : bytes;
}

// Workgroups of a launch over `items` work items, one each -- but a grid holds fewer than 2^32 work-items in
// all, so beyond that the grid is capped and the kernels, which all stride by the grid size, go round again.
// (64-lane workgroups: 67 M tiles, i.e. lists above 17 G elements.)
uint32_t grid_for(uint64_t items, uint32_t block) {
  uint64_t cap = 0xffffffffull / block;
  const long forced = knobs().max_grid;
  if (forced > 0) cap = std::min<uint64_t>(cap, (uint64_t)forced);
  return (uint32_t)std::min<uint64_t>(items, cap);
}

// Chunk length: a power of two that is a multiple of every compiled tile (at most 1,024 elements).
// Long chunks keep the table small; short ones waste fewer idle workgroups on the many tiny
// tensors of a small model.
constexpr uint32_t kMaxTileElems = 4096;
uint32_t pick_chunk_elems(uint64_t total_elems) {
  const long forced = knobs().chunk_elems;                     // tuning knob for sweeps
  if (forced >= (long)kMaxTileElems && forced <= (1l << 22) && (forced & (forced - 1)) == 0) return (uint32_t)forced;
  return total_elems >= (1ull << 28) ? 65536u : 16384u;
}

uint32_t shift_for(uint32_t tile_elems, uint32_t chunk_elems) {
  uint32_t s = 0;
  while ((tile_elems << s) < chunk_elems) ++s;
  return s;
}

int upload_plan(Plan &plan, const void *descs, size_t desc_bytes, const void *chunks, size_t n_chunks,
                size_t chunk_size) {
  plan.desc_bytes = (desc_bytes + 255) & ~size_t(255);
  const size_t total = plan.desc_bytes + std::max<size_t>(n_chunks, 1) * chunk_size;
  SWIFT_HIP(hipMalloc(&plan.dev_mem, total));
  plan.dev_bytes += total;
  // Synchronous copies: when they return the table is complete in device memory, so any stream
  // may read it.  This happens once per distinct tensor list.
  if (desc_bytes) SWIFT_HIP(hipMemcpy(plan.dev_mem, descs, desc_bytes, hipMemcpyHostToDevice));
  if (n_chunks)
    SWIFT_HIP(hipMemcpy(static_cast<char *>(plan.dev_mem) + plan.desc_bytes, chunks, n_chunks * chunk_size,
                        hipMemcpyHostToDevice));
  plan.n_chunks = (uint32_t)n_chunks;
  return SWIFT_OK;
}

// ------------------------------------------------------------------------------------------
// Optimizer calls.
struct Interval {
  uintptr_t lo, hi;
  bool written;
};

// Sorts the ranges by start address and checks that nothing that is written overlaps anything else.
// In order of start address, a range overlaps an earlier one iff it starts below the furthest end seen
// so far; gradients (read only) may overlap each other.
int check_no_overlap(Interval *iv, size_t n) {
  std::sort(iv, iv + n, [](const Interval &a, const Interval &b) { return a.lo < b.lo; });
  const Interval *far_any = nullptr, *far_written = nullptr;
  for (size_t k = 0; k < n; ++k) {
    const Interval &cur = iv[k];
    const Interval *hit = nullptr;
    if (far_written && cur.lo < far_written->hi) hit = far_written;
    else if (cur.written && far_any && cur.lo < far_any->hi) hit = far_any;
    if (hit)
      return fail(SWIFT_EINVAL, "buffers overlap: [%p, %p) and [%p, %p)", (void *)hit->lo, (void *)hit->hi, (void *)cur.lo,
                  (void *)cur.hi);
    if (!far_any || cur.hi > far_any->hi) far_any = &cur;
    if (cur.written && (!far_written || cur.hi > far_written->hi)) far_written = &cur;
  }
  return SWIFT_OK;
}

int validate_hparams(const swift_hparams *hp, bool undo, OptConsts *c) {
  if (!hp) return fail(SWIFT_EINVAL, "hparams is NULL");
  if (hp->kind < SWIFT_SGDM || hp->kind > SWIFT_SGD) return fail(SWIFT_EINVAL, "unknown optimizer kind %d", hp->kind);
  if (hp->grad_dtype != SWIFT_F32 && hp->grad_dtype != SWIFT_BF16)
    return fail(SWIFT_EINVAL, "unknown gradient dtype %d", hp->grad_dtype);
  if (hp->step < 1) return fail(SWIFT_EINVAL, "step must be >= 1 (got %lld)", (long long)hp->step);
  if (!std::isfinite(hp->lr)) return fail(SWIFT_EINVAL, "lr is not finite");
  if (!std::isfinite(hp->weight_decay) || hp->weight_decay < 0) return fail(SWIFT_EINVAL, "weight_decay must be finite and >= 0");
  if ((hp->flags & ~(int32_t)SWIFT_CLAMP_V) != 0 || hp->reserved != 0)
    return fail(SWIFT_EINVAL, "unknown flag bits 0x%x (reserved = %d)", (unsigned)hp->flags, hp->reserved);
  memset(c, 0, sizeof *c);
  c->clamp_v = (hp->flags & SWIFT_CLAMP_V) ? 1 : 0;
  c->eta = hp->lr;
  c->lam = hp->weight_decay;
  if (hp->kind == SWIFT_SGD) {                    // App. A "SGD" / "Undo SGD"
    const double oml = 1.0 - hp->lr * hp->weight_decay;
    if (undo && oml == 0) return fail(SWIFT_ENOTINVERTIBLE, "undo divides by 1 - lr*weight_decay = 0");
    c->inv_oml = oml != 0 ? 1.0 / oml : 0.0;
    return SWIFT_OK;
  }
  if (hp->kind == SWIFT_SGDM) {
    if (!(hp->momentum >= 0 && hp->momentum <= 1)) return fail(SWIFT_EINVAL, "momentum must be in [0, 1]");
    if (!(hp->dampening >= 0 && hp->dampening <= 1)) return fail(SWIFT_EINVAL, "dampening must be in [0, 1]");
    c->mu = hp->momentum;
    c->omt = 1.0 - hp->dampening;
    c->mu_is_zero = (hp->momentum == 0.0);
    c->inv_mu = c->mu_is_zero ? 0.0 : 1.0 / hp->momentum;
    return SWIFT_OK;
  }
  if (!(hp->beta1 >= 0 && hp->beta1 < 1) || !(hp->beta2 >= 0 && hp->beta2 < 1))
    return fail(SWIFT_EINVAL, "beta1 and beta2 must be in [0, 1)");
  if (!std::isfinite(hp->eps) || hp->eps < 0) return fail(SWIFT_EINVAL, "eps must be finite and >= 0");
  const double oml = 1.0 - hp->lr * hp->weight_decay;
  if (undo) {
    if (hp->beta1 == 0 || hp->beta2 == 0)
      return fail(SWIFT_ENOTINVERTIBLE, "undo divides by beta: beta1 = %g, beta2 = %g", hp->beta1, hp->beta2);
    if (hp->kind == SWIFT_ADAMW && oml == 0)
      return fail(SWIFT_ENOTINVERTIBLE, "undo divides by 1 - lr*weight_decay = 0");
  }
  c->b1 = hp->beta1;
  c->b2 = hp->beta2;
  c->c1 = 1.0 - hp->beta1;
  c->c2 = 1.0 - hp->beta2;
  c->inv_b1 = hp->beta1 != 0 ? 1.0 / hp->beta1 : 0.0;
  c->inv_b2 = hp->beta2 != 0 ? 1.0 / hp->beta2 : 0.0;
  c->rbc1 = 1.0 / (1.0 - std::pow(hp->beta1, (double)hp->step));   // t >= 1 and beta < 1: never 1/0
  c->rbc2 = 1.0 / (1.0 - std::pow(hp->beta2, (double)hp->step));
  c->eps = hp->eps;
  c->inv_oml = oml != 0 ? 1.0 / oml : 0.0;
  return SWIFT_OK;
}

int validate_list(const swift_tensor_list *l, const swift_hparams *hp) {
  if (!l) return fail(SWIFT_EINVAL, "tensor list is NULL");
  // (several launches take one 256-lane workgroup per tensor, and a grid holds fewer than 2^32 work-items)
  if (l->n < 0 || l->n > kMaxTensors) return fail(SWIFT_EINVAL, "tensor count %lld out of range (at most %lld)", (long long)l->n, (long long)kMaxTensors);
  if (l->n == 0) return SWIFT_OK;
  const bool hasm = kind_has_m(hp->kind), hasv = kind_has_v(hp->kind);
  if (!l->param || !l->grad || (hasm && !l->m) || !l->numel)
    return fail(SWIFT_EINVAL, "param, grad, m and numel arrays must not be NULL (m may be NULL for plain SGD only)");
  if (hasv && !l->v) return fail(SWIFT_EINVAL, "Adam/AdamW need the v array");
  const uintptr_t galign = hp->grad_dtype == SWIFT_BF16 ? 1 : 3;
  for (int64_t i = 0; i < l->n; ++i) {
    if (l->numel[i] < 0 || l->numel[i] > kMaxNumel)
      return fail(SWIFT_EINVAL, "numel[%lld] = %lld is negative or beyond 2^40", (long long)i, (long long)l->numel[i]);
    if (l->numel[i] == 0) continue;
    if (!l->param[i] || !l->grad[i] || (hasm && !l->m[i]) || (hasv && !l->v[i]))
      return fail(SWIFT_EINVAL, "tensor %lld has a NULL pointer", (long long)i);
    if (l->param_bf16 && (!l->param_bf16[i] || ((uintptr_t)l->param_bf16[i] & 1)))
      return fail(SWIFT_EINVAL, "tensor %lld: param_bf16 is NULL or not 2-byte aligned", (long long)i);
    if (((uintptr_t)l->param[i] & 3) || (hasm && ((uintptr_t)l->m[i] & 3)) || (hasv && ((uintptr_t)l->v[i] & 3)) ||
        ((uintptr_t)l->grad[i] & galign))
      return fail(SWIFT_EINVAL, "tensor %lld has a pointer that is not aligned to its element size", (long long)i);
  }
  return SWIFT_OK;
}

int build_opt_plan(const swift_tensor_list *l, const swift_hparams *hp, const uint8_t *host_mask, int dev,
                   hipStream_t stream, std::shared_ptr<Plan> *out) {
  const bool hasm = kind_has_m(hp->kind), hasv = kind_has_v(hp->kind);
  const bool bf16 = hp->grad_dtype == SWIFT_BF16;
  const bool hasxb = l->param_bf16 != nullptr;
  // header, then per tensor: numel, mask byte, the pointers (zero for an empty tensor, whose pointers are never read)
  const size_t per_tensor = 8 + 1 + 8 * (2 + (hasm ? 1 : 0) + (hasv ? 1 : 0) + (hasxb ? 1 : 0));
  std::string key(32 + (size_t)l->n * per_tensor, '\0');
  char *kp = &key[0];
  auto put = [&kp](const auto &v) {
    memcpy(kp, &v, sizeof v);
    kp += sizeof v;
  };
  put((uint8_t)'O');
  put((uint8_t)((hasv ? 1 : 0) | (hasm ? 2 : 0)));
  put((uint8_t)bf16);
  put((uint8_t)hasxb);
  put((int32_t)dev);
  put((int64_t)l->n);
  put((int64_t)knobs().chunk_elems);
  kp = &key[32];
  for (int64_t i = 0; i < l->n; ++i) {
    const int64_t n = l->numel[i];
    put(n);
    put((uint8_t)(host_mask ? (host_mask[i] != 0) : 1));
    const bool live = n != 0;
    put(live ? (const void *)l->param[i] : nullptr);
    put(live ? l->grad[i] : nullptr);
    if (hasm) put(live ? (const void *)l->m[i] : nullptr);
    if (hasv) put(live ? (const void *)l->v[i] : nullptr);
    if (hasxb) put(live ? (const void *)l->param_bf16[i] : nullptr);
  }
  if (auto hit = find_plan(key)) {
    bool stale = false;
    int rc = reuse_plan(hit, stream, &stale);
    if (rc) return rc;
    if (!stale) {
      *out = hit;
      return SWIFT_OK;
    }
  }

  // Miss: check every pointer against the runtime's allocation records, check that nothing that
  // is written overlaps anything else, then build and upload the chunk table (an allocation and
  // synchronous copies: not while the stream records a graph).
  {
    int rc = refuse_under_capture(stream, "this tensor list has not been used before");
    if (rc) return rc;
  }
  std::vector<Interval> iv;
  iv.reserve((size_t)l->n * 4);
  uint64_t total = 0;
  const size_t gsz = bf16 ? 2 : 4;
  for (int64_t i = 0; i < l->n; ++i) {
    const uint64_t n = (uint64_t)l->numel[i];
    if (n == 0) continue;
    int rc;
    if ((rc = check_device_range(l->param[i], n * 4, dev, "param", i))) return rc;
    if ((rc = check_device_range(l->grad[i], n * gsz, dev, "grad", i))) return rc;
    if (hasm && (rc = check_device_range(l->m[i], n * 4, dev, "m", i))) return rc;
    if (hasv && (rc = check_device_range(l->v[i], n * 4, dev, "v", i))) return rc;
    if (hasxb && (rc = check_device_range(l->param_bf16[i], n * 2, dev, "param_bf16", i))) return rc;
    if (hasxb) iv.push_back({(uintptr_t)l->param_bf16[i], (uintptr_t)l->param_bf16[i] + n * 2, true});
    const uintptr_t x = (uintptr_t)l->param[i], g = (uintptr_t)l->grad[i];
    iv.push_back({x, x + n * 4, true});
    iv.push_back({g, g + n * gsz, false});
    if (hasm) iv.push_back({(uintptr_t)l->m[i], (uintptr_t)l->m[i] + n * 4, true});
    if (hasv) iv.push_back({(uintptr_t)l->v[i], (uintptr_t)l->v[i] + n * 4, true});
    if (!host_mask || host_mask[i]) total += n;
  }
  if (int rc = check_no_overlap(iv.data(), iv.size())) return rc;

  auto plan = std::make_shared<Plan>();
  plan->key = std::move(key);
  plan->device = dev;
  plan->chunk_elems = pick_chunk_elems(total);
  const uint64_t ce = plan->chunk_elems;
  std::vector<ChunkDesc> chunks;
  chunks.reserve((size_t)(total / ce) + (size_t)l->n);
  plan->t_first_chunk.assign((size_t)l->n, 0);
  plan->t_numel.assign((size_t)l->n, 0);
  plan->t_active.assign((size_t)l->n, 0);
  for (int64_t i = 0; i < l->n; ++i) {
    if (host_mask && !host_mask[i]) continue;
    plan->t_active[(size_t)i] = 1;
    plan->t_first_chunk[(size_t)i] = chunks.size();
    const uint64_t n = (uint64_t)l->numel[i];
    if (n == 0) continue;
    plan->t_numel[(size_t)i] = n;
    char *x = static_cast<char *>(l->param[i]), *m = hasm ? static_cast<char *>(l->m[i]) : nullptr;
    char *v = hasv ? static_cast<char *>(l->v[i]) : nullptr;
    const char *g = static_cast<const char *>(l->grad[i]);
    char *xb = hasxb ? static_cast<char *>(l->param_bf16[i]) : nullptr;
    const uintptr_t bits = (uintptr_t)x | (uintptr_t)m | (uintptr_t)v;
    const uint32_t vec_ok = ((bits & 15) == 0) && (((uintptr_t)g & (bf16 ? 7 : 15)) == 0) && (((uintptr_t)xb & 7) == 0);
    for (uint64_t off = 0; off < n; off += ce) {
      ChunkDesc d;
      d.x = reinterpret_cast<float *>(x + off * 4);
      d.g = g + off * gsz;
      d.m = hasm ? reinterpret_cast<float *>(m + off * 4) : nullptr;
      d.v = hasv ? reinterpret_cast<float *>(v + off * 4) : nullptr;
      d.xb = hasxb ? reinterpret_cast<uint16_t *>(xb + off * 2) : nullptr;
      d.pad = 0;
      d.len = (uint32_t)std::min<uint64_t>(ce, n - off);
      d.tensor = (uint32_t)i;
      d.vec_ok = vec_ok;
      d.elem0 = (uint32_t)off;
      chunks.push_back(d);
    }
  }
  if (chunks.size() > 0x7fffffffull) return fail(SWIFT_EINVAL, "tensor list is too large");
  int rc = upload_plan(*plan, nullptr, 0, chunks.data(), chunks.size(), sizeof(ChunkDesc));
  if (rc) return rc;
  for (int64_t i = 0; i < l->n && !plan->probe_ptr; ++i)
    if (l->numel[i] > 0) set_probe(*plan, l->param[i]);
  keep_plan(plan);
  *out = plan;
  return SWIFT_OK;
}

typedef void (*OptKernel)(const ChunkDesc *, uint64_t, uint32_t, const OptConsts);
typedef void (*OptPackedKernel)(const ChunkDesc *, const uint64_t *, uint32_t, const OptConsts);
typedef void (*OptQueueKernel)(const ChunkDesc *, const uint64_t *, uint32_t, const OptConsts, unsigned int *, uint32_t);
constexpr long kQueueMaxCounters = 256;               // = kThreads: compact_chunks_kernel clears them with one workgroup
constexpr size_t kQueueCounterBytes = kQueueMaxCounters * 128;      // tile counters, 128 bytes apart, behind the slot count

#define SWIFT_PICK_KIND(KERNEL, U_, B_)                                                                        \
  switch (kind) {                                                                                              \
    case SWIFT_SGD: return SWIFT_PICK_FLAGS(KERNEL, kSGD, U_, B_);                                             \
    case SWIFT_SGDM: return SWIFT_PICK_FLAGS(KERNEL, kSGDM, U_, B_);                                           \
    case SWIFT_ADAM: return SWIFT_PICK_FLAGS(KERNEL, kADAM, U_, B_);                                           \
    default: return SWIFT_PICK_FLAGS(KERNEL, kADAMW, U_, B_);                                                  \
  }
#define SWIFT_PICK_FLAGS(KERNEL, K, U_, B_)                                                                    \
  (undo ? (bf16 ? SWIFT_PICK_XB(KERNEL, K, true, true, U_, B_) : SWIFT_PICK_XB(KERNEL, K, true, false, U_, B_)) \
        : (bf16 ? SWIFT_PICK_XB(KERNEL, K, false, true, U_, B_) : SWIFT_PICK_XB(KERNEL, K, false, false, U_, B_)))
#define SWIFT_PICK_XB(KERNEL, K, UNDO_, BF_, U_, B_) \
  (xb ? KERNEL<K, UNDO_, BF_, true, U_, B_> : KERNEL<K, UNDO_, BF_, false, U_, B_>)

template <int U, int BLOCK>
OptKernel pick_kernel_shape(int kind, bool undo, bool bf16, bool xb) {
  SWIFT_PICK_KIND(opt_kernel, U, BLOCK)
}

// The launch shapes that are compiled in.  Returns nullptr for any other (U, BLOCK).
OptKernel pick_kernel(const Tuning &t, int kind, bool undo, bool bf16, bool xb) {
#define SWIFT_SHAPE(U_, B_) if (t.u == U_ && t.block == B_) return pick_kernel_shape<U_, B_>(kind, undo, bf16, xb);
  SWIFT_SHAPES(SWIFT_SHAPE)
#undef SWIFT_SHAPE
  return nullptr;
}

// Device-mask launches always use the default shape.
OptPackedKernel pick_packed_kernel(int kind, bool undo, bool bf16, bool xb) {
  SWIFT_PICK_KIND(opt_packed_kernel, SWIFT_DEFAULT_U, SWIFT_DEFAULT_BLOCK)
}
OptQueueKernel pick_queue_kernel(int kind, bool undo, bool bf16, bool xb) {
  SWIFT_PICK_KIND(opt_queue_kernel, SWIFT_DEFAULT_U, SWIFT_DEFAULT_BLOCK)
}
#undef SWIFT_PICK_KIND
#undef SWIFT_PICK_FLAGS
#undef SWIFT_PICK_XB

// Scratch of the device-mask calls: where each tensor's chunks sit, room for the packed table and
// its slot count.  Calls that share a plan (the same tensors) share it, like the tensors themselves.
int packed_prepare(Plan &plan, hipStream_t stream) {
  std::lock_guard<std::mutex> lock(plan.lamb_mu);
  if (plan.packed_mem) return SWIFT_OK;
  if (int rc = refuse_under_capture(stream, "this tensor list has not been used with a device mask before")) return rc;
  std::vector<TensorChunks> spans(plan.t_numel.size());
  for (size_t i = 0; i < spans.size(); ++i) {
    spans[i].first = (uint32_t)plan.t_first_chunk[i];
    spans[i].count = (uint32_t)((plan.t_numel[i] + plan.chunk_elems - 1) / plan.chunk_elems);
  }
  const size_t table_off = (spans.size() * sizeof(TensorChunks) + 255) & ~size_t(255);
  const size_t count_off = table_off + std::max<size_t>(plan.n_chunks, 1) * sizeof(ChunkDesc);
  void *mem = nullptr;
  SWIFT_HIP(hipMalloc(&mem, count_off + 256 + kQueueCounterBytes));
  hipError_t e = hipMemcpy(mem, spans.data(), spans.size() * sizeof(TensorChunks), hipMemcpyHostToDevice);
  if (e != hipSuccess) {
    (void)hipFree(mem);
    return fail(SWIFT_EHIP, "device-mask scratch upload failed: %s", hipGetErrorName(e));
  }
  plan.packed_table_off = table_off;
  plan.packed_count_off = count_off;
  plan.packed_mem = mem;
  plan.dev_bytes += count_off + 256 + kQueueCounterBytes;
  return SWIFT_OK;
}

// An optimizer call in two halves: everything that can fail for a reason of the caller's making
// (arguments, pointers, tables) happens in opt_prepare, which enqueues nothing; opt_launch then
// enqueues the kernels.  The tracker puts its stream wait between the two.
struct OptLaunch {
  OptConsts c;
  DeviceInfo info;
  Tuning tune;
  OptKernel kernel = nullptr;
  OptPackedKernel packed_kernel = nullptr;
  OptQueueKernel queue_kernel = nullptr;
  std::shared_ptr<Plan> plan;
  const uint8_t *device_mask = nullptr;
  uint32_t n_tensors = 0, tpc_shift = 0;
  uint64_t n_slots = 0;
  bool empty = true;               // nothing to launch
};

int opt_prepare(const swift_tensor_list *l, const swift_hparams *hp, const uint8_t *host_mask,
                const uint8_t *device_mask, bool want_dmask, bool undo, hipStream_t stream, OptLaunch *out) {
  int rc = validate_hparams(hp, undo, &out->c);
  if (rc) return rc;
  if (hp->kind == SWIFT_LAMB)
    return fail(SWIFT_EINVAL, "LAMB needs the saved norms: use swift_lamb_step / swift_lamb_undo");
  if ((rc = validate_list(l, hp))) return rc;
  if (want_dmask && !device_mask && l->n > 0) return fail(SWIFT_EINVAL, "device mask is NULL");
  if (l->n == 0) return SWIFT_OK;
  int dev = -1;
  SWIFT_HIP(hipGetDevice(&dev));
  if ((rc = device_info(dev, &out->info))) return rc;
  const bool bf16 = hp->grad_dtype == SWIFT_BF16, xb = l->param_bf16 != nullptr;
  out->tune = opt_tuning(hp->kind, bf16, undo);
  if (want_dmask) out->tune.u = SWIFT_DEFAULT_U, out->tune.block = SWIFT_DEFAULT_BLOCK;     // the only packed-table shape
  out->kernel = pick_kernel(out->tune, hp->kind, undo, bf16, xb);
  if (!out->kernel)
    return fail(SWIFT_EINVAL, "launch shape U=%d BLOCK=%d is not compiled in", out->tune.u, out->tune.block);
  const uint32_t tile_elems = (uint32_t)out->tune.u * (uint32_t)out->tune.block * 4u;
  if (want_dmask && (rc = check_device_range(device_mask, (size_t)l->n, dev, "device_mask", 0))) return rc;
  if ((rc = build_opt_plan(l, hp, host_mask, dev, stream, &out->plan))) return rc;
  if (out->plan->n_chunks == 0) return SWIFT_OK;
  out->tpc_shift = shift_for(tile_elems, out->plan->chunk_elems);
  out->n_slots = (uint64_t)out->plan->n_chunks << out->tpc_shift;
  out->n_tensors = (uint32_t)l->n;
  if (want_dmask) {
    if ((rc = packed_prepare(*out->plan, stream))) return rc;
    out->packed_kernel = pick_packed_kernel(hp->kind, undo, bf16, xb);
    out->queue_kernel = pick_queue_kernel(hp->kind, undo, bf16, xb);
    out->device_mask = device_mask;
  }
  out->empty = false;
  return SWIFT_OK;
}

// The update over a packed table, for both device-mask entry points.  Queue mode: a resident grid
// (as many wavefronts as the residency cap lets a CU hold) that draws tiles from counters; strided
// mode: one workgroup per slot up to a cap, striding beyond it.
int launch_packed(OptPackedKernel packed_kernel, OptQueueKernel queue_kernel, const DeviceInfo &info, const Tuning &tune,
                  uint64_t n_slots, uint32_t tpc_shift, const OptConsts &c, const ChunkDesc *packed, const uint64_t *count,
                  unsigned int *counters, uint32_t log2c, hipStream_t stream) {
  const Knobs kn = knobs();
  if (kn.dmask_queue) {
    Tuning qt = tune;
    qt.waves_per_cu = (int)kn.dmask_queue_waves;
    const uint64_t resident = (uint64_t)info.cus * (uint64_t)std::max(qt.waves_per_cu, 1);
    hipLaunchKernelGGL(queue_kernel, dim3((uint32_t)std::min<uint64_t>(n_slots, resident)), dim3((uint32_t)tune.block),
                       lds_cap_bytes(info, qt), stream, packed, count, tpc_shift, c, counters, log2c);
    SWIFT_HIP(hipGetLastError());
    return SWIFT_OK;
  }
  uint64_t grid_cap = 0xffffffffull / (uint64_t)tune.block;
  if (kn.dmask_wgs_per_cu > 0) grid_cap = (uint64_t)info.cus * (uint64_t)kn.dmask_wgs_per_cu;
  hipLaunchKernelGGL(packed_kernel, dim3((uint32_t)std::min<uint64_t>(n_slots, grid_cap)), dim3((uint32_t)tune.block),
                     lds_cap_bytes(info, tune), stream, packed, count, tpc_shift, c);
  SWIFT_HIP(hipGetLastError());
  return SWIFT_OK;
}

int opt_launch(const OptLaunch &L, hipStream_t stream) {
  if (L.empty) return SWIFT_OK;
  const Plan &plan = *L.plan;
  const ChunkDesc *table = static_cast<const ChunkDesc *>(plan.chunks());
  if (!L.packed_kernel) {
    hipLaunchKernelGGL(L.kernel, dim3(grid_for(L.n_slots, (uint32_t)L.tune.block)), dim3((uint32_t)L.tune.block),
                       lds_cap_bytes(L.info, L.tune), stream, table, L.n_slots, L.tpc_shift, L.c);
    SWIFT_HIP(hipGetLastError());
    return SWIFT_OK;
  }
  // The host cannot size the grid to the marked tensors, and a workgroup that finds nothing to do
  // still costs a dispatch (0.2-0.3 ns) plus the latency of the table fetch it needed to find that
  // out.  So a small kernel first packs the chunk table by the mask, entirely on the device, and
  // leaves the slot count beside it (and clears the tile counters); the update kernel then runs
  // over the packed table and stops at that count, so every tile it takes is a marked one
  // (launch_packed: resident wavefronts that draw tiles from the counters, or a capped strided grid).
  char *pm = static_cast<char *>(plan.packed_mem);
  ChunkDesc *packed = reinterpret_cast<ChunkDesc *>(pm + plan.packed_table_off);
  uint64_t *count = reinterpret_cast<uint64_t *>(pm + plan.packed_count_off);
  unsigned int *counters = reinterpret_cast<unsigned int *>(pm + plan.packed_count_off + 256);
  const Knobs kn = knobs();
  uint32_t log2c = 0;
  while ((2u << log2c) <= (uint32_t)std::min<long>(std::max<long>(kn.dmask_counters, 1), kQueueMaxCounters)) ++log2c;
  hipLaunchKernelGGL(compact_chunks_kernel, dim3(L.n_tensors), dim3(kThreads), 0, stream, table,
                     reinterpret_cast<const TensorChunks *>(pm), L.n_tensors, L.device_mask, L.tpc_shift, packed, count,
                     counters, 1u << log2c);
  SWIFT_HIP(hipGetLastError());
  return launch_packed(L.packed_kernel, L.queue_kernel, L.info, L.tune, L.n_slots, L.tpc_shift, L.c, packed, count, counters,
                       log2c, stream);
}

int opt_call(const swift_tensor_list *l, const swift_hparams *hp, const uint8_t *host_mask,
             const uint8_t *device_mask, bool want_dmask, bool undo, void *stream_) {
  const hipStream_t stream = static_cast<hipStream_t>(stream_);
  OptLaunch L;
  int rc = opt_prepare(l, hp, host_mask, device_mask, want_dmask, undo, stream, &L);
  if (rc) return rc;
  return opt_launch(L, stream);
}

// ------------------------------------------------------------------------------------------
// swift_opt_undo_dmask_noalloc: the device-mask undo for callers that cannot allocate.  Chunk table,
// tensor spans, packed table and slot count live in one file-scope device array instead of per-list
// allocations; the chunk table is written by a kernel from descriptors that travel in its arguments
// (no host-to-device copy), so the call consists of kernel launches only.
constexpr int64_t kNoallocMaxTensors = SWIFT_NOALLOC_MAX_TENSORS;
constexpr int64_t kNoallocMaxChunks = SWIFT_NOALLOC_MAX_CHUNKS;
constexpr size_t kNoallocTableOff = 0;
constexpr size_t kNoallocPackedOff = kNoallocTableOff + (size_t)kNoallocMaxChunks * sizeof(ChunkDesc);
constexpr size_t kNoallocSpansOff = kNoallocPackedOff + (size_t)kNoallocMaxChunks * sizeof(ChunkDesc);
constexpr size_t kNoallocCountOff = kNoallocSpansOff + (size_t)kNoallocMaxTensors * sizeof(TensorChunks);
constexpr size_t kNoallocBytes = kNoallocCountOff + 256 + kQueueCounterBytes;

// Every GPU the library runs on holds its own copy of this array until the process ends.  In host
// code the name is only a handle for hipGetSymbolAddress; kernels get the address that call returned.
static __device__ __align__(256) unsigned char scratch[kNoallocBytes];

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices] = {};

// Address of `scratch` on device `dev`, which must be the current device; looked up once per device.
int scratch_for_device(int dev, void **out) {
  if (dev < 0 || dev >= kMaxDevices) return fail(SWIFT_EINVAL, "device %d is beyond the %d devices this entry point serves", dev, kMaxDevices);
  std::lock_guard<std::mutex> lock(g_scratch_mu);
  if (!g_scratch_ptr[dev]) {
    void *ptr = nullptr;
    SWIFT_HIP(hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)));
    if (!ptr) return fail(SWIFT_EHIP, "hipGetSymbolAddress returned a null address for the scratch array");
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return SWIFT_OK;
}

// Up to kExpandBatch tensors per launch travel by value in the kernel arguments (under the 4 KiB limit).
constexpr int kExpandBatch = 48;
struct ExpandTensor {
  float *x;
  const void *g;
  float *m;
  float *v;
  uint64_t numel;
  uint32_t first_chunk;      // position of the tensor's first chunk in the table
  uint32_t vec_ok;
};
struct ExpandBatch {
  ExpandTensor t[kExpandBatch];
  uint32_t first_tensor;     // index of t[0] in the caller's list
  uint32_t count;
  uint32_t chunk_elems;
  uint32_t g_elem_bytes;     // 4 (binary32 gradients) or 2 (bfloat16)
};

// One workgroup per tensor of the batch: writes the tensor's chunk entries and its span.
__global__ void __launch_bounds__(kThreads)
expand_chunks_kernel(const ExpandBatch b, ChunkDesc *__restrict__ table, TensorChunks *__restrict__ spans) {
  if (blockIdx.x >= b.count) return;
  const ExpandTensor t = b.t[blockIdx.x];
  const uint64_t ce = b.chunk_elems;
  const uint32_t n_chunks = (uint32_t)((t.numel + ce - 1) / ce);
  for (uint32_t k = threadIdx.x; k < n_chunks; k += kThreads) {
    const uint64_t off = (uint64_t)k * ce;
    const uint64_t left = t.numel - off;
    ChunkDesc d;
    d.x = t.x + off;
    d.g = static_cast<const char *>(t.g) + off * b.g_elem_bytes;
    d.m = t.m ? t.m + off : nullptr;
    d.v = t.v ? t.v + off : nullptr;
    d.xb = nullptr;
    d.len = (uint32_t)(left < ce ? left : ce);
    d.tensor = b.first_tensor + blockIdx.x;
    d.vec_ok = t.vec_ok;
    d.elem0 = (uint32_t)off;
    d.pad = 0;
    table[t.first_chunk + k] = d;
  }
  if (threadIdx.x == 0) spans[b.first_tensor + blockIdx.x] = TensorChunks{t.first_chunk, n_chunks};
}

// Host-side work areas of the entry point (no heap use on the call path); guarded by g_noalloc_mu.
std::mutex g_noalloc_mu;
Interval g_noalloc_iv[kNoallocMaxTensors * 4];

int noalloc_undo_dmask(const swift_tensor_list *l, const swift_hparams *hp, const uint8_t *device_mask, void *stream_) {
  OptConsts c;
  int rc = validate_hparams(hp, true, &c);
  if (rc) return rc;
  if (hp->kind == SWIFT_LAMB) return fail(SWIFT_EINVAL, "LAMB needs the saved norms: use swift_lamb_undo");
  if ((rc = validate_list(l, hp))) return rc;
  if (l->n == 0) return SWIFT_OK;
  if (l->param_bf16) return fail(SWIFT_EINVAL, "swift_opt_undo_dmask_noalloc does not take param_bf16");
  if (!device_mask) return fail(SWIFT_EINVAL, "device mask is NULL");
  if (l->n > kNoallocMaxTensors)
    return fail(SWIFT_EINVAL, "swift_opt_undo_dmask_noalloc takes at most %lld tensors per call (got %lld)",
                (long long)kNoallocMaxTensors, (long long)l->n);
  uint64_t total = 0;
  for (int64_t i = 0; i < l->n; ++i) total += (uint64_t)l->numel[i];
  // the shortest chunk length (a power of two, at least the small-list length) whose table fits
  uint32_t ce = 16384;
  auto chunks_at = [&](uint64_t len) {
    uint64_t n = 0;
    for (int64_t i = 0; i < l->n; ++i) n += ((uint64_t)l->numel[i] + len - 1) / len;
    return n;
  };
  while (ce < (1u << 22) && chunks_at(ce) > (uint64_t)kNoallocMaxChunks) ce *= 2;
  if (chunks_at(ce) > (uint64_t)kNoallocMaxChunks)
    return fail(SWIFT_EINVAL, "swift_opt_undo_dmask_noalloc: %llu elements in %lld tensors need more than %lld chunks of "
                "%u elements; split the list", (unsigned long long)total, (long long)l->n, (long long)kNoallocMaxChunks, ce);
  int dev = -1;
  SWIFT_HIP(hipGetDevice(&dev));
  DeviceInfo info;
  if ((rc = device_info(dev, &info))) return rc;
  void *base = nullptr;
  if ((rc = scratch_for_device(dev, &base))) return rc;
  const bool bf16 = hp->grad_dtype == SWIFT_BF16, hasm = kind_has_m(hp->kind), hasv = kind_has_v(hp->kind);
  const size_t gsz = bf16 ? 2 : 4;
  if ((rc = check_device_range(device_mask, (size_t)l->n, dev, "device_mask", 0))) return rc;
  std::lock_guard<std::mutex> lock(g_noalloc_mu);
  size_t n_iv = 0;
  for (int64_t i = 0; i < l->n; ++i) {
    const uint64_t n = (uint64_t)l->numel[i];
    if (n == 0) continue;
    if ((rc = check_device_range(l->param[i], n * 4, dev, "param", i))) return rc;
    if ((rc = check_device_range(l->grad[i], n * gsz, dev, "grad", i))) return rc;
    if (hasm && (rc = check_device_range(l->m[i], n * 4, dev, "m", i))) return rc;
    if (hasv && (rc = check_device_range(l->v[i], n * 4, dev, "v", i))) return rc;
    const uintptr_t x = (uintptr_t)l->param[i], g = (uintptr_t)l->grad[i];
    g_noalloc_iv[n_iv++] = {x, x + n * 4, true};
    g_noalloc_iv[n_iv++] = {g, g + n * gsz, false};
    if (hasm) g_noalloc_iv[n_iv++] = {(uintptr_t)l->m[i], (uintptr_t)l->m[i] + n * 4, true};
    if (hasv) g_noalloc_iv[n_iv++] = {(uintptr_t)l->v[i], (uintptr_t)l->v[i] + n * 4, true};
  }
  if ((rc = check_no_overlap(g_noalloc_iv, n_iv))) return rc;

  char *sb = static_cast<char *>(base);
  ChunkDesc *table = reinterpret_cast<ChunkDesc *>(sb + kNoallocTableOff);
  ChunkDesc *packed = reinterpret_cast<ChunkDesc *>(sb + kNoallocPackedOff);
  TensorChunks *spans = reinterpret_cast<TensorChunks *>(sb + kNoallocSpansOff);
  uint64_t *count = reinterpret_cast<uint64_t *>(sb + kNoallocCountOff);
  const hipStream_t stream = static_cast<hipStream_t>(stream_);
  Tuning tune = opt_tuning(hp->kind, bf16, true);
  tune.u = SWIFT_DEFAULT_U, tune.block = SWIFT_DEFAULT_BLOCK;
  const uint32_t tile_elems = (uint32_t)tune.u * (uint32_t)tune.block * 4u;
  const uint32_t tpc_shift = shift_for(tile_elems, ce);

  // 1. the chunk table and the spans, written on the device from by-value descriptors
  ExpandBatch batch;
  uint32_t next_chunk = 0;
  for (int64_t i0 = 0; i0 < l->n; i0 += kExpandBatch) {
    const int64_t cnt = std::min<int64_t>(kExpandBatch, l->n - i0);
    memset(&batch, 0, sizeof batch);
    batch.first_tensor = (uint32_t)i0;
    batch.count = (uint32_t)cnt;
    batch.chunk_elems = ce;
    batch.g_elem_bytes = (uint32_t)gsz;
    for (int64_t k = 0; k < cnt; ++k) {
      const int64_t i = i0 + k;
      ExpandTensor &t = batch.t[k];
      t.numel = (uint64_t)l->numel[i];
      t.first_chunk = next_chunk;
      if (t.numel) {
        t.x = static_cast<float *>(l->param[i]);
        t.g = l->grad[i];
        t.m = hasm ? static_cast<float *>(l->m[i]) : nullptr;
        t.v = hasv ? static_cast<float *>(l->v[i]) : nullptr;
        const uintptr_t bits = (uintptr_t)t.x | (uintptr_t)t.m | (uintptr_t)t.v;
        t.vec_ok = ((bits & 15) == 0) && (((uintptr_t)t.g & (bf16 ? 7 : 15)) == 0);
      }
      next_chunk += (uint32_t)((t.numel + ce - 1) / ce);
    }
    hipLaunchKernelGGL(expand_chunks_kernel, dim3((uint32_t)cnt), dim3(kThreads), 0, stream, batch, table, spans);
    SWIFT_HIP(hipGetLastError());
  }
  if (next_chunk == 0) return SWIFT_OK;
  // 2. pack the table by the mask (every entry of `packed` below next_chunk and the count are rewritten,
  //    so nothing of an earlier call is read), 3. the undo over the packed table
  const uint64_t n_slots = (uint64_t)next_chunk << tpc_shift;
  unsigned int *counters = reinterpret_cast<unsigned int *>(sb + kNoallocCountOff + 256);
  uint32_t log2c = 0;
  while ((2u << log2c) <= (uint32_t)std::min<long>(std::max<long>(knobs().dmask_counters, 1), kQueueMaxCounters)) ++log2c;
  hipLaunchKernelGGL(compact_chunks_kernel, dim3((uint32_t)l->n), dim3(kThreads), 0, stream,
                     static_cast<const ChunkDesc *>(table), static_cast<const TensorChunks *>(spans), (uint32_t)l->n,
                     device_mask, tpc_shift, packed, count, counters, 1u << log2c);
  SWIFT_HIP(hipGetLastError());
  return launch_packed(pick_packed_kernel(hp->kind, true, bf16, false), pick_queue_kernel(hp->kind, true, bf16, false), info, tune,
                       n_slots, tpc_shift, c, packed, count, counters, log2c, stream);
}

// ------------------------------------------------------------------------------------------
// LAMB: step = moments + partial sums, norms, apply; undo = one launch.
// Launch shapes (one wavefront per tile): U 16-byte vectors per lane in pass 1 (one partial sum per
// tile) and in pass 3.  The environment variables exist for sweeps.
typedef void (*LambMomentsKernel)(const ChunkDesc *, uint64_t, uint32_t, const OptConsts, double2 *);
typedef void (*LambApplyKernel)(const ChunkDesc *, uint64_t, uint32_t, const OptConsts, const double *);

LambMomentsKernel pick_lamb_moments(int u, bool bf16) {
  switch (u) {
    case 1: return bf16 ? lamb_moments_kernel<true, 1, 64> : lamb_moments_kernel<false, 1, 64>;
    case 2: return bf16 ? lamb_moments_kernel<true, 2, 64> : lamb_moments_kernel<false, 2, 64>;
    default: return bf16 ? lamb_moments_kernel<true, 4, 64> : lamb_moments_kernel<false, 4, 64>;
  }
}

LambApplyKernel pick_lamb_apply(int u, bool xb) {
  switch (u) {
    case 1: return xb ? lamb_apply_kernel<true, 1, 64> : lamb_apply_kernel<false, 1, 64>;
    case 2: return xb ? lamb_apply_kernel<true, 2, 64> : lamb_apply_kernel<false, 2, 64>;
    default: return xb ? lamb_apply_kernel<true, 4, 64> : lamb_apply_kernel<false, 4, 64>;
  }
}

int clamp_u(long u) { return u <= 1 ? 1 : (u == 2 ? 2 : 4); }

int lamb_prepare(Plan &plan, uint32_t tile_elems, hipStream_t stream) {
  std::lock_guard<std::mutex> lock(plan.lamb_mu);
  if (plan.lamb_spans && plan.lamb_tile_elems == tile_elems) return SWIFT_OK;
  if (int rc = refuse_under_capture(stream, "this tensor list has not been stepped with LAMB before")) return rc;
  if (plan.lamb_spans) {               // the pass-1 tile was changed (a sweep): rebuild the scratch
    (void)hipFree(plan.lamb_spans);    // (hipFree waits for kernels that may still read it)
    (void)hipFree(plan.lamb_partial);
    plan.lamb_spans = plan.lamb_partial = nullptr;
  }
  const uint64_t tpc = plan.chunk_elems / tile_elems;
  std::vector<TensorSpan> spans(plan.t_numel.size());
  for (size_t i = 0; i < spans.size(); ++i) {
    spans[i].first_slot = plan.t_first_chunk[i] * tpc;
    spans[i].n_slots = (plan.t_numel[i] + tile_elems - 1) / tile_elems;   // only the last chunk is short
    spans[i].active = plan.t_active[i];
    spans[i].pad = 0;
  }
  void *dspans = nullptr, *dpartial = nullptr;
  SWIFT_HIP(hipMalloc(&dspans, std::max<size_t>(spans.size(), 1) * sizeof(TensorSpan)));
  hipError_t e = hipMemcpy(dspans, spans.data(), spans.size() * sizeof(TensorSpan), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMalloc(&dpartial, std::max<uint64_t>((uint64_t)plan.n_chunks * tpc, 1) * sizeof(double2));
  if (e != hipSuccess) {
    (void)hipFree(dspans);
    return fail(SWIFT_EHIP, "LAMB scratch allocation failed: %s", hipGetErrorName(e));
  }
  plan.lamb_partial = dpartial;
  plan.lamb_tile_elems = tile_elems;
  plan.lamb_spans = dspans;
  plan.dev_bytes += std::max<size_t>(spans.size(), 1) * sizeof(TensorSpan) +
                    std::max<uint64_t>((uint64_t)plan.n_chunks * tpc, 1) * sizeof(double2);
  return SWIFT_OK;
}

int lamb_call(const swift_tensor_list *l, const swift_hparams *hp, const uint8_t *host_mask, double *norms,
              bool undo, void *stream_) {
  OptConsts c;
  int rc = validate_hparams(hp, undo, &c);
  if (rc) return rc;
  if (hp->kind != SWIFT_LAMB) return fail(SWIFT_EINVAL, "swift_lamb_* needs kind = SWIFT_LAMB");
  if ((rc = validate_list(l, hp))) return rc;
  if (l->n == 0) return SWIFT_OK;
  if (!norms) return fail(SWIFT_EINVAL, "norms_device is NULL");
  if ((uintptr_t)norms & 7) return fail(SWIFT_EINVAL, "norms_device is not 8-byte aligned");
  int dev = -1;
  SWIFT_HIP(hipGetDevice(&dev));
  DeviceInfo info;
  if ((rc = device_info(dev, &info))) return rc;
  if ((rc = check_device_range(norms, (size_t)l->n * 16, dev, "norms_device", 0))) return rc;
  const bool bf16 = hp->grad_dtype == SWIFT_BF16, xb = l->param_bf16 != nullptr;
  std::shared_ptr<Plan> plan;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if ((rc = build_opt_plan(l, hp, host_mask, dev, stream, &plan))) return rc;
  const Knobs kn = knobs();
  const int u1 = clamp_u(kn.lamb_u1), u3 = clamp_u(kn.lamb_u3);
  const uint32_t tile1 = (uint32_t)u1 * 256u, tile3 = (uint32_t)u3 * 256u, tileu = 256u;
  const uint32_t s1 = shift_for(tile1, plan->chunk_elems), s3 = shift_for(tile3, plan->chunk_elems);
  const uint32_t su = shift_for(tileu, plan->chunk_elems);
  const uint64_t slots1 = (uint64_t)plan->n_chunks << s1, slots3 = (uint64_t)plan->n_chunks << s3;
  const uint64_t slotsu = (uint64_t)plan->n_chunks << su;
  const Tuning t1{u1, 64, (int)kn.lamb_waves_p1};
  const Tuning t3{u3, 64, (int)kn.lamb_waves_p3};
  const Tuning tu = opt_tuning(SWIFT_ADAMW, bf16, true);
  const ChunkDesc *chunks = static_cast<const ChunkDesc *>(plan->chunks());
  if (undo) {
    if (plan->n_chunks == 0) return SWIFT_OK;
    const auto k = bf16 ? (xb ? lamb_undo_kernel<true, true, 1, 64> : lamb_undo_kernel<true, false, 1, 64>)
                        : (xb ? lamb_undo_kernel<false, true, 1, 64> : lamb_undo_kernel<false, false, 1, 64>);
    hipLaunchKernelGGL(k, dim3(grid_for(slotsu, 64)), dim3(64), lds_cap_bytes(info, tu),
                       stream, chunks, slotsu, su, c, static_cast<const double *>(norms));
    SWIFT_HIP(hipGetLastError());
    return SWIFT_OK;
  }
  if ((rc = lamb_prepare(*plan, tile1, stream))) return rc;
  if (plan->n_chunks) {
    hipLaunchKernelGGL(pick_lamb_moments(u1, bf16), dim3(grid_for(slots1, 64)), dim3(64),
                       lds_cap_bytes(info, t1), stream, chunks, slots1, s1, c, static_cast<double2 *>(plan->lamb_partial));
    SWIFT_HIP(hipGetLastError());
  }
  hipLaunchKernelGGL(lamb_norms_kernel, dim3((uint32_t)l->n), dim3(kThreads), 0, stream,
                     static_cast<const TensorSpan *>(plan->lamb_spans), static_cast<const double2 *>(plan->lamb_partial), norms);
  SWIFT_HIP(hipGetLastError());
  if (plan->n_chunks) {
    hipLaunchKernelGGL(pick_lamb_apply(u3, xb), dim3(grid_for(slots3, 64)), dim3(64),
                       lds_cap_bytes(info, t3), stream, chunks, slots3, s3, c, static_cast<const double *>(norms));
    SWIFT_HIP(hipGetLastError());
  }
  return SWIFT_OK;
}

// ------------------------------------------------------------------------------------------
// Optimizer step / undo fused with the digest of the new state.
int fused_prepare(Plan &plan, uint32_t tile_elems, hipStream_t stream) {
  std::lock_guard<std::mutex> lock(plan.lamb_mu);
  if (plan.fused_spans && plan.fused_tile_elems == tile_elems) return SWIFT_OK;
  if (int rc = refuse_under_capture(stream, "this tensor list has not been used with the fused digest before")) return rc;
  const uint64_t tile_slots = (uint64_t)std::max<uint32_t>(plan.n_chunks, 1) * (plan.chunk_elems / tile_elems);
  if (plan.fused_spans) {              // the tile was changed (a sweep): only the tile sums change size
    (void)hipFree(plan.fused_tiles);   // (hipFree waits for kernels that may still use it)
    plan.fused_tiles = nullptr;
    SWIFT_HIP(hipMalloc(&plan.fused_tiles, tile_slots * 3 * sizeof(uint64_t)));
    plan.fused_tile_elems = tile_elems;
    return SWIFT_OK;
  }
  std::vector<TensorSpan> spans(plan.t_numel.size());
  for (size_t i = 0; i < spans.size(); ++i) {
    spans[i].first_slot = plan.t_first_chunk[i];
    spans[i].n_slots = (plan.t_numel[i] + plan.chunk_elems - 1) / plan.chunk_elems;
    spans[i].active = plan.t_active[i];
    spans[i].pad = 0;
  }
  void *dspans = nullptr, *dslots = nullptr, *dtiles = nullptr;
  SWIFT_HIP(hipMalloc(&dspans, std::max<size_t>(spans.size(), 1) * sizeof(TensorSpan)));
  hipError_t e = hipMemcpy(dspans, spans.data(), spans.size() * sizeof(TensorSpan), hipMemcpyHostToDevice);
  if (e == hipSuccess) e = hipMalloc(&dslots, std::max<size_t>(plan.n_chunks, 1) * 3 * sizeof(uint64_t));
  if (e == hipSuccess) e = hipMalloc(&dtiles, tile_slots * 3 * sizeof(uint64_t));
  if (e != hipSuccess) {
    (void)hipFree(dspans);
    if (dslots) (void)hipFree(dslots);
    return fail(SWIFT_EHIP, "digest scratch allocation failed: %s", hipGetErrorName(e));
  }
  plan.fused_slots = dslots;
  plan.fused_tiles = dtiles;
  plan.fused_tile_elems = tile_elems;
  plan.fused_spans = dspans;
  plan.dev_bytes += std::max<size_t>(spans.size(), 1) * sizeof(TensorSpan) +
                    (std::max<size_t>(plan.n_chunks, 1) + tile_slots) * 3 * sizeof(uint64_t);
  return SWIFT_OK;
}

typedef void (*FusedKernel)(const ChunkDesc *, uint64_t, uint32_t, const OptConsts, uint64_t *);

template <int U>
FusedKernel pick_fused_u(int kind, bool undo, bool bf16, bool xb) {
#define SWIFT_PICK2(K, UNDO_, BF_) (xb ? opt_digest_kernel<K, UNDO_, BF_, true, U, 64> : opt_digest_kernel<K, UNDO_, BF_, false, U, 64>)
#define SWIFT_PICK(K)                                                         \
  (undo ? (bf16 ? SWIFT_PICK2(K, true, true) : SWIFT_PICK2(K, true, false))   \
        : (bf16 ? SWIFT_PICK2(K, false, true) : SWIFT_PICK2(K, false, false)))
  switch (kind) {
    case SWIFT_SGD: return SWIFT_PICK(kSGD);
    case SWIFT_SGDM: return SWIFT_PICK(kSGDM);
    case SWIFT_ADAM: return SWIFT_PICK(kADAM);
    default: return SWIFT_PICK(kADAMW);
  }
#undef SWIFT_PICK
#undef SWIFT_PICK2
}

// Vectors per lane of the fused kernel: the default, plus the alternatives of a sweep build.
FusedKernel pick_fused(int u, int kind, bool undo, bool bf16, bool xb) {
#ifdef SWIFT_SWEEP_SHAPES
  if (u == 1) return pick_fused_u<1>(kind, undo, bf16, xb);
  if (u == 2) return pick_fused_u<2>(kind, undo, bf16, xb);
  if (u == 4) return pick_fused_u<4>(kind, undo, bf16, xb);
#endif
  if (u == SWIFT_FUSED_U) return pick_fused_u<SWIFT_FUSED_U>(kind, undo, bf16, xb);
  return nullptr;
}

int fused_call(const swift_tensor_list *l, const swift_hparams *hp, const uint8_t *host_mask, uint64_t *digests,
               bool undo, void *stream_) {
  OptConsts c;
  int rc = validate_hparams(hp, undo, &c);
  if (rc) return rc;
  if (hp->kind == SWIFT_LAMB) return fail(SWIFT_EINVAL, "the fused digest entry points do not take LAMB");
  if ((rc = validate_list(l, hp))) return rc;
  if (l->n == 0) return SWIFT_OK;
  for (int64_t i = 0; i < l->n; ++i)
    if (l->numel[i] >= (int64_t)1 << 32)
      return fail(SWIFT_EINVAL, "tensor %lld has 2^32 elements or more: its digest index would not fit", (long long)i);
  if (!digests) return fail(SWIFT_EINVAL, "digests_device is NULL");
  if ((uintptr_t)digests & 7) return fail(SWIFT_EINVAL, "digests_device is not 8-byte aligned");
  const uint32_t n_groups = 1u + (kind_has_m(hp->kind) ? 1u : 0u) + (kind_has_v(hp->kind) ? 1u : 0u);   // theta [, m [, v]]
  int dev = -1;
  SWIFT_HIP(hipGetDevice(&dev));
  DeviceInfo info;
  if ((rc = device_info(dev, &info))) return rc;
  if ((rc = check_device_range(digests, (size_t)l->n * n_groups * 8, dev, "digests_device", 0))) return rc;
  const bool bf16 = hp->grad_dtype == SWIFT_BF16;
  std::shared_ptr<Plan> plan;
  hipStream_t stream = static_cast<hipStream_t>(stream_);
  if ((rc = build_opt_plan(l, hp, host_mask, dev, stream, &plan))) return rc;
  Tuning tune = opt_tuning(hp->kind, bf16, undo);
  tune.u = (int)knobs().fused_u;
  tune.block = 64;
  // the digest arithmetic makes this kernel ALU-heavy: more resident wavefronts overlap it with memory
  tune.waves_per_cu = (int)knobs().fused_waves_per_cu;
  const FusedKernel fused_kernel = pick_fused(tune.u, hp->kind, undo, bf16, l->param_bf16 != nullptr);
  if (!fused_kernel) return fail(SWIFT_EINVAL, "fused launch shape U=%d is not compiled in", tune.u);
  const uint32_t tile_elems = 256u * (uint32_t)tune.u;
  if ((rc = fused_prepare(*plan, tile_elems, stream))) return rc;
  uint64_t *slots = static_cast<uint64_t *>(plan->fused_slots), *tiles = static_cast<uint64_t *>(plan->fused_tiles);
  if (plan->n_chunks) {
    const uint32_t shift = shift_for(tile_elems, plan->chunk_elems);
    const uint64_t n_slots = (uint64_t)plan->n_chunks << shift;
    const ChunkDesc *table = static_cast<const ChunkDesc *>(plan->chunks());
    hipLaunchKernelGGL(fused_kernel, dim3(grid_for(n_slots, 64)),
                       dim3(64), lds_cap_bytes(info, tune), stream, table, n_slots, shift, c, tiles);
    SWIFT_HIP(hipGetLastError());
    hipLaunchKernelGGL(chunk_digest_kernel, dim3(plan->n_chunks), dim3(kThreads), 0, stream, table, shift, tile_elems,
                       n_groups, static_cast<const uint64_t *>(tiles), slots);
    SWIFT_HIP(hipGetLastError());
  }
  hipLaunchKernelGGL(digest_gather_kernel, dim3((uint32_t)l->n), dim3(64), 0, stream,
                     static_cast<const TensorSpan *>(plan->fused_spans), static_cast<const uint64_t *>(slots), (uint32_t)l->n,
                     n_groups, digests);
  SWIFT_HIP(hipGetLastError());
  return SWIFT_OK;
}

// ------------------------------------------------------------------------------------------
// Digest.
int64_t digest_count(int64_t n_buf, const int64_t *numel, int64_t shard_elems, bool set_error) {
  if (n_buf < 0 || (n_buf > 0 && !numel) || shard_elems < 0 || shard_elems >= (int64_t)1 << 32)
    return set_error ? fail(SWIFT_EINVAL, "digest: bad n_buf, numel or shard_elems") : SWIFT_EINVAL;
  int64_t total = 0;
  for (int64_t i = 0; i < n_buf; ++i) {
    if (numel[i] < 0 || numel[i] > kMaxNumel)
      return set_error ? fail(SWIFT_EINVAL, "digest: numel[%lld] is negative or beyond 2^40", (long long)i) : SWIFT_EINVAL;
    if (shard_elems == 0) {
      if (numel[i] >= (int64_t)1 << 32)
        return set_error ? fail(SWIFT_EINVAL, "digest: buffer %lld has 2^32 words or more; give shard_elems", (long long)i)
                         : SWIFT_EINVAL;
      total += 1;
    } else {
      total += (numel[i] + shard_elems - 1) / shard_elems;
    }
  }
  return total;
}

// Digest chunks: one workgroup and one 64-bit partial sum per chunk.  The launch needs about sixteen
// workgroups per compute unit to fill the chip, so the length follows the total size.
uint32_t digest_chunk_elems(uint64_t total, int cus) {
  const uint32_t tile = 4u * kThreads * 4;                     // chunk lengths are multiples of four rounds of the kernel
  const long forced = knobs().digest_chunk_elems;              // tuning knob for sweeps
  if (forced >= (long)tile && forced <= (1l << 22) && forced % tile == 0) return (uint32_t)forced;
  // measured with whole-tensor shards: 32 Ki to 128 Ki words are within 1 % of each other on lists of 0.3 to 7 G
  // parameters, 256 Ki is 2-5 % slower on the smaller ones (coarser tail), 8 Ki and less pay for short loops
  const uint32_t cap = SWIFT_DIGEST_CHUNK;
  const uint64_t want = total / (16ull * (uint64_t)cus);
  uint32_t ce = tile;
  while (ce < cap && (uint64_t)ce * 2 <= want) ce *= 2;
  return ce;
}

int build_digest_plan(int64_t n_buf, const void *const *buf, const int64_t *numel, int64_t shard_elems, int dev,
                      int cus, hipStream_t stream, std::shared_ptr<Plan> *out) {
  std::string key;
  key.reserve(64 + (size_t)n_buf * 16);
  key_add(key, (uint8_t)'D');
  key_add(key, dev);
  key_add(key, n_buf);
  key_add(key, shard_elems);
  key_add(key, knobs().digest_chunk_elems);
  for (int64_t i = 0; i < n_buf; ++i) {
    key_add(key, numel[i]);
    key_add(key, buf[i]);
  }
  if (auto hit = find_plan(key)) {
    bool stale = false;
    int rc = reuse_plan(hit, stream, &stale);
    if (rc) return rc;
    if (!stale) {
      *out = hit;
      return SWIFT_OK;
    }
  }
  {
    int rc = refuse_under_capture(stream, "this buffer list has not been digested before");
    if (rc) return rc;
  }
  std::vector<DigestDesc> descs((size_t)n_buf);
  uint64_t total = 0, n_out = 0;
  for (int64_t i = 0; i < n_buf; ++i) {
    const uint64_t n = (uint64_t)numel[i];
    descs[(size_t)i] = {static_cast<const uint32_t *>(buf[i]), (int64_t)n, n_out};
    n_out += shard_elems ? (n + shard_elems - 1) / shard_elems : 1;
    if (n == 0) continue;
    if (!buf[i]) return fail(SWIFT_EINVAL, "digest: buffer %lld is NULL", (long long)i);
    if ((uintptr_t)buf[i] & 3) return fail(SWIFT_EINVAL, "digest: buffer %lld is not 4-byte aligned", (long long)i);
    int rc = check_device_range(buf[i], n * 4, dev, "buf", i);
    if (rc) return rc;
    total += n;
  }
  auto plan = std::make_shared<Plan>();
  plan->key = std::move(key);
  plan->device = dev;
  plan->n_out = n_out;
  plan->chunk_elems = digest_chunk_elems(total, cus);
  const uint64_t ce = plan->chunk_elems;
  std::vector<ChunkRef> chunks;
  chunks.reserve((size_t)(total / ce) + (size_t)n_out);
  std::vector<DigestSpan> spans((size_t)n_out, DigestSpan{0, 0});
  bool single = true;                                       // every shard is one chunk
  for (int64_t i = 0; i < n_buf; ++i) {
    const uint64_t n = (uint64_t)numel[i];
    if (n == 0) {
      if (shard_elems == 0) plan->digest_has_empty = true;  // one output, no chunk
      continue;
    }
    const uint64_t S = shard_elems ? (uint64_t)shard_elems : n;
    const uint64_t cps = (S + ce - 1) / ce;                 // chunk numbers per full shard
    const uint64_t n_shards = (n + S - 1) / S;
    if (cps * n_shards > 0xffffffffull) return fail(SWIFT_EINVAL, "digest: buffer %lld needs too many chunks", (long long)i);
    if (cps > 1) single = false;
    for (uint64_t s = 0; s < n_shards; ++s) {
      const uint64_t shard_len = std::min<uint64_t>(S, n - s * S);
      const uint64_t nc = (shard_len + ce - 1) / ce;
      spans[(size_t)(descs[(size_t)i].first_out + s)] = DigestSpan{chunks.size(), nc};
      for (uint64_t k = 0; k < nc; ++k) chunks.push_back({(uint32_t)i, (uint32_t)(s * cps + k)});
    }
  }
  if (chunks.size() > 0xffffffffull) return fail(SWIFT_EINVAL, "digest: too many chunks");
  int rc = upload_plan(*plan, descs.data(), descs.size() * sizeof(DigestDesc), chunks.data(), chunks.size(),
                       sizeof(ChunkRef));
  if (rc) return rc;
  if (!single) {                                            // chunk sums are gathered per shard by a second kernel
    const size_t span_bytes = spans.size() * sizeof(DigestSpan), part_bytes = chunks.size() * sizeof(uint64_t);
    SWIFT_HIP(hipMalloc(&plan->digest_spans, span_bytes));
    SWIFT_HIP(hipMemcpy(plan->digest_spans, spans.data(), span_bytes, hipMemcpyHostToDevice));
    SWIFT_HIP(hipMalloc(&plan->digest_partial, part_bytes));
    plan->dev_bytes += span_bytes + part_bytes;
  }
  for (int64_t i = 0; i < n_buf && !plan->probe_ptr; ++i)
    if (numel[i] > 0) set_probe(*plan, buf[i]);
  keep_plan(plan);
  *out = plan;
  return SWIFT_OK;
}

// ------------------------------------------------------------------------------------------
// Update tracker: the paper's own bookkeeping (Implementation, "Update-undo").  Per iteration the
// training loop updates tensors group by group as their gradients become final; every tensor
// whose update kernels have been launched is marked, and after a failure exactly the marked
// tensors are undone -- once the kernels already launched have run to completion.
struct Tracker {
  int64_t n_tensors = 0;
  int64_t step = 0;                    // iteration whose update is in progress (0: none)
  int device = -1;
  std::vector<uint8_t> marks;
  // Streams that carried tracked launches of this iteration (nearly always one).  Work enqueued later on the
  // same stream runs after them by stream order; another stream is made to wait through an event recorded
  // when the wait is needed, so a tracked launch costs no event of its own.
  std::vector<hipStream_t> streams;
  std::vector<hipEvent_t> pool;        // events for cross-stream waits, reused
  std::mutex mu;
};

// The host waits until every tracked launch of this iteration has finished.
int tracker_wait(Tracker &t) {
  for (hipStream_t s : t.streams) SWIFT_HIP(hipStreamSynchronize(s));
  return SWIFT_OK;
}

// `stream` waits, on the device, for every tracked launch of this iteration.
int tracker_order_after(Tracker &t, hipStream_t stream) {
  size_t used = 0;
  for (hipStream_t s : t.streams) {
    if (s == stream) continue;
    if (used == t.pool.size()) {
      hipEvent_t e;
      SWIFT_HIP(hipEventCreateWithFlags(&e, hipEventDisableTiming));
      t.pool.push_back(e);
    }
    hipEvent_t e = t.pool[used++];
    SWIFT_HIP(hipEventRecord(e, s));
    SWIFT_HIP(hipStreamWaitEvent(stream, e, 0));
  }
  return SWIFT_OK;
}

}  // namespace
}  // namespace swift

using namespace swift;

extern "C" {

int swift_opt_step(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *host_mask, void *hip_stream) {
  return guarded([&] { return opt_call(list, hp, host_mask, nullptr, false, false, hip_stream); });
}

int swift_opt_undo(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *host_mask, void *hip_stream) {
  return guarded([&] { return opt_call(list, hp, host_mask, nullptr, false, true, hip_stream); });
}

int swift_opt_step_dmask(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *device_mask,
                         void *hip_stream) {
  return guarded([&] { return opt_call(list, hp, nullptr, device_mask, true, false, hip_stream); });
}

int swift_opt_undo_dmask(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *device_mask,
                         void *hip_stream) {
  return guarded([&] { return opt_call(list, hp, nullptr, device_mask, true, true, hip_stream); });
}

int swift_opt_undo_dmask_noalloc(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *device_mask,
                                 void *hip_stream) {
  return guarded([&] { return noalloc_undo_dmask(list, hp, device_mask, hip_stream); });   // (an error message may allocate host memory)
}

int swift_opt_step_digest(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *host_mask,
                          uint64_t *digests_device, void *hip_stream) {
  return guarded([&] { return fused_call(list, hp, host_mask, digests_device, false, hip_stream); });
}

int swift_opt_undo_digest(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *host_mask,
                          uint64_t *digests_device, void *hip_stream) {
  return guarded([&] { return fused_call(list, hp, host_mask, digests_device, true, hip_stream); });
}

int swift_lamb_step(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *host_mask,
                    double *norms_device, void *hip_stream) {
  return guarded([&] { return lamb_call(list, hp, host_mask, norms_device, false, hip_stream); });
}

int swift_lamb_undo(const swift_tensor_list *list, const swift_hparams *hp, const uint8_t *host_mask,
                    const double *norms_device, void *hip_stream) {
  return guarded([&] { return lamb_call(list, hp, host_mask, const_cast<double *>(norms_device), true, hip_stream); });
}

int64_t swift_digest_count(int64_t n_buf, const int64_t *numel, int64_t shard_elems) {
  return digest_count(n_buf, numel, shard_elems, true);
}

int swift_state_digest(int64_t n_buf, const void *const *buf, const int64_t *numel, int64_t shard_elems,
                       uint64_t *out_device, void *hip_stream) {
  return guarded([&]() -> int {
    const int64_t n_out = digest_count(n_buf, numel, shard_elems, true);
    if (n_out < 0) return (int)n_out;
    if (n_buf > 0 && !buf) return fail(SWIFT_EINVAL, "digest: buf array is NULL");
    if (n_out == 0) return SWIFT_OK;
    if (!out_device) return fail(SWIFT_EINVAL, "digest: out_device is NULL");
    if ((uintptr_t)out_device & 7) return fail(SWIFT_EINVAL, "digest: out_device is not 8-byte aligned");
    int dev = -1, rc;
    SWIFT_HIP(hipGetDevice(&dev));
    DeviceInfo info;
    if ((rc = device_info(dev, &info))) return rc;
    if ((rc = check_device_range(out_device, (size_t)n_out * 8, dev, "out_device", 0))) return rc;
    std::shared_ptr<Plan> plan;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    if ((rc = build_digest_plan(n_buf, buf, numel, shard_elems, dev, info.cus, stream, &plan))) return rc;
    uint64_t *out = out_device;
    uint64_t *partial = static_cast<uint64_t *>(plan->digest_partial);
    // Shards of several chunks: chunk sums, then one wavefront per shard adds them up and writes every output
    // (an empty buffer's too).  Single-chunk shards: each output is written by its one chunk; only the digests
    // of empty buffers (0) need a fill, by a kernel, not a memset node, so that the call can be captured.
    if (!partial && plan->digest_has_empty) {
      const uint32_t fill_grid = (uint32_t)std::min<uint64_t>(((uint64_t)n_out + kThreads - 1) / kThreads, 1024);
      hipLaunchKernelGGL(fill_u64_kernel, dim3(fill_grid), dim3(kThreads), 0, stream, out, (uint64_t)n_out, (uint64_t)0);
      SWIFT_HIP(hipGetLastError());
    }
    if (plan->n_chunks) {
      const uint32_t grid = grid_for(plan->n_chunks, kThreads);  // one workgroup per chunk
      const Tuning dtune{1, kThreads, (int)knobs().digest_waves_per_cu};
      hipLaunchKernelGGL(digest_kernel, dim3(grid), dim3(kThreads), lds_cap_bytes(info, dtune), stream,
                         static_cast<const DigestDesc *>(plan->descs()), static_cast<const ChunkRef *>(plan->chunks()),
                         plan->n_chunks, plan->chunk_elems, (uint64_t)shard_elems, partial, out);
      SWIFT_HIP(hipGetLastError());
    }
    if (partial) {
      const DigestSpan *spans = static_cast<const DigestSpan *>(plan->digest_spans);
      if ((uint64_t)plan->n_chunks >= 64ull * (uint64_t)n_out && (uint64_t)n_out <= 0x7fffffffull) {
        hipLaunchKernelGGL(digest_reduce_kernel<true>, dim3((uint32_t)n_out), dim3(kThreads), 0, stream, spans,
                           static_cast<const uint64_t *>(partial), (uint64_t)n_out, out);
      } else {
        const uint64_t per_block = kThreads / 64;
        if (((uint64_t)n_out + per_block - 1) / per_block > 0x7fffffffull) return fail(SWIFT_EINVAL, "digest: too many outputs");
        hipLaunchKernelGGL(digest_reduce_kernel<false>, dim3((uint32_t)(((uint64_t)n_out + per_block - 1) / per_block)),
                           dim3(kThreads), 0, stream, spans, static_cast<const uint64_t *>(partial), (uint64_t)n_out, out);
      }
      SWIFT_HIP(hipGetLastError());
    }
    return SWIFT_OK;
  });
}

int swift_mask_from_digests(int64_t n_tensors, int64_t n_groups, const uint64_t *before_device,
                            const uint64_t *after_device, uint8_t *mask_device, void *hip_stream) {
  return guarded([&]() -> int {
    if (n_tensors < 0 || n_tensors > (int64_t)0x7fffffff || n_groups < 1 || n_groups > 64)
      return fail(SWIFT_EINVAL, "mask_from_digests: n_tensors or n_groups out of range");
    if (n_tensors == 0) return SWIFT_OK;
    if (!before_device || !after_device || !mask_device) return fail(SWIFT_EINVAL, "mask_from_digests: NULL pointer");
    if (((uintptr_t)before_device | (uintptr_t)after_device) & 7)
      return fail(SWIFT_EINVAL, "mask_from_digests: digest arrays are not 8-byte aligned");
    int dev = -1, rc;
    SWIFT_HIP(hipGetDevice(&dev));
    const size_t dbytes = (size_t)n_tensors * (size_t)n_groups * 8;
    if ((rc = check_device_range(before_device, dbytes, dev, "before_device", 0))) return rc;
    if ((rc = check_device_range(after_device, dbytes, dev, "after_device", 0))) return rc;
    if ((rc = check_device_range(mask_device, (size_t)n_tensors, dev, "mask_device", 0))) return rc;
    const uint32_t grid = (uint32_t)std::min<int64_t>((n_tensors + kThreads - 1) / kThreads, 1024);
    hipLaunchKernelGGL(mask_from_digests_kernel, dim3(grid), dim3(kThreads), 0, static_cast<hipStream_t>(hip_stream),
                       (uint32_t)n_tensors, (uint32_t)n_groups, before_device, after_device, mask_device);
    SWIFT_HIP(hipGetLastError());
    return SWIFT_OK;
  });
}

int swift_stream_copy(void *dst_device, const void *src_device, int64_t bytes, void *hip_stream) {
  return guarded([&]() -> int {
    if (bytes < 0 || (bytes & 15) || bytes > 4 * kMaxNumel)
      return fail(SWIFT_EINVAL, "stream_copy: bytes must be a non-negative multiple of 16 (at most 2^42)");
    if (bytes == 0) return SWIFT_OK;
    if (!dst_device || !src_device) return fail(SWIFT_EINVAL, "stream_copy: NULL pointer");
    if (((uintptr_t)dst_device | (uintptr_t)src_device) & 15) return fail(SWIFT_EINVAL, "stream_copy: pointers must be 16-byte aligned");
    int dev = -1, rc;
    SWIFT_HIP(hipGetDevice(&dev));
    DeviceInfo info;
    if ((rc = device_info(dev, &info))) return rc;
    if ((rc = check_device_range(dst_device, (size_t)bytes, dev, "dst_device", 0))) return rc;
    if ((rc = check_device_range(src_device, (size_t)bytes, dev, "src_device", 0))) return rc;
    const char *d = static_cast<const char *>(dst_device), *s = static_cast<const char *>(src_device);
    if (d < s + bytes && s < d + bytes) return fail(SWIFT_EINVAL, "stream_copy: ranges overlap");
    // A copy moves only 2 x 16 bytes per lane, so unlike the update kernels it wants every wavefront slot of
    // a CU filled: one vector per lane and no residency cap measured best (6.7 TB/s; 4.3 with the update
    // kernels' cap of 11).  Knobs for sweeps.
    const int u = clamp_u(knobs().copy_u);
    const Tuning tune{u, SWIFT_DEFAULT_BLOCK, (int)knobs().copy_waves_per_cu};
    const uint64_t n16 = (uint64_t)bytes / 16;
    const uint64_t tile = (uint64_t)u * SWIFT_DEFAULT_BLOCK;
    const uint64_t tiles = (n16 + tile - 1) / tile;
    const uint32_t grid = grid_for(tiles, SWIFT_DEFAULT_BLOCK);
    const auto launch = [&](auto kernel) {
      hipLaunchKernelGGL(kernel, dim3(grid), dim3(SWIFT_DEFAULT_BLOCK), lds_cap_bytes(info, tune),
                         static_cast<hipStream_t>(hip_stream), static_cast<u32x4 *>(dst_device),
                         static_cast<const u32x4 *>(src_device), n16);
    };
    if (u == 1) launch(copy_kernel<1, SWIFT_DEFAULT_BLOCK>);
    else if (u == 2) launch(copy_kernel<2, SWIFT_DEFAULT_BLOCK>);
    else launch(copy_kernel<4, SWIFT_DEFAULT_BLOCK>);
    SWIFT_HIP(hipGetLastError());
    return SWIFT_OK;
  });
}

struct swift_tracker {
  Tracker t;
};

int swift_tracker_create(int64_t n_tensors, swift_tracker **out) {
  return guarded([&]() -> int {
    if (!out) return fail(SWIFT_EINVAL, "tracker: out is NULL");
    *out = nullptr;
    if (n_tensors < 0 || n_tensors > (int64_t)0x7fffffff) return fail(SWIFT_EINVAL, "tracker: tensor count out of range");
    swift_tracker *tr = new (std::nothrow) swift_tracker();
    if (!tr) return fail(SWIFT_EHIP, "tracker: out of host memory");
    tr->t.n_tensors = n_tensors;
    tr->t.marks.assign((size_t)n_tensors, 0);
    *out = tr;
    return SWIFT_OK;
  });
}

int swift_tracker_destroy(swift_tracker *tr) {
  if (!tr) return SWIFT_OK;
  Tracker &t = tr->t;
  {
    std::lock_guard<std::mutex> lock(t.mu);
    // launches in flight own nothing of the tracker's (an event may be destroyed while a stream still waits for it)
    for (hipEvent_t e : t.pool) (void)hipEventDestroy(e);
    t.pool.clear();
  }
  delete tr;
  return SWIFT_OK;
}

int swift_tracker_begin(swift_tracker *tr, int64_t step) {
  if (!tr) return fail(SWIFT_EINVAL, "tracker is NULL");
  if (step < 1) return fail(SWIFT_EINVAL, "tracker: step must be >= 1");
  Tracker &t = tr->t;
  std::lock_guard<std::mutex> lock(t.mu);
  // the previous iteration's update is complete on every replica once the next one begins (the
  // paper's argument for keeping a single gradient version): its marks are dropped
  t.streams.clear();
  std::fill(t.marks.begin(), t.marks.end(), 0);
  t.step = step;
  return SWIFT_OK;
}

int swift_tracker_step(swift_tracker *tr, const swift_tensor_list *group, const int64_t *tensor_ids,
                       const swift_hparams *hp, void *grad_ready_event, void *hip_stream) {
  return guarded([&]() -> int {
    if (!tr) return fail(SWIFT_EINVAL, "tracker is NULL");
    if (!group || !hp) return fail(SWIFT_EINVAL, "tracker: group or hparams is NULL");
    if (group->n > 0 && !tensor_ids) return fail(SWIFT_EINVAL, "tracker: tensor_ids is NULL");
    Tracker &t = tr->t;
    std::lock_guard<std::mutex> lock(t.mu);
    if (t.step == 0) return fail(SWIFT_EINVAL, "tracker: swift_tracker_begin has not been called");
    if (hp->step != t.step)
      return fail(SWIFT_EINVAL, "tracker: hparams.step = %lld but iteration %lld is in progress", (long long)hp->step,
                  (long long)t.step);
    // validate the ids in one pass: 2 = "named by this call" while the call is being checked
    int bad = SWIFT_OK;
    int64_t checked = 0;
    for (; checked < group->n && bad == SWIFT_OK; ++checked) {
      const int64_t id = tensor_ids[checked];
      if (id < 0 || id >= t.n_tensors) bad = fail(SWIFT_EINVAL, "tracker: tensor id %lld out of range", (long long)id);
      else if (t.marks[(size_t)id] == 1) bad = fail(SWIFT_EINVAL, "tracker: tensor %lld was already updated in this iteration", (long long)id);
      else if (t.marks[(size_t)id] == 2) bad = fail(SWIFT_EINVAL, "tracker: tensor id %lld appears twice", (long long)id);
      else t.marks[(size_t)id] = 2;
    }
    auto unmark = [&](int64_t upto) {
      for (int64_t k = 0; k < upto; ++k) {
        const int64_t id = tensor_ids[k];
        if (id >= 0 && id < t.n_tensors && t.marks[(size_t)id] == 2) t.marks[(size_t)id] = 0;
      }
    };
    if (bad != SWIFT_OK) {
      unmark(checked);
      return bad;
    }
    struct Rollback {                    // any early return below leaves no tensor half-marked
      decltype(unmark) &undo;
      int64_t n;
      bool armed = true;
      ~Rollback() { if (armed) undo(n); }
    } rollback{unmark, group->n};
    int dev = -1;
    SWIFT_HIP(hipGetDevice(&dev));
    if (t.device < 0) t.device = dev;
    if (dev != t.device) return fail(SWIFT_EINVAL, "tracker: created for device %d, current device is %d", t.device, dev);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // everything that can be refused is checked before anything is enqueued, the stream wait included
    OptLaunch launch;
    if (int rc = opt_prepare(group, hp, nullptr, nullptr, false, false, stream, &launch)) return rc;
    // the update waits (on the device) for the gradient to be final, as the paper's loop waits for the
    // all-reduce of that tensor before launching its update kernels
    if (grad_ready_event) SWIFT_HIP(hipStreamWaitEvent(stream, static_cast<hipEvent_t>(grad_ready_event), 0));
    if (int rc = opt_launch(launch, stream)) return rc;   // the launch itself failed (SWIFT_EHIP): nothing is marked
    if (std::find(t.streams.begin(), t.streams.end(), stream) == t.streams.end()) t.streams.push_back(stream);
    rollback.armed = false;
    for (int64_t k = 0; k < group->n; ++k) t.marks[(size_t)tensor_ids[k]] = 1;
    return SWIFT_OK;
  });
}

int swift_tracker_marks(swift_tracker *tr, uint8_t *host_mask_out) {
  if (!tr) return fail(SWIFT_EINVAL, "tracker is NULL");
  if (!host_mask_out && tr->t.n_tensors > 0) return fail(SWIFT_EINVAL, "tracker: host_mask_out is NULL");
  Tracker &t = tr->t;
  std::lock_guard<std::mutex> lock(t.mu);
  int rc = tracker_wait(t);            // launched update kernels run to completion before the marks are read (Implementation, "Update-undo")
  if (rc) return rc;
  if (t.n_tensors) memcpy(host_mask_out, t.marks.data(), (size_t)t.n_tensors);
  return SWIFT_OK;
}

int swift_tracker_undo(swift_tracker *tr, const swift_tensor_list *list, const swift_hparams *hp, void *hip_stream) {
  return guarded([&]() -> int {
    if (!tr) return fail(SWIFT_EINVAL, "tracker is NULL");
    if (!list || !hp) return fail(SWIFT_EINVAL, "tracker: list or hparams is NULL");
    Tracker &t = tr->t;
    std::lock_guard<std::mutex> lock(t.mu);
    if (list->n != t.n_tensors) return fail(SWIFT_EINVAL, "tracker: the list has %lld tensors, the tracker %lld", (long long)list->n, (long long)t.n_tensors);
    if (t.step == 0 || hp->step != t.step)
      return fail(SWIFT_EINVAL, "tracker: hparams.step = %lld but iteration %lld is in progress", (long long)hp->step,
                  (long long)t.step);
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    // the kernels already launched run to completion first (Implementation, "Update-undo"): by stream order,
    // or through an event where they went to another stream; the host does not wait
    OptLaunch launch;
    if (int rc = opt_prepare(list, hp, t.marks.data(), nullptr, false, true, stream, &launch)) return rc;
    if (int rc = tracker_order_after(t, stream)) return rc;
    if (int rc = opt_launch(launch, stream)) return rc;
    t.streams.clear();
    std::fill(t.marks.begin(), t.marks.end(), 0);   // the state is back at the start of the iteration
    return SWIFT_OK;
  });
}

int swift_logging_groups(int64_t n_machines, const double *compute_time, const double *message_bytes,
                         double checkpoint_interval, double bandwidth, double storage_limit, int parallel_recovery,
                         int32_t *group_of, double *storage_out, double *recovery_out) {
  if (n_machines < 1 || n_machines > (int64_t)0x7fffffff) return fail(SWIFT_EINVAL, "n_machines = %lld out of range", (long long)n_machines);
  if (!compute_time || (n_machines > 1 && !message_bytes) || !group_of)
    return fail(SWIFT_EINVAL, "compute_time, message_bytes and group_of must not be NULL");
  if (!(checkpoint_interval > 0) || !std::isfinite(checkpoint_interval))
    return fail(SWIFT_EINVAL, "checkpoint_interval must be finite and > 0");
  if (!(bandwidth > 0)) return fail(SWIFT_EINVAL, "bandwidth must be > 0 (infinity allowed)");
  if (std::isnan(storage_limit)) return fail(SWIFT_EINVAL, "storage_limit is NaN");
  for (int64_t i = 0; i < n_machines; ++i)
    if (!(compute_time[i] >= 0) || !std::isfinite(compute_time[i]))
      return fail(SWIFT_EINVAL, "compute_time[%lld] must be finite and >= 0", (long long)i);
  for (int64_t i = 0; i + 1 < n_machines; ++i)
    if (!(message_bytes[i] >= 0) || !std::isfinite(message_bytes[i]))
      return fail(SWIFT_EINVAL, "message_bytes[%lld] must be finite and >= 0", (long long)i);
  return guarded([&]() -> int {
    const LoggingGroups r = plan_logging_groups(n_machines, compute_time, message_bytes, checkpoint_interval, bandwidth,
                                                storage_limit, parallel_recovery != 0);
    memcpy(group_of, r.group_of.data(), (size_t)n_machines * sizeof(int32_t));
    if (storage_out) *storage_out = r.storage;
    if (recovery_out) *recovery_out = r.recovery;
    return SWIFT_OK;
  });
}

int swift_arena_layout(int64_t n, const int64_t *numel, int32_t grad_dtype, int32_t with_v, int64_t *offsets,
                       int64_t *total_bytes) {
  if (n < 0 || n > (int64_t)0x7fffffff || (n > 0 && (!numel || !offsets)))
    return fail(SWIFT_EINVAL, "arena_layout: bad n, numel or offsets");
  if (grad_dtype != SWIFT_F32 && grad_dtype != SWIFT_BF16) return fail(SWIFT_EINVAL, "arena_layout: unknown gradient dtype %d", grad_dtype);
  const int streams = with_v > 0 ? 4 : (with_v == 0 ? 3 : 2);
  int64_t off = 0;
  for (int64_t i = 0; i < n; ++i) {
    if (numel[i] < 0 || numel[i] > kMaxNumel) return fail(SWIFT_EINVAL, "arena_layout: numel[%lld] is negative or beyond 2^40", (long long)i);
    for (int k = 0; k < streams; ++k) {
      const int64_t bytes = numel[i] * ((k == 1 && grad_dtype == SWIFT_BF16) ? 2 : 4);
      offsets[i * streams + k] = off;
      // 1 MiB and more: round up to 8 KiB, then 2 KiB on top, so that consecutive buffers start an odd multiple
      // of 2 KiB apart; smaller buffers are only kept 256-byte aligned
      off += bytes < (1 << 20) ? (bytes + 255) / 256 * 256 : (bytes + 8191) / 8192 * 8192 + 2048;
    }
  }
  if (total_bytes) *total_bytes = off;
  return SWIFT_OK;
}

int swift_cache_stats(int64_t *n_lists, int64_t *device_bytes) {
  int64_t n = 0, bytes = 0;
  {
    std::lock_guard<std::mutex> lock(g_plan_mu);
    if (g_plans)
      for (const auto &p : g_plans->lru) {
        ++n;
        bytes += (int64_t)p->dev_bytes;
      }
  }
  if (n_lists) *n_lists = n;
  if (device_bytes) *device_bytes = bytes;
  return SWIFT_OK;
}

int swift_cache_trim(int64_t max_device_bytes) {
  if (max_device_bytes < 0) return fail(SWIFT_EINVAL, "cache_trim: max_device_bytes must be >= 0");
  std::list<std::shared_ptr<Plan>> drop;
  {
    std::lock_guard<std::mutex> lock(g_plan_mu);
    if (g_plans) {
      int64_t bytes = 0;
      for (const auto &p : g_plans->lru) bytes += (int64_t)p->dev_bytes;
      // least recently used first; plans that a captured graph may replay stay
      for (auto it = g_plans->lru.end(); bytes > max_device_bytes && it != g_plans->lru.begin();) {
        --it;
        if ((*it)->pinned) continue;
        bytes -= (int64_t)(*it)->dev_bytes;
        g_plans->index.erase((*it)->key);
        drop.push_back(*it);
        it = g_plans->lru.erase(it);
      }
    }
  }
  drop.clear();   // ~Plan frees (and thereby synchronises) on each plan's device
  return SWIFT_OK;
}

int swift_shutdown(void) {
  std::list<std::shared_ptr<Plan>> drop;
  {
    std::lock_guard<std::mutex> lock(g_plan_mu);
    if (g_plans) {
      drop.swap(g_plans->lru);
      g_plans->index.clear();
    }
  }
  drop.clear();   // ~Plan frees (and thereby synchronises) on each plan's device
  return SWIFT_OK;
}

const char *swift_last_error(void) { return g_last_error.c_str(); }

}  // extern "C"
