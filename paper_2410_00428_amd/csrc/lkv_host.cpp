// Host side of liblkv: context life cycle, the layer-wise block allocator and block tables
// (paper Sections 3.2.1 and 3.2.2), and the stream/event orchestration of offload and reload
// (Section 4).  All arithmetic on KV data happens in the kernels; this file only validates,
// keeps the logical state and enqueues.
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <thread>

#include "lkv_internal.hpp"

namespace {

thread_local std::string g_create_error;

lkv_status fail(const lkv_ctx *c, lkv_status st, const char *fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  if (c) c->err = buf; else g_create_error = buf;
  return st;
}

#define LKV_HIP(c, call)                                                                   \
  do {                                                                                     \
    hipError_t e_ = (call);                                                                \
    if (e_ != hipSuccess)                                                                  \
      return fail((c), LKV_ERR_DEVICE, "%s failed: %s", #call, hipGetErrorString(e_));      \
  } while (0)

hipEvent_t &event_of(lkv_ctx *c, int32_t layer, int32_t ev) { return c->events[(size_t)layer * 4 + ev]; }

lkv_status record_event(lkv_ctx *c, int32_t layer, int32_t ev, hipStream_t s) {
  LKV_HIP(c, hipEventRecord(event_of(c, layer, ev), s));
  c->event_recorded[(size_t)layer * 4 + ev] = 1;
  return LKV_OK;
}

lkv_status wait_event(lkv_ctx *c, int32_t layer, int32_t ev, hipStream_t s) {
  uint8_t &pending = c->event_recorded[(size_t)layer * 4 + ev];
  if (!pending) return LKV_OK;
  // an event that has already happened needs no wait packet in the stream (and is forgotten)
  hipError_t q = hipEventQuery(event_of(c, layer, ev));
  if (q == hipSuccess) {
    pending = 0;
    return LKV_OK;
  }
  if (q != hipErrorNotReady) return fail(c, LKV_ERR_DEVICE, "hipEventQuery failed: %s", hipGetErrorString(q));
  (void)hipGetLastError();  // "not ready" is an answer, not an error: do not leave it for the next launch check
  LKV_HIP(c, hipStreamWaitEvent(s, event_of(c, layer, ev), 0));
  return LKV_OK;
}

bool bad_layer(const lkv_ctx *c, int32_t layer) { return layer < 0 || layer >= c->cfg.num_layers; }

lkv_status staging_create(lkv_ctx *c, lkv::Staging &st, bool twin) {
  LKV_HIP(c, hipMalloc((void **)&st.buf, (size_t)(c->staging_blocks * c->block_bytes)));
  if (twin) {
    LKV_HIP(c, hipMalloc((void **)&st.buf2, (size_t)(c->staging_blocks * c->block_bytes)));
    for (auto &e : st.twin_gathered) LKV_HIP(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
  }
  size_t ids_bytes = sizeof(int32_t) * (size_t)c->staging_blocks * lkv::Staging::kSlots;
  LKV_HIP(c, hipMalloc((void **)&st.ids_dev, ids_bytes));
  LKV_HIP(c, hipHostMalloc((void **)&st.ids_pinned, ids_bytes, hipHostMallocDefault));
  for (auto &e : st.slot_done) LKV_HIP(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
  LKV_HIP(c, hipEventCreateWithFlags(&st.buf_free, hipEventDisableTiming));
  for (auto &e : st.copy_done) LKV_HIP(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
  LKV_HIP(c, hipStreamCreateWithFlags(&st.aux, hipStreamNonBlocking));  // default priority
  LKV_HIP(c, hipEventCreateWithFlags(&st.entry, hipEventDisableTiming));
  for (auto &e : st.half_kernel) LKV_HIP(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
  return LKV_OK;
}

void staging_destroy(lkv::Staging &st) {
  if (st.buf) (void)hipFree(st.buf);
  if (st.buf2) (void)hipFree(st.buf2);
  for (auto &e : st.twin_gathered)
    if (e) (void)hipEventDestroy(e);
  if (st.ids_dev) (void)hipFree(st.ids_dev);
  if (st.ids_pinned) (void)hipHostFree(st.ids_pinned);
  for (auto &e : st.slot_done)
    if (e) (void)hipEventDestroy(e);
  if (st.buf_free) (void)hipEventDestroy(st.buf_free);
  for (auto &e : st.copy_done)
    if (e) (void)hipEventDestroy(e);
  if (st.entry) (void)hipEventDestroy(st.entry);
  for (auto &e : st.half_kernel)
    if (e) (void)hipEventDestroy(e);
  if (st.aux) (void)hipStreamDestroy(st.aux);
  st = lkv::Staging{};
}

// Puts ids[0..n) into the next slot of the ring and enqueues their copy to the device.
lkv_status stage_ids(lkv_ctx *c, lkv::Staging &st, const int32_t *ids, int64_t n, hipStream_t s,
                     int *slot_out) {
  int slot = st.next_slot;
  st.next_slot = (st.next_slot + 1) % lkv::Staging::kSlots;
  // the slot's previous kernel must have consumed its ids before the host overwrites them
  LKV_HIP(c, hipEventSynchronize(st.slot_done[slot]));
  int32_t *pinned = st.ids_pinned + (size_t)slot * c->staging_blocks;
  int32_t *dev = st.ids_dev + (size_t)slot * c->staging_blocks;
  std::memcpy(pinned, ids, sizeof(int32_t) * (size_t)n);
  LKV_HIP(c, hipMemcpyAsync(dev, pinned, sizeof(int32_t) * (size_t)n, hipMemcpyHostToDevice, s));
  *slot_out = slot;
  return LKV_OK;
}

// Host-link copies are paced: with a deep backlog of queued copies the runtime was measured to move
// later ones at a quarter of the link rate, so the host waits until at most kMaxInFlight are queued.
lkv_status pace_copy(lkv_ctx *c, lkv::Staging &st) {
  if (st.copies_issued >= lkv::Staging::kMaxInFlight)
    LKV_HIP(c, hipEventSynchronize(st.copy_done[(st.copies_issued - lkv::Staging::kMaxInFlight) % lkv::Staging::kCopyRing]));
  return LKV_OK;
}
lkv_status copy_issued(lkv_ctx *c, lkv::Staging &st, hipStream_t s) {
  LKV_HIP(c, hipEventRecord(st.copy_done[st.copies_issued % lkv::Staging::kCopyRing], s));
  st.copies_issued += 1;
  return LKV_OK;
}

// The same pacing for the unit copies of the pageable calls, on the ring unit events (see Staging).
lkv_status pace_unit_copy(lkv_ctx *c, lkv::Staging &st) {
  if (st.copies_issued >= lkv::Staging::kMaxInFlight) {
    hipEvent_t ev = st.unit_copies[(st.copies_issued - lkv::Staging::kMaxInFlight) % lkv::Staging::kCopyRing];
    if (ev) LKV_HIP(c, hipEventSynchronize(ev));
  }
  return LKV_OK;
}
void unit_copy_issued(lkv::Staging &st, hipEvent_t unit_event) {
  st.unit_copies[st.copies_issued % lkv::Staging::kCopyRing] = unit_event;
  st.copies_issued += 1;
}

// Section 3.2.3: ask before every unit whether the link is taken by traffic that must not be delayed.
void link_gate(lkv_ctx *c) {
  if (!c->gate_busy) return;
  for (int32_t k = 0; k < c->gate_max_checks && c->gate_busy(c->gate_user); ++k) {
    c->stats.gate_busy_answers += 1;
    if (c->gate_delay_us > 0) std::this_thread::sleep_for(std::chrono::microseconds(c->gate_delay_us));
  }
}

void tier_destroy(lkv_ctx *c) {  // the device is idle when this is called
  c->tier.stop();
  for (lkv::Staging *sg : {&c->d2h, &c->h2d}) {  // forget the ring unit events that are destroyed below
    for (auto &e : sg->unit_copies) e = nullptr;
    for (int h = 0; h < 2; ++h) {
      sg->half_copy[h] = nullptr;
      sg->half_used[h] = false;
    }
  }
  for (auto &e : c->unit_ev)
    if (e) (void)hipEventDestroy(e);
  c->unit_ev.clear();
  if (c->ring) (void)hipHostFree(c->ring);
  c->ring = nullptr;
  c->unit_blocks = 0;
}

lkv_status tier_build(lkv_ctx *c, int64_t unit_bytes, int32_t units, int32_t threads) {
  // defaults from a sweep on the target: 32 MiB units reach 94% of the pinned-copy rate (16 MiB: 89%, 4 MiB: 68%;
  // every unit pays one gather launch and one copy start), 4 threads keep up with the link (one does not)
  if (unit_bytes <= 0) unit_bytes = (int64_t)32 << 20;
  if (units <= 0) units = 4;
  if (threads <= 0) threads = 4;
  int64_t blocks = unit_bytes / c->block_bytes;
  if (blocks < 1) blocks = 1;
  // two units of device staging, so that the kernel of one unit and the link copy of the other overlap
  if (blocks > c->staging_blocks / 2) blocks = c->staging_blocks / 2 > 0 ? c->staging_blocks / 2 : 1;
  if (c->tier.running()) {
    if (!c->tier.wait_all()) return fail(c, LKV_ERR_DEVICE, "host tier: waiting for a device copy failed");
    LKV_HIP(c, hipDeviceSynchronize());
    tier_destroy(c);
  }
  LKV_HIP(c, hipHostMalloc((void **)&c->ring, (size_t)(blocks * c->block_bytes * units), hipHostMallocDefault));
  c->unit_ev.assign((size_t)units, nullptr);
  for (auto &e : c->unit_ev) LKV_HIP(c, hipEventCreateWithFlags(&e, hipEventDisableTiming));
  c->unit_blocks = blocks;
  c->tier.start(c->ring, blocks * c->block_bytes, units, threads, c->cfg.num_layers);
  return LKV_OK;
}

lkv_status tier_ensure(lkv_ctx *c) { return c->tier.running() ? LKV_OK : tier_build(c, 0, 0, 0); }

// The job a worker runs once the link copy of ring unit u (recorded in unit_ev[u]) has finished.
lkv::HostTier::Job unit_job(lkv_ctx *c, int u) {
  lkv::HostTier::Job j;
  hipEvent_t ev = c->unit_ev[(size_t)u];
  int dev = c->device;
  j.ready = [ev, dev] { return hipSetDevice(dev) == hipSuccess && hipEventSynchronize(ev) == hipSuccess; };
  j.unit = u;
  return j;
}

lkv_status check_ids(const lkv_ctx *c, const int32_t *ids, int64_t n) {
  for (int64_t i = 0; i < n; ++i)
    if (ids[i] < 0 || ids[i] >= c->cfg.num_pool_blocks)
      return fail(c, LKV_ERR_INVALID_ARG, "block_ids[%lld] = %d is outside the pool (%lld blocks)",
                  (long long)i, ids[i], (long long)c->cfg.num_pool_blocks);
  return LKV_OK;
}

// Adds one finished (start, stop) pair to the statistics and hands its events back to the free list.
void fold_one(lkv_ctx *c, const lkv_ctx::Timed &t, float ms) {
  const int64_t ns = (int64_t)((double)ms * 1e6);
  switch (t.kind) {
    case lkv_ctx::kTimedUnpack:
      c->stats.unpack_kernel_ns += ns;
      c->stats.unpack_kernel_bytes += t.bytes;
      break;
    case lkv_ctx::kTimedPack:
      c->stats.pack_kernel_ns += ns;
      c->stats.pack_kernel_bytes += t.bytes;
      break;
    case lkv_ctx::kTimedWrite:
      c->stats.write_kernel_ns += ns;
      c->stats.write_kernel_launches += 1;
      c->stats.write_kernel_bytes += t.bytes;
      break;
    case lkv_ctx::kTimedPrefill:
      c->stats.prefill_kernel_ns += ns;
      c->stats.prefill_kernel_launches += 1;
      break;
    default:
      c->stats.decode_kernel_ns += ns;
      c->stats.decode_kernel_launches += 1;
      break;
  }
  c->spare_events.push_back(t.a);
  c->spare_events.push_back(t.b);
}

// Folds the profiled launches into the statistics: all of them (wait = true: blocks until each has finished), or
// only those that have finished already (wait = false), the others staying in the list.
lkv_status fold_timed(lkv_ctx *c, bool wait) {
  size_t kept = 0;
  for (size_t i = 0; i < c->timed.size(); ++i) {
    const lkv_ctx::Timed t = c->timed[i];
    if (wait) {
      LKV_HIP(c, hipEventSynchronize(t.b));
    } else if (hipEventQuery(t.b) != hipSuccess) {
      (void)hipGetLastError();  // "not ready" is an answer, not an error: do not leave it for the next launch check
      c->timed[kept++] = t;
      continue;
    }
    float ms = 0.f;
    LKV_HIP(c, hipEventElapsedTime(&ms, t.a, t.b));
    fold_one(c, t, ms);
  }
  c->timed.resize(kept);
  return LKV_OK;
}

// Kernel profiling: a region (one launch, or a launch and the merge kernel behind it) gets a pair of timing events
// from a small free list; the launchers attach them to the region's kernels (launch_timed).  A transfer of many
// units profiles thousands of launches between two reads of the statistics: finished pairs are folded on the
// way, whenever kTimedBacklog more have been added, so that the number of live events stays bounded.
constexpr size_t kTimedBacklog = 512;
lkv_status timed_begin(lkv_ctx *c, hipStream_t, hipEvent_t *a) {
  *a = nullptr;
  if (!c->profiling) return LKV_OK;
  for (hipEvent_t *e : {&c->prof_start, &c->prof_stop}) {
    if (c->spare_events.empty()) {
      LKV_HIP(c, hipEventCreate(e));
    } else {
      *e = c->spare_events.back();
      c->spare_events.pop_back();
    }
  }
  c->prof_start_used = c->prof_stop_used = false;
  *a = c->prof_start;
  return LKV_OK;
}

lkv_status timed_end(lkv_ctx *c, hipStream_t, hipEvent_t a, int64_t bytes, int kind) {
  if (!a) return LKV_OK;
  hipEvent_t b = c->prof_stop;
  const bool launched = c->prof_start_used && c->prof_stop_used;
  c->prof_start = c->prof_stop = nullptr;
  if (!launched) {  // the region launched nothing (or failed half way): no time to read
    c->spare_events.push_back(a);
    c->spare_events.push_back(b);
    return LKV_OK;
  }
  c->timed.push_back({a, b, bytes, kind});
  if (c->timed.size() >= c->timed_fold_at) {
    if (lkv_status st = fold_timed(c, false)) return st;
    c->timed_fold_at = c->timed.size() + kTimedBacklog;
  }
  return LKV_OK;
}

constexpr int64_t kDefaultDecodeWorkspace = (int64_t)32 << 20;

}  // namespace

extern "C" {

static lkv_status create_impl(const lkv_config *cfg, lkv_ctx **out, bool with_device) {
  if (!cfg || !out) return fail(nullptr, LKV_ERR_INVALID_ARG, "lkv_create: NULL argument");
  *out = nullptr;
  if (cfg->num_layers <= 0 || cfg->num_q_heads <= 0 || cfg->num_kv_heads <= 0 || cfg->head_dim <= 0 ||
      cfg->block_size <= 0 || cfg->num_pool_blocks <= 0)
    return fail(nullptr, LKV_ERR_INVALID_ARG, "lkv_create: sizes must be positive");
  if (cfg->num_q_heads % cfg->num_kv_heads)
    return fail(nullptr, LKV_ERR_INVALID_ARG, "lkv_create: num_kv_heads must divide num_q_heads");
  if (cfg->dtype != LKV_F32 && cfg->dtype != LKV_BF16 && cfg->dtype != LKV_FP8_E4M3)
    return fail(nullptr, LKV_ERR_INVALID_ARG, "lkv_create: unknown dtype %d", cfg->dtype);
  if (cfg->dtype == LKV_FP8_E4M3 && (!(cfg->k_scale >= 0.f) || !(cfg->v_scale >= 0.f) || std::isinf(cfg->k_scale) ||
                                     std::isinf(cfg->v_scale)))
    return fail(nullptr, LKV_ERR_INVALID_ARG, "lkv_create: k_scale and v_scale must be finite and positive (0 = 1.0)");
  if (cfg->num_pool_blocks > INT32_MAX)
    return fail(nullptr, LKV_ERR_INVALID_ARG, "lkv_create: block ids are 32-bit");
  if (cfg->decode_partition < 0 || cfg->decode_partition % 64)
    return fail(nullptr, LKV_ERR_INVALID_ARG, "lkv_create: decode_partition must be a multiple of 64");
  int64_t elem = cfg->dtype == LKV_F32 ? 4 : cfg->dtype == LKV_BF16 ? 2 : 1;
  if ((cfg->head_dim * elem) % 16)
    return fail(nullptr, LKV_ERR_UNSUPPORTED, "lkv_create: head_dim*element size must be a multiple of 16 bytes");
  if (cfg->pool && ((uintptr_t)cfg->pool & 255))
    return fail(nullptr, LKV_ERR_INVALID_ARG, "lkv_create: pool must be 256-byte aligned");

  lkv_ctx *c = new (std::nothrow) lkv_ctx();
  if (!c) return fail(nullptr, LKV_ERR_HOST_MEMORY, "lkv_create: out of host memory");
  c->cfg = *cfg;
  c->elem = elem;
  c->row_bytes = cfg->head_dim * elem;
  c->in_row_bytes = cfg->head_dim * (cfg->dtype == LKV_F32 ? 4 : 2);
  if (cfg->dtype == LKV_FP8_E4M3) {
    c->k_scale = cfg->k_scale > 0.f ? cfg->k_scale : 1.f;
    c->v_scale = cfg->v_scale > 0.f ? cfg->v_scale : 1.f;
  }
  c->token_bytes = 2 * cfg->num_kv_heads * c->row_bytes;
  c->block_bytes = cfg->block_size * c->token_bytes;
  c->scale = cfg->softmax_scale != 0.f ? cfg->softmax_scale : 1.0f / std::sqrt((float)cfg->head_dim);
  int64_t staging = cfg->staging_bytes > 0 ? cfg->staging_bytes : (int64_t)256 << 20;
  c->staging_blocks = staging / c->block_bytes;
  if (c->staging_blocks < 1) c->staging_blocks = 1;
  if (c->staging_blocks > cfg->num_pool_blocks) c->staging_blocks = cfg->num_pool_blocks;

  auto bail = [&](lkv_status st) {
    g_create_error = c->err;
    lkv_destroy(c);
    return st;
  };
  c->free_list.resize((size_t)cfg->num_pool_blocks);
  for (int64_t i = 0; i < cfg->num_pool_blocks; ++i)
    c->free_list[(size_t)i] = (int32_t)(cfg->num_pool_blocks - 1 - i);  // id 0 handed out first
  if (!with_device) {
    c->logical_only = true;
    *out = c;
    return LKV_OK;
  }
  hipError_t e = hipGetDevice(&c->device);
  if (e != hipSuccess) {
    c->err = std::string("hipGetDevice failed: ") + hipGetErrorString(e);
    return bail(LKV_ERR_DEVICE);
  }
  e = lkv::static_scratch_init(c->device);  // address of this device's fixed decode scratch, looked up once
  if (e != hipSuccess) {
    c->err = std::string("hipGetSymbolAddress of the fixed decode scratch failed: ") + hipGetErrorString(e);
    return bail(LKV_ERR_DEVICE);
  }
  if (cfg->pool) {
    c->pool = (char *)cfg->pool;
  } else {
    e = hipMalloc((void **)&c->pool, (size_t)(cfg->num_pool_blocks * c->block_bytes));
    if (e != hipSuccess) {
      c->pool = nullptr;
      c->err = std::string("hipMalloc of the pool failed: ") + hipGetErrorString(e);
      return bail(LKV_ERR_DEVICE);
    }
    c->owns_pool = true;
  }
  lkv_status st = staging_create(c, c->d2h, true);
  if (st == LKV_OK) st = staging_create(c, c->h2d, false);
  if (st != LKV_OK) return bail(st);
  c->events.assign((size_t)cfg->num_layers * 4, nullptr);
  c->event_recorded.assign((size_t)cfg->num_layers * 4, 0);
  for (auto &ev : c->events) {
    e = hipEventCreateWithFlags(&ev, hipEventDisableTiming);
    if (e != hipSuccess) {
      c->err = std::string("hipEventCreate failed: ") + hipGetErrorString(e);
      return bail(LKV_ERR_DEVICE);
    }
  }
  // the split-K workspace of decode attention: allocated here (and by lkv_reserve_decode_workspace), never by the
  // hot call
  e = hipMalloc((void **)&c->ws, (size_t)kDefaultDecodeWorkspace);
  if (e != hipSuccess) {
    c->ws = nullptr;
    c->err = std::string("hipMalloc of the decode workspace failed: ") + hipGetErrorString(e);
    return bail(LKV_ERR_DEVICE);
  }
  c->ws_bytes = kDefaultDecodeWorkspace;
  e = hipEventCreateWithFlags(&c->ws_done, hipEventDisableTiming);
  if (e != hipSuccess) {
    c->err = std::string("hipEventCreate failed: ") + hipGetErrorString(e);
    return bail(LKV_ERR_DEVICE);
  }
  *out = c;
  return LKV_OK;
}

lkv_status lkv_create(const lkv_config *cfg, lkv_ctx **out) { return create_impl(cfg, out, true); }
lkv_status lkv_create_logical(const lkv_config *cfg, lkv_ctx **out) { return create_impl(cfg, out, false); }

void lkv_destroy(lkv_ctx *c) {
  if (!c) return;
  if (c->logical_only) {
    delete c;
    return;
  }
  (void)hipDeviceSynchronize();
  tier_destroy(c);
  staging_destroy(c->d2h);
  staging_destroy(c->h2d);
  for (auto &ev : c->events)
    if (ev) (void)hipEventDestroy(ev);
  for (auto &t : c->timed) {
    (void)hipEventDestroy(t.a);
    (void)hipEventDestroy(t.b);
  }
  for (auto &e : c->spare_events) (void)hipEventDestroy(e);
  if (c->ws) (void)hipFree(c->ws);
  if (c->ws_done) (void)hipEventDestroy(c->ws_done);
  if (c->owns_pool && c->pool) (void)hipFree(c->pool);
  delete c;
}

const char *lkv_last_error(const lkv_ctx *c) { return c ? c->err.c_str() : g_create_error.c_str(); }

lkv_status lkv_pool_info(const lkv_ctx *c, void **pool, int64_t *bytes, int64_t *block_bytes) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (pool) *pool = c->pool;
  if (bytes) *bytes = c->cfg.num_pool_blocks * c->block_bytes;
  if (block_bytes) *block_bytes = c->block_bytes;
  return LKV_OK;
}

// ---------------------------------------------------------------- logical state
lkv_status lkv_pool_reset(lkv_ctx *c, const int32_t *free_order, int64_t n) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (!free_order || n != c->cfg.num_pool_blocks)
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_pool_reset: free_order must list all %lld blocks",
                (long long)c->cfg.num_pool_blocks);
  std::vector<uint8_t> seen((size_t)n, 0);
  for (int64_t i = 0; i < n; ++i) {
    int32_t b = free_order[i];
    if (b < 0 || b >= n || seen[(size_t)b])
      return fail(c, LKV_ERR_INVALID_ARG, "lkv_pool_reset: free_order is not a permutation (entry %lld)", (long long)i);
    seen[(size_t)b] = 1;
  }
  c->layers.clear();
  c->free_list.resize((size_t)n);
  for (int64_t i = 0; i < n; ++i) c->free_list[(size_t)(n - 1 - i)] = free_order[i];
  return LKV_OK;
}

lkv_status lkv_alloc_layer_blocks(lkv_ctx *c, int64_t seq, int32_t layer, int64_t num_tokens_total) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (bad_layer(c, layer) || num_tokens_total < 0)
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_alloc_layer_blocks: bad layer %d or token count %lld", layer,
                (long long)num_tokens_total);
  int64_t bs = c->cfg.block_size;
  int64_t want = (num_tokens_total + bs - 1) / bs;
  auto it = c->layers.find({seq, layer});
  int64_t have = it == c->layers.end() ? 0 : (int64_t)it->second.table.size();
  int64_t grow = want > have ? want - have : 0;
  if (grow > (int64_t)c->free_list.size())
    return fail(c, LKV_ERR_NO_BLOCKS, "lkv_alloc_layer_blocks: need %lld blocks, %lld free", (long long)grow,
                (long long)c->free_list.size());
  lkv::LayerState &st = c->layers[{seq, layer}];
  st.table.reserve((size_t)(have + grow));
  for (int64_t i = 0; i < grow; ++i) {
    st.table.push_back(c->free_list.back());
    c->free_list.pop_back();
  }
  st.residency = LKV_RES_GPU;
  return LKV_OK;
}

lkv_status lkv_free_layer_blocks(lkv_ctx *c, int64_t seq, int32_t layer, int32_t to_host) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (bad_layer(c, layer)) return fail(c, LKV_ERR_INVALID_ARG, "lkv_free_layer_blocks: bad layer %d", layer);
  auto it = c->layers.find({seq, layer});
  if (it == c->layers.end() || it->second.residency != LKV_RES_GPU)
    return fail(c, LKV_ERR_NOT_RESIDENT, "lkv_free_layer_blocks: (seq %lld, layer %d) holds no blocks",
                (long long)seq, layer);
  for (int32_t b : it->second.table) c->free_list.push_back(b);
  if (to_host) {
    it->second.table.clear();
    it->second.residency = LKV_RES_HOST;
  } else {
    c->layers.erase(it);
  }
  return LKV_OK;
}

lkv_status lkv_free_seq(lkv_ctx *c, int64_t seq) {
  if (!c) return LKV_ERR_INVALID_ARG;
  for (int32_t layer = 0; layer < c->cfg.num_layers; ++layer) {
    auto it = c->layers.find({seq, layer});
    if (it == c->layers.end()) continue;
    for (int32_t b : it->second.table) c->free_list.push_back(b);
    c->layers.erase(it);
  }
  return LKV_OK;
}

lkv_status lkv_get_block_table(const lkv_ctx *c, int64_t seq, int32_t layer, int32_t *out, int64_t cap, int64_t *n) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (bad_layer(c, layer) || !n || cap < 0) return fail(c, LKV_ERR_INVALID_ARG, "lkv_get_block_table: bad argument");
  auto it = c->layers.find({seq, layer});
  if (it == c->layers.end()) {
    *n = 0;
    return LKV_OK;
  }
  if (it->second.residency == LKV_RES_HOST) {
    *n = 0;
    return fail(c, LKV_ERR_NOT_RESIDENT, "lkv_get_block_table: (seq %lld, layer %d) is on the host", (long long)seq, layer);
  }
  *n = (int64_t)it->second.table.size();
  if (*n > cap || (*n && !out))
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_get_block_table: table has %lld entries, capacity %lld", (long long)*n,
                (long long)cap);
  if (*n) std::memcpy(out, it->second.table.data(), sizeof(int32_t) * (size_t)*n);
  return LKV_OK;
}

lkv_status lkv_build_slot_mapping(const lkv_ctx *c, int64_t seq, int32_t layer, int64_t pos0, int64_t count,
                                  int64_t *out) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (bad_layer(c, layer) || pos0 < 0 || count < 0 || (count && !out))
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_build_slot_mapping: bad argument");
  auto it = c->layers.find({seq, layer});
  if (it == c->layers.end() || it->second.residency != LKV_RES_GPU)
    return fail(c, LKV_ERR_NOT_RESIDENT, "lkv_build_slot_mapping: (seq %lld, layer %d) is not in the pool",
                (long long)seq, layer);
  const auto &t = it->second.table;
  int64_t bs = c->cfg.block_size;
  if ((pos0 + count + bs - 1) / bs > (int64_t)t.size())
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_build_slot_mapping: positions %lld..%lld exceed the %zu allocated blocks",
                (long long)pos0, (long long)(pos0 + count), t.size());
  for (int64_t i = 0; i < count; ++i) {
    int64_t p = pos0 + i;
    out[i] = (int64_t)t[(size_t)(p / bs)] * bs + p % bs;
  }
  return LKV_OK;
}

lkv_status lkv_layer_residency(const lkv_ctx *c, int64_t seq, int32_t layer, int32_t *out) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (bad_layer(c, layer) || !out) return fail(c, LKV_ERR_INVALID_ARG, "lkv_layer_residency: bad argument");
  auto it = c->layers.find({seq, layer});
  int32_t res = it == c->layers.end() ? (int32_t)LKV_RES_NONE : it->second.residency;
  if (!c->logical_only && (res == LKV_RES_HOST || res == LKV_RES_GPU)) {
    // a host layer whose copy out (or whose CPU copies behind the pinned ring) has not finished, a GPU layer whose
    // reload has not finished: the transfer's event answers without blocking
    const int32_t ev = res == LKV_RES_HOST ? LKV_EV_OFFLOADED : LKV_EV_RELOADED;
    const size_t idx = (size_t)layer * 4 + ev;
    bool pending = false;
    if (c->event_recorded[idx]) {
      const hipError_t q = hipEventQuery(c->events[idx]);
      if (q == hipErrorNotReady) {
        (void)hipGetLastError();
        pending = true;
      } else if (q != hipSuccess) {
        return fail(c, LKV_ERR_DEVICE, "lkv_layer_residency: hipEventQuery failed: %s", hipGetErrorString(q));
      }
    }
    if (!pending && res == LKV_RES_HOST && const_cast<lkv_ctx *>(c)->tier.running() && const_cast<lkv_ctx *>(c)->tier.busy_key(layer)) pending = true;
    if (pending) res = LKV_RES_IN_FLIGHT;
  }
  *out = res;
  return LKV_OK;
}

int64_t lkv_num_free_blocks(const lkv_ctx *c) { return c ? (int64_t)c->free_list.size() : -1; }

lkv_status lkv_plan_retained_layers(int32_t num_layers, int32_t x, int32_t *mask) {
  if (num_layers <= 0 || x < 0 || x > num_layers || !mask) return LKV_ERR_INVALID_ARG;
  // The retained share after l layers is the integer part of l*x/L; a layer is retained when
  // taking it raises that share, which spaces the retained layers evenly.
  int64_t before = 0;
  for (int32_t l = 0; l < num_layers; ++l) {
    int64_t after = ((int64_t)(l + 1) * x) / num_layers;
    mask[l] = after > before ? 1 : 0;
    before = after;
  }
  return LKV_OK;
}

// ---------------------------------------------------------------- device hot path
lkv_status lkv_write_kv(lkv_ctx *c, int32_t layer, const void *K, const void *V, const int64_t *slot_mapping,
                        int64_t num_tokens, void *stream) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_write_kv: this context has no device resources (lkv_create_logical)");
  if (bad_layer(c, layer) || num_tokens < 0) return fail(c, LKV_ERR_INVALID_ARG, "lkv_write_kv: bad layer or count");
  hipStream_t s = (hipStream_t)stream;
  // a reload of this layer that is still in flight rewrites whole blocks: stay behind it
  if (lkv_status st = wait_event(c, layer, LKV_EV_RELOADED, s)) return st;
  if (num_tokens > 0) {
    if (!K || !V || !slot_mapping) return fail(c, LKV_ERR_INVALID_ARG, "lkv_write_kv: NULL pointer");
    if (((uintptr_t)K | (uintptr_t)V) & 15) return fail(c, LKV_ERR_INVALID_ARG, "lkv_write_kv: K and V must be 16-byte aligned");
    hipEvent_t t0;
    if (lkv_status st = timed_begin(c, s, &t0)) return st;
    LKV_HIP(c, lkv::launch_write_kv(c, K, V, slot_mapping, num_tokens, s));
    if (lkv_status st = timed_end(c, s, t0, num_tokens * (2 * c->cfg.num_kv_heads * c->in_row_bytes + c->token_bytes), lkv_ctx::kTimedWrite)) return st;
  }
  c->stats.write_kv_calls += 1;
  c->stats.write_kv_bytes += num_tokens * c->token_bytes;
  return record_event(c, layer, LKV_EV_KV_WRITTEN, s);
}

lkv_status lkv_prefill_attention(lkv_ctx *c, int32_t layer, const void *Q, const void *K, const void *V, void *O,
                                 const int32_t *cu_seqlens, int32_t num_seqs, int32_t max_seqlen,
                                 int64_t total_tokens, int32_t causal, void *stream) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_prefill_attention: this context has no device resources (lkv_create_logical)");
  if (bad_layer(c, layer) || num_seqs < 0 || max_seqlen < 0 || total_tokens < 0)
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_prefill_attention: bad layer or count");
  if (!lkv::prefill_supported(c))
    return fail(c, LKV_ERR_UNSUPPORTED, "lkv_prefill_attention: head_dim %d with dtype %d is not built", c->cfg.head_dim,
                c->cfg.dtype);
  if (num_seqs == 0 || max_seqlen == 0 || total_tokens == 0) return LKV_OK;
  if (!Q || !K || !V || !O || !cu_seqlens) return fail(c, LKV_ERR_INVALID_ARG, "lkv_prefill_attention: NULL pointer");
  if (((uintptr_t)Q | (uintptr_t)K | (uintptr_t)V | (uintptr_t)O) & 15)
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_prefill_attention: tensors must be 16-byte aligned");
  hipEvent_t t0;
  if (lkv_status st = timed_begin(c, (hipStream_t)stream, &t0)) return st;
  LKV_HIP(c, lkv::launch_prefill(c, Q, K, V, O, cu_seqlens, num_seqs, max_seqlen, total_tokens, causal, (hipStream_t)stream));
  if (lkv_status st = timed_end(c, (hipStream_t)stream, t0, 0, lkv_ctx::kTimedPrefill)) return st;
  c->stats.prefill_calls += 1;
  return LKV_OK;
}

lkv_status lkv_pack_layer_blocks(lkv_ctx *c, int32_t layer, const int32_t *block_ids, int64_t n, void *pinned_dst,
                                 void *stream) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_pack_layer_blocks: this context has no device resources (lkv_create_logical)");
  if (bad_layer(c, layer) || n < 0 || (n && (!block_ids || !pinned_dst)))
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_pack_layer_blocks: bad argument");
  if (lkv_status st = check_ids(c, block_ids, n)) return st;
  hipStream_t s = (hipStream_t)stream;
  lkv::Staging &sg = c->d2h;
  // The gathers run on the helper stream, behind everything the caller's stream holds at this point, behind the
  // layer's write and (after a pageable transfer) behind the last user of the staging memory; the link copies run
  // on the caller's stream, each behind its gather.  Two staging buffers alternate from chunk to chunk AND from
  // call to call: the gather of a chunk overlaps the copy of the one before it, so the link is busy back to back.
  LKV_HIP(c, hipEventRecord(sg.entry, s));
  LKV_HIP(c, hipStreamWaitEvent(sg.aux, sg.entry, 0));
  if (lkv_status st = wait_event(c, layer, LKV_EV_KV_WRITTEN, sg.aux)) return st;
  if (sg.last_user == 2 && sg.buf_used) LKV_HIP(c, hipStreamWaitEvent(sg.aux, sg.buf_free, 0));
  sg.last_user = 1;
  for (int64_t first = 0; first < n; first += c->staging_blocks) {
    int64_t m = n - first < c->staging_blocks ? n - first : c->staging_blocks;
    int slot;
    link_gate(c);
    const int b = (int)(sg.twin_chunks & 1);
    char *stage = b ? sg.buf2 : sg.buf;
    if (lkv_status st = stage_ids(c, sg, block_ids + first, m, sg.aux, &slot)) return st;
    if (sg.twin_used[b]) LKV_HIP(c, hipStreamWaitEvent(sg.aux, sg.twin_copied[b], 0));  // its last copy has left
    hipEvent_t t0;
    if (lkv_status st = timed_begin(c, sg.aux, &t0)) return st;
    LKV_HIP(c, lkv::launch_gather_blocks(c, sg.ids_dev + (size_t)slot * c->staging_blocks, m, stage, sg.aux));
    if (lkv_status st = timed_end(c, sg.aux, t0, 2 * m * c->block_bytes, lkv_ctx::kTimedPack)) return st;
    LKV_HIP(c, hipEventRecord(sg.slot_done[slot], sg.aux));
    LKV_HIP(c, hipEventRecord(sg.twin_gathered[b], sg.aux));
    if (first + m == n)
      if (lkv_status st = record_event(c, layer, LKV_EV_PACKED, sg.aux)) return st;
    LKV_HIP(c, hipStreamWaitEvent(s, sg.twin_gathered[b], 0));
    if (lkv_status st = pace_copy(c, sg)) return st;
    LKV_HIP(c, hipMemcpyAsync((char *)pinned_dst + first * c->block_bytes, stage, (size_t)(m * c->block_bytes),
                              hipMemcpyDeviceToHost, s));
    // one event record between two copies, no more (every packet between them costs link time): the pacing's
    // event of this copy also tells when the buffer may be gathered into again and when the staging memory is free
    sg.twin_copied[b] = sg.copy_done[sg.copies_issued % lkv::Staging::kCopyRing];
    if (lkv_status st = copy_issued(c, sg, s)) return st;
    sg.pack_last = sg.twin_copied[b];
    sg.twin_used[b] = true;
    sg.twin_chunks += 1;
    sg.buf_used = true;
  }
  if (n == 0)
    if (lkv_status st = record_event(c, layer, LKV_EV_PACKED, sg.aux)) return st;
  c->stats.pack_calls += 1;
  c->stats.pack_bytes += n * c->block_bytes;
  return record_event(c, layer, LKV_EV_OFFLOADED, s);
}

lkv_status lkv_unpack_layer_blocks(lkv_ctx *c, int32_t layer, const int32_t *block_ids, int64_t n,
                                   const void *pinned_src, void *stream) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_unpack_layer_blocks: this context has no device resources (lkv_create_logical)");
  if (bad_layer(c, layer) || n < 0 || (n && (!block_ids || !pinned_src)))
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_unpack_layer_blocks: bad argument");
  if (lkv_status st = check_ids(c, block_ids, n)) return st;
  hipStream_t s = (hipStream_t)stream;
  lkv::Staging &sg = c->h2d;
  for (int64_t first = 0; first < n; first += c->staging_blocks) {
    int64_t m = n - first < c->staging_blocks ? n - first : c->staging_blocks;
    int slot;
    link_gate(c);
    if (lkv_status st = stage_ids(c, sg, block_ids + first, m, s, &slot)) return st;
    if (sg.buf_used) LKV_HIP(c, hipStreamWaitEvent(s, sg.buf_free, 0));
    if (lkv_status st = pace_copy(c, sg)) return st;
    LKV_HIP(c, hipMemcpyAsync(sg.buf, (const char *)pinned_src + first * c->block_bytes, (size_t)(m * c->block_bytes),
                              hipMemcpyHostToDevice, s));
    if (lkv_status st = copy_issued(c, sg, s)) return st;
    hipEvent_t t0;
    if (lkv_status st = timed_begin(c, s, &t0)) return st;
    LKV_HIP(c, lkv::launch_scatter_blocks(c, sg.ids_dev + (size_t)slot * c->staging_blocks, m, sg.buf, s));
    if (lkv_status st = timed_end(c, s, t0, 2 * m * c->block_bytes, lkv_ctx::kTimedUnpack)) return st;
    LKV_HIP(c, hipEventRecord(sg.slot_done[slot], s));
    LKV_HIP(c, hipEventRecord(sg.buf_free, s));
    sg.buf_used = true;
  }
  c->stats.unpack_calls += 1;
  c->stats.unpack_bytes += n * c->block_bytes;
  return record_event(c, layer, LKV_EV_RELOADED, s);
}

lkv_status lkv_host_tier_config(lkv_ctx *c, int64_t unit_bytes, int32_t num_units, int32_t threads) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_host_tier_config: this context has no device resources (lkv_create_logical)");
  if (unit_bytes < 0 || num_units < 0 || threads < 0 || num_units > 1024 || threads > 64)
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_host_tier_config: bad argument");
  LKV_HIP(c, hipSetDevice(c->device));
  return tier_build(c, unit_bytes, num_units, threads);
}

lkv_status lkv_host_tier_synchronize(lkv_ctx *c, int32_t layer) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_host_tier_synchronize: this context has no device resources (lkv_create_logical)");
  if (layer < -1 || layer >= c->cfg.num_layers) return fail(c, LKV_ERR_INVALID_ARG, "lkv_host_tier_synchronize: bad layer");
  if (!c->tier.running()) return LKV_OK;
  bool ok = layer < 0 ? c->tier.wait_all() : c->tier.wait_key(layer);
  return ok ? LKV_OK : fail(c, LKV_ERR_DEVICE, "host tier: waiting for a device copy failed");
}

lkv_status lkv_set_link_gate(lkv_ctx *c, lkv_link_busy_fn busy, void *user, int64_t delay_us, int32_t max_checks) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (delay_us < 0 || max_checks < 0) return fail(c, LKV_ERR_INVALID_ARG, "lkv_set_link_gate: bad argument");
  c->gate_busy = busy;
  c->gate_user = user;
  c->gate_delay_us = delay_us;
  c->gate_max_checks = max_checks;
  return LKV_OK;
}

lkv_status lkv_offload_layer_pageable(lkv_ctx *c, int32_t layer, const int32_t *block_ids, int64_t n, void *host_dst,
                                      void *stream) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_offload_layer_pageable: this context has no device resources (lkv_create_logical)");
  if (bad_layer(c, layer) || n < 0 || (n && (!block_ids || !host_dst)))
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_offload_layer_pageable: bad argument");
  if (lkv_status st = check_ids(c, block_ids, n)) return st;
  if (lkv_status st = tier_ensure(c)) return st;
  // units of an earlier offload of this layer may still be on their way into the same buffer
  if (!c->tier.wait_key(layer)) return fail(c, LKV_ERR_DEVICE, "host tier: waiting for a device copy failed");
  hipStream_t s = (hipStream_t)stream;
  if (lkv_status st = wait_event(c, layer, LKV_EV_KV_WRITTEN, s)) return st;
  lkv::Staging &sg = c->d2h;
  const bool two_halves = 2 * c->unit_blocks <= c->staging_blocks;  // else one unit at a time, as a staging chunk
  // the gathers run on the helper stream, behind everything the caller's stream holds at this point and behind the
  // last user of the staging buffer
  LKV_HIP(c, hipEventRecord(sg.entry, s));
  LKV_HIP(c, hipStreamWaitEvent(sg.aux, sg.entry, 0));
  if (sg.buf_used) LKV_HIP(c, hipStreamWaitEvent(sg.aux, sg.last_user == 1 ? sg.pack_last : sg.buf_free, 0));
  sg.last_user = 2;
  for (int64_t first = 0; first < n; first += c->unit_blocks) {
    int64_t m = n - first < c->unit_blocks ? n - first : c->unit_blocks;
    link_gate(c);
    int u = c->tier.acquire();
    // from here to submit() every early return hands the unit back
    auto fail_unit = [&](lkv_status st) {
      c->tier.release(u);
      return st;
    };
    const int h = two_halves ? (int)(sg.units_issued & 1) : 0;
    char *half = sg.buf + (size_t)h * (size_t)(c->unit_blocks * c->block_bytes);
    int slot;
    if (lkv_status st = stage_ids(c, sg, block_ids + first, m, sg.aux, &slot)) return fail_unit(st);
    hipError_t e = sg.half_used[h] ? hipStreamWaitEvent(sg.aux, sg.half_copy[h], 0) : hipSuccess;
    hipEvent_t t0 = nullptr;
    if (e == hipSuccess)
      if (lkv_status st = timed_begin(c, sg.aux, &t0)) return fail_unit(st);
    if (e == hipSuccess) e = lkv::launch_gather_blocks(c, sg.ids_dev + (size_t)slot * c->staging_blocks, m, half, sg.aux);
    if (e == hipSuccess)
      if (lkv_status st = timed_end(c, sg.aux, t0, 2 * m * c->block_bytes, lkv_ctx::kTimedPack)) return fail_unit(st);
    if (e == hipSuccess) e = hipEventRecord(sg.slot_done[slot], sg.aux);
    if (e == hipSuccess) e = hipEventRecord(sg.half_kernel[h], sg.aux);
    if (e == hipSuccess && first + m == n)
      if (lkv_status st = record_event(c, layer, LKV_EV_PACKED, sg.aux)) return fail_unit(st);
    if (e == hipSuccess) e = hipStreamWaitEvent(s, sg.half_kernel[h], 0);
    if (e == hipSuccess)
      if (lkv_status st = pace_unit_copy(c, sg)) return fail_unit(st);
    if (e == hipSuccess)
      e = hipMemcpyAsync(c->tier.unit_ptr(u), half, (size_t)(m * c->block_bytes), hipMemcpyDeviceToHost, s);
    if (e == hipSuccess) e = hipEventRecord(c->unit_ev[(size_t)u], s);
    if (e == hipSuccess && first + m == n) e = hipEventRecord(sg.buf_free, s);
    if (e != hipSuccess) return fail_unit(fail(c, LKV_ERR_DEVICE, "lkv_offload_layer_pageable: %s", hipGetErrorString(e)));
    unit_copy_issued(sg, c->unit_ev[(size_t)u]);
    sg.half_copy[h] = c->unit_ev[(size_t)u];
    sg.half_used[h] = true;
    sg.buf_used = true;
    sg.units_issued += 1;
    lkv::HostTier::Job j = unit_job(c, u);
    j.dst = (char *)host_dst + first * c->block_bytes;
    j.src = c->tier.unit_ptr(u);
    j.bytes = m * c->block_bytes;
    j.key = layer;
    c->tier.submit(std::move(j));
  }
  if (n == 0)
    if (lkv_status st = record_event(c, layer, LKV_EV_PACKED, s)) return st;
  c->stats.pageable_offload_calls += 1;
  c->stats.pageable_offload_bytes += n * c->block_bytes;
  return record_event(c, layer, LKV_EV_OFFLOADED, s);
}

lkv_status lkv_reload_layer_pageable(lkv_ctx *c, int32_t layer, const int32_t *block_ids, int64_t n,
                                     const void *host_src, void *stream) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_reload_layer_pageable: this context has no device resources (lkv_create_logical)");
  if (bad_layer(c, layer) || n < 0 || (n && (!block_ids || !host_src)))
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_reload_layer_pageable: bad argument");
  if (lkv_status st = check_ids(c, block_ids, n)) return st;
  if (lkv_status st = tier_ensure(c)) return st;
  if (!c->tier.wait_key(layer)) return fail(c, LKV_ERR_DEVICE, "host tier: waiting for a device copy failed");
  hipStream_t s = (hipStream_t)stream;
  lkv::Staging &sg = c->h2d;
  const bool two_halves = 2 * c->unit_blocks <= c->staging_blocks;
  // the scatters run on the helper stream, behind everything the caller's stream holds at this point
  LKV_HIP(c, hipEventRecord(sg.entry, s));
  LKV_HIP(c, hipStreamWaitEvent(sg.aux, sg.entry, 0));
  if (sg.buf_used) LKV_HIP(c, hipStreamWaitEvent(s, sg.buf_free, 0));
  for (int64_t first = 0; first < n; first += c->unit_blocks) {
    int64_t m = n - first < c->unit_blocks ? n - first : c->unit_blocks;
    link_gate(c);
    int u = c->tier.acquire();
    auto fail_unit = [&](lkv_status st) {
      c->tier.release(u);
      return st;
    };
    c->tier.copy_parallel(c->tier.unit_ptr(u), (const char *)host_src + first * c->block_bytes, m * c->block_bytes);
    const int h = two_halves ? (int)(sg.units_issued & 1) : 0;
    char *half = sg.buf + (size_t)h * (size_t)(c->unit_blocks * c->block_bytes);
    int slot;
    if (lkv_status st = stage_ids(c, sg, block_ids + first, m, sg.aux, &slot)) return fail_unit(st);
    hipError_t e = sg.half_used[h] ? hipStreamWaitEvent(s, sg.half_kernel[h], 0) : hipSuccess;  // its last scatter
    if (e == hipSuccess)
      if (lkv_status st = pace_unit_copy(c, sg)) return fail_unit(st);
    if (e == hipSuccess)
      e = hipMemcpyAsync(half, c->tier.unit_ptr(u), (size_t)(m * c->block_bytes), hipMemcpyHostToDevice, s);
    if (e == hipSuccess) e = hipEventRecord(c->unit_ev[(size_t)u], s);
    if (e == hipSuccess) e = hipStreamWaitEvent(sg.aux, c->unit_ev[(size_t)u], 0);
    if (e != hipSuccess) return fail_unit(fail(c, LKV_ERR_DEVICE, "lkv_reload_layer_pageable: %s", hipGetErrorString(e)));
    unit_copy_issued(sg, c->unit_ev[(size_t)u]);
    c->tier.submit(unit_job(c, u));  // the unit is free again once the link copy has read it
    hipEvent_t t0;
    if (lkv_status st = timed_begin(c, sg.aux, &t0)) return st;
    LKV_HIP(c, lkv::launch_scatter_blocks(c, sg.ids_dev + (size_t)slot * c->staging_blocks, m, half, sg.aux));
    if (lkv_status st = timed_end(c, sg.aux, t0, 2 * m * c->block_bytes, lkv_ctx::kTimedUnpack)) return st;
    LKV_HIP(c, hipEventRecord(sg.slot_done[slot], sg.aux));
    LKV_HIP(c, hipEventRecord(sg.half_kernel[h], sg.aux));
    if (first + m == n) LKV_HIP(c, hipEventRecord(sg.buf_free, sg.aux));
    sg.half_used[h] = true;
    sg.buf_used = true;
    sg.units_issued += 1;
  }
  // what the caller puts on its stream after this call finds the blocks written
  if (n > 0) LKV_HIP(c, hipStreamWaitEvent(s, sg.buf_free, 0));
  c->stats.pageable_reload_calls += 1;
  c->stats.pageable_reload_bytes += n * c->block_bytes;
  return record_event(c, layer, LKV_EV_RELOADED, s);
}

lkv_status lkv_paged_decode_attention(lkv_ctx *c, int32_t layer, const void *Q, void *O, const int32_t *block_table,
                                      int32_t max_blocks_per_seq, const int32_t *context_lens, int32_t num_seqs,
                                      void *stream) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_paged_decode_attention: this context has no device resources (lkv_create_logical)");
  if (bad_layer(c, layer) || num_seqs < 0 || max_blocks_per_seq < 0)
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_paged_decode_attention: bad layer or count");
  if (!lkv::decode_supported(c))
    return fail(c, LKV_ERR_UNSUPPORTED,
                "lkv_paged_decode_attention: head_dim %d / block_size %d / dtype %d / %d query heads per kv head is not built",
                c->cfg.head_dim, c->cfg.block_size, c->cfg.dtype, c->cfg.num_q_heads / c->cfg.num_kv_heads);
  if (num_seqs == 0) return LKV_OK;
  if (!Q || !O || !context_lens || (max_blocks_per_seq && !block_table))
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_paged_decode_attention: NULL pointer");
  if (((uintptr_t)Q | (uintptr_t)O) & 15)
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_paged_decode_attention: Q and O must be 16-byte aligned");
  hipStream_t s = (hipStream_t)stream;
  const int64_t need = lkv::decode_workspace_bytes(c, num_seqs, max_blocks_per_seq);
  if (need > c->ws_bytes)
    return fail(c, LKV_ERR_INVALID_ARG,
                "lkv_paged_decode_attention: %d sequences with tables of %d blocks need a split-K workspace of %lld bytes, "
                "the context has %lld: call lkv_reserve_decode_workspace first (this call never allocates)",
                num_seqs, max_blocks_per_seq, (long long)need, (long long)c->ws_bytes);
  if (lkv_status st = wait_event(c, layer, LKV_EV_RELOADED, s)) return st;
  // the context's one workspace: a split launch on another stream than the last split launch waits for that one
  if (need > 0 && c->ws_in_use && c->ws_stream != s) LKV_HIP(c, hipStreamWaitEvent(s, c->ws_done, 0));
  hipEvent_t t0;
  if (lkv_status st = timed_begin(c, s, &t0)) return st;
  LKV_HIP(c, lkv::launch_paged_decode(c, Q, O, block_table, max_blocks_per_seq, context_lens, num_seqs, c->ws, s));
  if (lkv_status st = timed_end(c, s, t0, 0, lkv_ctx::kTimedDecode)) return st;
  if (need > 0) {
    LKV_HIP(c, hipEventRecord(c->ws_done, s));
    c->ws_stream = s;
    c->ws_in_use = true;
  }
  c->stats.decode_calls += 1;
  return LKV_OK;
}

lkv_status lkv_paged_decode_attention_static(lkv_ctx *c, int32_t layer, const void *Q, void *O,
                                             const int32_t *block_table, int32_t max_blocks_per_seq,
                                             const int32_t *context_lens, int32_t num_seqs, void *stream) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_paged_decode_attention_static: this context has no device resources (lkv_create_logical)");
  if (bad_layer(c, layer) || num_seqs < 0 || max_blocks_per_seq < 0)
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_paged_decode_attention_static: bad layer or count");
  if (!lkv::decode_supported(c))
    return fail(c, LKV_ERR_UNSUPPORTED,
                "lkv_paged_decode_attention_static: head_dim %d / block_size %d / dtype %d / %d query heads per kv head is not built",
                c->cfg.head_dim, c->cfg.block_size, c->cfg.dtype, c->cfg.num_q_heads / c->cfg.num_kv_heads);
  if (num_seqs == 0) return LKV_OK;
  if (!Q || !O || !context_lens || (max_blocks_per_seq && !block_table))
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_paged_decode_attention_static: NULL pointer");
  if (((uintptr_t)Q | (uintptr_t)O) & 15)
    return fail(c, LKV_ERR_INVALID_ARG, "lkv_paged_decode_attention_static: Q and O must be 16-byte aligned");
  const int64_t need = lkv::decode_workspace_bytes(c, num_seqs, max_blocks_per_seq);
  if (need > (int64_t)LKV_STATIC_DECODE_SCRATCH_BYTES)
    return fail(c, LKV_ERR_INVALID_ARG,
                "lkv_paged_decode_attention_static: %d sequences with tables of %d blocks need %lld bytes of split-K "
                "partial results, the fixed scratch holds %lld",
                num_seqs, max_blocks_per_seq, (long long)need, (long long)LKV_STATIC_DECODE_SCRATCH_BYTES);
  float *ws = lkv::static_scratch(c->device);  // the address hipGetSymbolAddress gave at lkv_create, never the symbol
  if (!ws) return fail(c, LKV_ERR_DEVICE, "lkv_paged_decode_attention_static: the fixed scratch of device %d is unknown", c->device);
  hipStream_t s = (hipStream_t)stream;
  if (lkv_status st = wait_event(c, layer, LKV_EV_RELOADED, s)) return st;
  // no profiling events here: taking one from the free list may create it
  LKV_HIP(c, lkv::launch_paged_decode(c, Q, O, block_table, max_blocks_per_seq, context_lens, num_seqs, ws, s));
  c->stats.decode_calls += 1;
  return LKV_OK;
}

lkv_status lkv_reserve_decode_workspace(lkv_ctx *c, int32_t num_seqs, int32_t max_blocks_per_seq) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_reserve_decode_workspace: this context has no device resources (lkv_create_logical)");
  if (num_seqs < 0 || max_blocks_per_seq < 0) return fail(c, LKV_ERR_INVALID_ARG, "lkv_reserve_decode_workspace: bad count");
  if (!lkv::decode_supported(c)) return fail(c, LKV_ERR_UNSUPPORTED, "lkv_reserve_decode_workspace: no decode kernel for this shape");
  const int64_t need = lkv::decode_workspace_bytes(c, num_seqs, max_blocks_per_seq);
  if (need <= c->ws_bytes) return LKV_OK;
  LKV_HIP(c, hipSetDevice(c->device));
  LKV_HIP(c, hipDeviceSynchronize());  // earlier launches may still use the old workspace
  if (c->ws) LKV_HIP(c, hipFree(c->ws));
  c->ws = nullptr;
  c->ws_bytes = 0;
  LKV_HIP(c, hipMalloc((void **)&c->ws, (size_t)need));
  c->ws_bytes = need;
  return LKV_OK;
}

// ---------------------------------------------------------------- ordering and statistics
lkv_status lkv_stream_wait_event(lkv_ctx *c, int32_t layer, int32_t ev, void *stream) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_stream_wait_event: this context has no device resources (lkv_create_logical)");
  if (bad_layer(c, layer) || ev < 0 || ev > 3) return fail(c, LKV_ERR_INVALID_ARG, "lkv_stream_wait_event: bad argument");
  return wait_event(c, layer, ev, (hipStream_t)stream);
}

lkv_status lkv_event_synchronize(lkv_ctx *c, int32_t layer, int32_t ev) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_event_synchronize: this context has no device resources (lkv_create_logical)");
  if (bad_layer(c, layer) || ev < 0 || ev > 3) return fail(c, LKV_ERR_INVALID_ARG, "lkv_event_synchronize: bad argument");
  if (c->event_recorded[(size_t)layer * 4 + ev]) LKV_HIP(c, hipEventSynchronize(event_of(c, layer, ev)));
  if (ev == LKV_EV_OFFLOADED && c->tier.running() && !c->tier.wait_key(layer))
    return fail(c, LKV_ERR_DEVICE, "host tier: waiting for a device copy failed");
  return LKV_OK;
}

lkv_status lkv_set_profiling(lkv_ctx *c, int32_t on) {
  if (!c) return LKV_ERR_INVALID_ARG;
  if (c->logical_only) return fail(c, LKV_ERR_DEVICE, "lkv_set_profiling: this context has no device resources");
  c->profiling = on != 0;
  return LKV_OK;
}

lkv_status lkv_get_stats(lkv_ctx *c, lkv_stats *out, int64_t size) {
  if (!c || !out || size < 0) return LKV_ERR_INVALID_ARG;
  if (lkv_status st = fold_timed(c, true)) return st;
  c->timed_fold_at = kTimedBacklog;
  c->stats.tier_copy_bytes = c->tier.copied_bytes();
  c->stats.tier_copy_ns = c->tier.copy_ns();
  c->stats.ring_wait_ns = c->tier.ring_wait_ns();
  size_t n = (size_t)size < sizeof(lkv_stats) ? (size_t)size : sizeof(lkv_stats);
  std::memcpy(out, &c->stats, n);
  return LKV_OK;
}

}  // extern "C"
