// Internal declarations shared by the host code and the kernel launchers of liblkv.
#pragma once

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>
#include <string>
#include <unordered_map>
#include <vector>

#include "host_tier.hpp"
#include "lkv.h"

namespace lkv {

struct LayerKey {
  int64_t seq;
  int32_t layer;
  bool operator==(const LayerKey &o) const { return seq == o.seq && layer == o.layer; }
};
struct LayerKeyHash {
  size_t operator()(const LayerKey &k) const {
    return std::hash<int64_t>()(k.seq * 1000003 + k.layer);
  }
};
struct LayerState {
  std::vector<int32_t> table;  // block ids in token order
  int32_t residency = LKV_RES_NONE;
};

// One transfer direction's device staging plus the bookkeeping that keeps two streams from
// using it at once.
struct Staging {
  char *buf = nullptr;          // device
  int32_t *ids_dev = nullptr;   // device, capacity ids_cap per slot
  int32_t *ids_pinned = nullptr;  // pinned host mirror, same shape
  static constexpr int kSlots = 8;
  hipEvent_t slot_done[kSlots] = {};  // ids slot consumed by its kernel
  int next_slot = 0;
  hipEvent_t buf_free = nullptr;  // last user of buf has finished with it
  bool buf_used = false;
  // pacing: at most kMaxInFlight host-link copies of this direction are queued at any time
  static constexpr int kCopyRing = 4, kMaxInFlight = 2;
  hipEvent_t copy_done[kCopyRing] = {};
  int64_t copies_issued = 0;
  // The pageable calls move a layer in many small units.  With the gather (or scatter) kernel of a unit on the
  // caller's stream the link would idle between two copies while the kernel runs and the queues hand over; so the
  // kernels run on a helper stream, over the two halves of buf in turn, and only events connect them to the copies.
  hipStream_t aux = nullptr;
  hipEvent_t entry = nullptr;             // the caller's stream at the start of a call: the helper stream starts after it
  // Between two link copies the caller's stream carries one wait and one event record, no more (every packet
  // between two copies costs link time): the event of the ring unit a copy goes to or comes from serves the worker
  // threads, the pacing and the other stream.  Offload: half_kernel[h] = gather into half h done (helper stream),
  // half_copy[h] = the ring unit event of the last copy out of half h.  Reload: half_copy[h] = the ring unit event of
  // the last copy into half h, half_kernel[h] = scatter out of half h done (helper stream).
  hipEvent_t half_kernel[2] = {};
  hipEvent_t half_copy[2] = {};           // not owned: handles of ring unit events
  bool half_used[2] = {false, false};
  int64_t units_issued = 0;               // picks the half
  hipEvent_t unit_copies[kCopyRing] = {}; // not owned: the ring unit events of the last copies, for the pacing
  // The pinned offload (lkv_pack_layer_blocks) alternates between buf and a second buffer of the same size, so that
  // the gather of one chunk (on the helper stream) runs while the link copy of the chunk before it is still going:
  // the link never waits for a gather, however slowly the gather gets CUs next to an attention kernel.
  char *buf2 = nullptr;
  hipEvent_t twin_gathered[2] = {};       // gather into buffer b done (helper stream)
  hipEvent_t twin_copied[2] = {};         // not owned: the pacing event of the last copy out of buffer b
  hipEvent_t pack_last = nullptr;         // not owned: the pacing event of the last copy of the pinned offload
  bool twin_used[2] = {false, false};
  int64_t twin_chunks = 0;                // picks the buffer
  int last_user = 0;                      // 0 nobody yet, 1 the pinned calls, 2 the pageable calls
};

}  // namespace lkv

struct lkv_ctx {
  lkv_config cfg{};
  int device = 0;
  int64_t elem = 0;         // bytes per element
  int64_t row_bytes = 0;    // head_dim*elem
  int64_t token_bytes = 0;  // tau
  int64_t block_bytes = 0;  // beta
  float scale = 0.f;
  float k_scale = 1.f, v_scale = 1.f;  // 8-bit pools: value = code * scale
  int64_t in_row_bytes = 0;            // one head row of what lkv_write_kv is given (bf16 for 8-bit pools)
  char *pool = nullptr;
  bool owns_pool = false;
  bool logical_only = false;  // created without device resources: host state only
  int64_t staging_blocks = 0;  // blocks that fit one staging buffer
  lkv::Staging d2h, h2d;
  std::vector<hipEvent_t> events;  // [layer][4]
  std::vector<uint8_t> event_recorded;
  // split-K workspace of decode attention; ws_done is recorded behind every split launch, and a split launch on
  // another stream than the last one waits for it (one workspace per context: two launches must not overlap)
  float *ws = nullptr;
  int64_t ws_bytes = 0;
  hipEvent_t ws_done = nullptr;
  hipStream_t ws_stream = nullptr;
  bool ws_in_use = false;
  // logical state
  std::vector<int32_t> free_list;  // stack, back() is handed out next
  std::unordered_map<lkv::LayerKey, lkv::LayerState, lkv::LayerKeyHash> layers;
  lkv_stats stats{};
  // kernel profiling: (start, stop, bytes, which kernel) of launches not yet folded into stats
  enum TimedKind { kTimedPack, kTimedUnpack, kTimedWrite, kTimedPrefill, kTimedDecode };
  struct Timed {
    hipEvent_t a, b;
    int64_t bytes;
    int kind;
  };
  // the profiled region that is being launched right now: its start event goes to the first kernel of the region,
  // its stop event to the last one (launch_timed below); null while profiling is off
  mutable hipEvent_t prof_start = nullptr, prof_stop = nullptr;
  mutable bool prof_start_used = false, prof_stop_used = false;
  // pageable host tier: pinned ring, one event per ring unit, the CPU threads
  lkv::HostTier tier;
  char *ring = nullptr;
  std::vector<hipEvent_t> unit_ev;
  int64_t unit_blocks = 0;
  // link gate
  lkv_link_busy_fn gate_busy = nullptr;
  void *gate_user = nullptr;
  int64_t gate_delay_us = 0;
  int32_t gate_max_checks = 0;
  bool profiling = false;
  std::vector<Timed> timed;
  size_t timed_fold_at = 512;  // list length at which finished pairs are folded on the way
  std::vector<hipEvent_t> spare_events;
  mutable std::string err;
};

// Launches a kernel of the hot path.  While profiling is on, the region's timing events are attached to the
// kernels themselves (start of the region's first kernel, end of its last): the time read from them is the kernels'
// own, as a profiler reports it, without the stream's hand-over before and after a launch.
template <typename Kernel, typename... Args>
inline void launch_timed(const lkv_ctx *c, bool first, bool last, Kernel kernel, dim3 grid, dim3 block, hipStream_t s,
                         Args... args) {
  hipEvent_t a = first ? c->prof_start : nullptr, b = last ? c->prof_stop : nullptr;
  hipExtLaunchKernelGGL(kernel, grid, block, 0, s, a, b, 0, args...);
  if (a) c->prof_start_used = true;
  if (b) c->prof_stop_used = true;
}

namespace lkv {

// All launchers return hipSuccess or the launch error; arguments are validated by the callers.
hipError_t launch_write_kv(const lkv_ctx *c, const void *K, const void *V, const int64_t *slots,
                           int64_t num_tokens, hipStream_t s);
// gather: dst[i*beta ..] = pool[ids[i]*beta ..];  scatter: the inverse.
hipError_t launch_gather_blocks(const lkv_ctx *c, const int32_t *ids_dev, int64_t n, char *dst, hipStream_t s);
hipError_t launch_scatter_blocks(const lkv_ctx *c, const int32_t *ids_dev, int64_t n, const char *src, hipStream_t s);

int64_t decode_workspace_bytes(const lkv_ctx *c, int32_t num_seqs, int32_t max_blocks_per_seq);
hipError_t launch_paged_decode(const lkv_ctx *c, const void *Q, void *O, const int32_t *block_table,
                               int32_t max_blocks_per_seq, const int32_t *context_lens, int32_t num_seqs,
                               float *ws, hipStream_t s);
bool decode_supported(const lkv_ctx *c);
// The fixed split-K scratch of lkv_paged_decode_attention_static: static_scratch_init looks its address up once per
// device (that device must be current), static_scratch returns it (nullptr before the lookup).
#define LKV_STATIC_DECODE_SCRATCH_BYTES (8 << 20)
hipError_t static_scratch_init(int device);
float *static_scratch(int device);

hipError_t launch_prefill(const lkv_ctx *c, const void *Q, const void *K, const void *V, void *O,
                          const int32_t *cu_seqlens, int32_t num_seqs, int32_t max_seqlen, int64_t total_tokens,
                          int32_t causal, hipStream_t s);
bool prefill_supported(const lkv_ctx *c);

}  // namespace lkv
