/*
 * lkv -- layer-wise paged KV cache for AMD MI355X (gfx950): C ABI.
 *
 * The method (LayerKV, arXiv 2410.00428) makes one LAYER of one request the unit of KV-cache
 * allocation, residency and host offload (Section 3: layer-wise KV block allocation,
 * management and offloading).  This library is the data path of that idea:
 *
 *   - a single device pool holds the KV blocks of every layer (Section 4: one tensor
 *     allocated at start-up rather than one per layer), each block belonging to one layer of
 *     one request (Section 3.2.1);
 *   - every (request, layer) has its own block table and a residency state, GPU or host
 *     (Section 3.2.2: the extended block table);
 *   - keys/values are written into a layer's blocks, prompts are processed with causal
 *     attention (Section 2.1.1), a layer's blocks are packed and copied to pinned host memory
 *     on a side stream while compute continues and copied back layer by layer for decoding
 *     (Sections 3.2.1 and 4), and decoding attends through the layer's block table
 *     (Sections 2.1.2, 2.2: paged attention over non-contiguous blocks);
 *   - the same images can live in ordinary host memory behind a small ring of pinned transfer
 *     units drained by CPU threads (Section 4), each unit passing a caller-given link check
 *     (Section 3.2.3);
 *   - the host-side policy of the method as pure functions: the prefill and offload cost
 *     models and the number of layers to retain (Sections 3.1, 3.2.1), the SLO-aware admission
 *     of queued prefills (Section 3.1, Algorithm 1), the free-block forecast and the pressure
 *     rule (Section 3.2.1).
 *
 * Conventions
 *   Pointers  "device" = memory of the current HIP device; "host" = ordinary host memory,
 *             "pinned" = page-locked host memory (hipHostMalloc).  The caller owns every
 *             buffer it passes; the library owns lkv_ctx, its staging buffers, its split-K
 *             workspace and its events.  The pool is the caller's if lkv_config.pool is set.
 *   Streams   `stream` is a hipStream_t passed as void* (NULL = the default stream).  Device
 *             calls only enqueue work and return; results are ready when the stream reaches
 *             that point.  Host arrays (block_ids) are consumed before the call returns.
 *   Errors    every call returns an lkv_status; nothing throws or aborts across the ABI.
 *             lkv_last_error() gives a text for the last failure on that context.  Arguments
 *             the host can see (layer range, NULL pointers, counts, ids given as host arrays)
 *             are validated; indices that live in device memory (slot_mapping, block_table,
 *             context_lens) are the caller's responsibility: they must lie inside the pool (the
 *             kernels skip a slot and clamp a table entry outside it rather than touch memory
 *             outside the pool; the results are then wrong, not a fault).
 *   Threads   a context is not thread-safe; use one thread per context or lock outside.
 *
 * Storage format of the pool (also the format of an offloaded image)
 *   e = element size (4 for LKV_F32, 2 for LKV_BF16, 1 for LKV_FP8_E4M3), tau = 2*num_kv_heads*head_dim*e bytes
 *   per token per layer, beta = block_size*tau bytes per block.  Block b starts at byte
 *   b*beta.  Inside a block the order is [kv_head][K then V][token in block][channel]:
 *     K of token slot (b, o), head h, channel c:  b*beta + h*(2*block_size*head_dim*e)
 *                                                 + o*head_dim*e + c*e
 *     V of the same:                              that + block_size*head_dim*e
 *   A slot number is b*block_size + o.  An offloaded image of ids[0..n) is the n blocks
 *   verbatim, block ids[i] at byte i*beta.
 */
#ifndef LKV_H
#define LKV_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lkv_ctx lkv_ctx;

typedef enum {
  LKV_OK = 0,
  LKV_ERR_INVALID_ARG = 1,  /* bad layer, NULL pointer, negative count, id outside the pool ... */
  LKV_ERR_NO_BLOCKS = 2,    /* the free list cannot cover the allocation; nothing was changed  */
  LKV_ERR_NOT_RESIDENT = 3, /* the (request, layer) has no blocks in the pool right now        */
  LKV_ERR_HOST_MEMORY = 4,  /* a host allocation failed                                        */
  LKV_ERR_DEVICE = 5,       /* a HIP call failed; see lkv_last_error                           */
  LKV_ERR_UNSUPPORTED = 6   /* shape outside what the kernels are built for                    */
} lkv_status;

/* LKV_FP8_E4M3: the pool holds one-byte OCP E4M3 codes (1 sign, 4 exponent, 3 mantissa bits, bias 7, largest value
 * 448, no infinities) of K / k_scale and V / v_scale; queries, the keys and values given to lkv_write_kv, prompts
 * and outputs stay bf16.  The paper names KV-cache quantisation as the next step (its Future Work section) without
 * fixing a format: this is this library's choice.  It halves tau, beta, every offload image and the bytes decode
 * attention reads.  Attention kernels: head_dim 128 only. */
typedef enum { LKV_F32 = 0, LKV_BF16 = 1, LKV_FP8_E4M3 = 2 } lkv_dtype;

/* residency of one (request, layer), Section 3.2.2: where its KV lives.  LKV_RES_IN_FLIGHT is reported instead of
 * GPU or HOST while a transfer of that layer which this context has queued is not finished yet (a HOST layer whose
 * device-to-host copy, CPU copies of a pageable offload included, is still running: the image is not complete; a GPU
 * layer whose reload has been queued and has not finished: its blocks do not hold the data yet).  The transfer
 * events are per layer, so every request's entry for that layer reads IN_FLIGHT meanwhile. */
enum { LKV_RES_NONE = 0, LKV_RES_GPU = 1, LKV_RES_HOST = 2, LKV_RES_IN_FLIGHT = 3 };

/* per-layer events the library records (Section 4: transfers run on their own stream,
 * concurrently with compute, and are ordered against it per layer) */
typedef enum {
  LKV_EV_KV_WRITTEN = 0, /* lkv_write_kv of the layer has been enqueued up to here            */
  LKV_EV_PACKED = 1,     /* the layer's blocks have been gathered out of the pool: the blocks
                            may be reused from here on                                         */
  LKV_EV_OFFLOADED = 2,  /* the device-to-host copy of the layer has finished                  */
  LKV_EV_RELOADED = 3    /* the layer's blocks are back in the pool                            */
} lkv_event;

typedef struct {
  int32_t num_layers;
  int32_t num_q_heads;
  int32_t num_kv_heads;     /* must divide num_q_heads; q head h uses kv head h/(Hq/Hkv).  Decode
                             * attention: Hq/Hkv <= 16 for bf16 / 8-bit pools with head_dim 128, <= 8
                             * otherwise (LKV_ERR_UNSUPPORTED beyond); prefill takes any ratio           */
  int32_t head_dim;         /* attention kernels: 64 or 128; head_dim*e must be a multiple of 16 */
  int32_t block_size;       /* tokens per block; attention kernels: 16                         */
  int32_t dtype;            /* lkv_dtype                                                       */
  int64_t num_pool_blocks;  /* layer-blocks in the pool                                        */
  float softmax_scale;      /* 0 => 1/sqrt(head_dim)                                           */
  int32_t decode_partition; /* tokens per split-K partition of decode attention (multiple of
                               64); 0 => library default                                       */
  void *pool;               /* device, num_pool_blocks*beta bytes, 256-byte aligned, or NULL
                               to let the library allocate (and free) it                       */
  int64_t staging_bytes;    /* device staging per transfer direction; 0 => 256 MiB.  A layer
                               image larger than this is moved in several chunks               */
  float k_scale, v_scale;   /* LKV_FP8_E4M3 only: stored code = nearest E4M3 value (ties to even, saturating
                               at +-448, NaN kept) of x * (1.0f / scale), the product rounded once to
                               float; 0 => 1.0                                                   */
} lkv_config;

typedef struct {
  int64_t write_kv_calls, write_kv_bytes;     /* bytes = tokens written * tau (read + write counted once) */
  int64_t prefill_calls;
  int64_t decode_calls;
  int64_t pack_calls, pack_bytes;             /* bytes gathered out of the pool = bytes sent to host */
  int64_t unpack_calls, unpack_bytes;
  /* filled only while kernel profiling is on (lkv_set_profiling): time the gather / scatter kernels of
   * pack / unpack spent on the GPU (HIP events on the stream they ran on), and the bytes they moved
   * (read + write) in those launches */
  int64_t pack_kernel_ns, pack_kernel_bytes;
  int64_t unpack_kernel_ns, unpack_kernel_bytes;
  /* likewise while profiling is on: GPU time between an event recorded right before and one right after the
   * kernel launches of lkv_write_kv, lkv_prefill_attention and lkv_paged_decode_attention (the latter includes
   * the combine kernel when the context is split), and how many calls were timed */
  int64_t write_kernel_ns, write_kernel_launches;
  int64_t prefill_kernel_ns, prefill_kernel_launches;
  int64_t decode_kernel_ns, decode_kernel_launches;
  /* pageable host tier: calls and bytes of lkv_offload_layer_pageable / lkv_reload_layer_pageable; bytes the
   * CPU threads have copied between the pinned ring and pageable memory and the time they spent in memcpy
   * (summed over threads); time the calling thread waited for a free ring unit; how often the link gate
   * answered "busy" (lkv_set_link_gate) */
  int64_t pageable_offload_calls, pageable_offload_bytes;
  int64_t pageable_reload_calls, pageable_reload_bytes;
  int64_t tier_copy_bytes, tier_copy_ns;
  int64_t ring_wait_ns;
  int64_t gate_busy_answers;
  /* bytes (read + write) moved by the lkv_write_kv launches counted in write_kernel_ns */
  int64_t write_kernel_bytes;
} lkv_stats;

/* ------------------------------------------------------------------ life cycle */
/* Creates a context on the current HIP device.  Allocates the pool if cfg->pool is NULL, two
 * staging buffers and the per-layer events.  All blocks start free in ascending id order. */
lkv_status lkv_create(const lkv_config *cfg, lkv_ctx **out);
/* The same context without any device resource: only the logical-state calls below work (a
 * scheduler process without a GPU can plan with it); device calls return LKV_ERR_DEVICE. */
lkv_status lkv_create_logical(const lkv_config *cfg, lkv_ctx **out);
/* Waits for the device, then frees everything the library owns.  NULL is allowed. */
void lkv_destroy(lkv_ctx *ctx);
/* Text of the last error on ctx (or of the last failed lkv_create if ctx is NULL). */
const char *lkv_last_error(const lkv_ctx *ctx);
/* Device pointer of the pool and its size in bytes (either may be NULL). */
lkv_status lkv_pool_info(const lkv_ctx *ctx, void **pool, int64_t *bytes, int64_t *block_bytes);

/* ------------------------------------------------------------------ logical state (host only; Sections 3.2.1, 3.2.2)
 * The free list is a stack.  lkv_pool_reset makes every block free and drops every table;
 * free_order (host, a permutation of 0..n-1, n = num_pool_blocks) gives the order in which
 * blocks are handed out: free_order[0] first.  Freeing a table pushes its ids in table order,
 * so the table's last block is the next one handed out. */
lkv_status lkv_pool_reset(lkv_ctx *ctx, const int32_t *free_order, int64_t n);
/* Grows the table of (seq, layer) to ceil(num_tokens_total/block_size) blocks (never shrinks)
 * and marks the layer GPU-resident.  For a host-resident layer this is the reload's
 * allocation: fresh ids, not the old ones.  LKV_ERR_NO_BLOCKS leaves everything unchanged. */
lkv_status lkv_alloc_layer_blocks(lkv_ctx *ctx, int64_t seq, int32_t layer, int64_t num_tokens_total);
/* Returns the blocks of (seq, layer) to the free list.  to_host != 0 records that the layer now
 * lives on the host (after an offload); 0 forgets the layer.  The caller must have ordered the
 * release after LKV_EV_PACKED of the data it still needs. */
lkv_status lkv_free_layer_blocks(lkv_ctx *ctx, int64_t seq, int32_t layer, int32_t to_host);
/* A finished request releases all its layers, lowest layer first (Section 2.2). */
lkv_status lkv_free_seq(lkv_ctx *ctx, int64_t seq);
/* Copies the table of (seq, layer) to out (host, capacity cap entries); *n = its length. */
lkv_status lkv_get_block_table(const lkv_ctx *ctx, int64_t seq, int32_t layer, int32_t *out, int64_t cap, int64_t *n);
/* out[i] (host) = slot of token position pos0+i of (seq, layer): table[p/bs]*bs + p%bs. */
lkv_status lkv_build_slot_mapping(const lkv_ctx *ctx, int64_t seq, int32_t layer, int64_t pos0, int64_t count, int64_t *out);
/* *out = LKV_RES_* of (seq, layer).  Never blocks: an unfinished transfer is found by querying its event. */
lkv_status lkv_layer_residency(const lkv_ctx *ctx, int64_t seq, int32_t layer, int32_t *out);
int64_t lkv_num_free_blocks(const lkv_ctx *ctx);
/* Which layers keep their KV on the GPU when x of num_layers are retained: spread evenly,
 * mask[l] = 1 (host array of num_layers entries) for retained layers.  For 8 layers and x = 4
 * the retained layers are 1,3,5,7 (the example of Section 3.2.2). */
lkv_status lkv_plan_retained_layers(int32_t num_layers, int32_t x, int32_t *mask);

/* ------------------------------------------------------------------ host-side policy (no context, no device)
 * Pure functions of their arguments; times in seconds.  A time function returns NaN for invalid arguments. */

/* Cost models of Section 3.1 (prefill time, the first equation labelled "prefill") and Section 3.2.1 (offload
 * time, the second equation with that label). */
typedef struct {
  double alpha;             /* empirical correction of the prefill model                              */
  double n_param;           /* model parameters                                                      */
  double n_hidden;          /* hidden size                                                           */
  double device_flops;      /* FLOP per second of the device                                         */
  double beta;              /* empirical correction of the offload model                             */
  int32_t num_layers;       /* L                                                                     */
  int32_t head_dim;         /* d_heads                                                               */
  int32_t num_heads;        /* n_heads: the heads whose K and V are stored (KV heads)                */
  double bytes_per_elem;    /* f_precision in bytes                                                  */
  double link_bytes_per_s;  /* PCIe bandwidth                                                        */
} lkv_cost_model;
/* alpha * seqlen * (2 n_param + 2 seqlen n_hidden) / device_flops */
double lkv_prefill_time(const lkv_cost_model *m, int64_t seqlen);
/* beta * seqlen * 2 (L - x) d_heads n_heads f_precision / link bandwidth: x layers stay on the GPU */
double lkv_offload_time(const lkv_cost_model *m, int64_t seqlen, int32_t x);
/* The smallest x in 0..L whose offload time does not exceed the prefill time of the same prompt (Section 3.2.1:
 * the offload then hides behind the computation), and which layers stay: *x_out = x; retained_mask (host,
 * num_layers entries, may be NULL) as lkv_plan_retained_layers gives it for that x. */
lkv_status lkv_plan_offload(const lkv_cost_model *m, int64_t seqlen, int32_t *x_out, int32_t *retained_mask);

/* One request in the decoding phase as the SLO-aware scheduler sees it (Section 3.1). */
typedef struct {
  double t_tpot;                  /* its TPOT target, seconds per token                               */
  int64_t n_past;                 /* tokens generated so far                                          */
  double t_past;                  /* decoding time spent so far, waiting included                     */
  int64_t predicted_lower_bound;  /* lower bound of the predicted range of its complete output length */
} lkv_decode_request;
/* Eq. 1: T_tpot (N_past + N_future) - (T_past + T_future), with N_future = max(1, predicted_lower_bound -
 * N_past) and T_future = current TPOT * N_future; the current TPOT is T_past / N_past, or the target for a
 * request that has produced nothing yet. */
double lkv_allow_prefill_time(const lkv_decode_request *r);
/* Algorithm 1: *n_out = the largest n such that the prefill times of the first n queued requests (host array,
 * queue order) add up to LESS than the smallest allowance of the decoding requests (host array); with nothing
 * decoding the whole queue is admitted. */
lkv_status lkv_max_prefills(const lkv_decode_request *decoding, int32_t num_decoding, const double *prefill_times,
                            int32_t num_queued, int32_t *n_out);

/* Free-block forecast (Section 3.2.1): Avail(t+1) = Avail(t) + Released(t) - Allocated(t) for `stages` stages
 * from Avail(0) = avail0.  avail_out (host, `stages` entries, may be NULL) receives Avail(1..stages);
 * *first_below (may be NULL) the first stage t >= 1 whose forecast is below `threshold`, or -1. */
lkv_status lkv_forecast_avail(int64_t avail0, const int64_t *released, const int64_t *allocated, int32_t stages,
                              int64_t threshold, int64_t *avail_out, int32_t *first_below);
/* Pressure rule (Section 3.2.1): which retained layers to give up when `deficit_blocks` more free blocks are
 * needed.  Requests are listed most recent first; retained[r] layers of request r are on the GPU, each holding
 * blocks_per_layer[r] blocks.  First every request in turn gives half of its retained layers (rounded up)
 * until the deficit is covered; only if all halves together are not enough do the requests, in the same order,
 * give the rest.  give[r] (host) = layers request r gives up. */
lkv_status lkv_pressure_offload(int64_t deficit_blocks, const int32_t *retained, const int64_t *blocks_per_layer,
                                int32_t num_requests, int32_t *give);

/* ------------------------------------------------------------------ device hot path */
/* K, V: device, [num_tokens][num_kv_heads][head_dim], contiguous.  slot_mapping: device,
 * int64[num_tokens]; token t goes to slot slot_mapping[t]; a negative slot skips the token, and so does a slot
 * past the end of the pool (a caller's mistake that must not write outside it).  With an LKV_FP8_E4M3 pool K and V
 * are bf16 and are stored as codes (see lkv_dtype).
 * Waits (on `stream`) for LKV_EV_RELOADED of the layer, then records LKV_EV_KV_WRITTEN of
 * `layer` on `stream`.  (Sections 2.1.1, 3.2.1) */
lkv_status lkv_write_kv(lkv_ctx *ctx, int32_t layer, const void *K, const void *V,
                        const int64_t *slot_mapping, int64_t num_tokens, void *stream);

/* Softmax attention over packed variable-length prompts (Section 2.1.1).  Q, O: device,
 * [T][num_q_heads][head_dim]; K, V: device, [T][num_kv_heads][head_dim]; cu_seqlens: device,
 * int32[num_seqs+1], sequence s is tokens cu[s]..cu[s+1].  Row i of a sequence sees keys
 * 0..i if causal != 0, all keys otherwise.  max_seqlen >= the longest sequence (sizes the
 * grid).  total_tokens = T (host-known, = cu[num_seqs]; the launch is sized from it and from max_seqlen: with
 * values smaller than the batch's, rows of O stay unwritten).  cu_seqlens is device memory the host cannot check:
 * the kernels cut every sequence to 0 <= cu[s] <= cu[s+1] <= total_tokens and to max_seqlen tokens, so entries
 * that are out of order or too large give wrong or unwritten rows but never touch memory outside the four tensors'
 * total_tokens rows.  `layer` selects no data; it names
 * the layer whose compute this is, for the statistics.  bf16: fp32 accumulation, probabilities
 * rounded to bf16 before the value product; f32: fp32 throughout. */
lkv_status lkv_prefill_attention(lkv_ctx *ctx, int32_t layer, const void *Q, const void *K, const void *V,
                                 void *O, const int32_t *cu_seqlens, int32_t num_seqs,
                                 int32_t max_seqlen, int64_t total_tokens, int32_t causal, void *stream);

/* Offload image of one layer (Sections 3.2.1, 4): gathers blocks block_ids[0..n) (host array) into device staging
 * and copies them to pinned_dst (n*beta bytes).  The copies run on `stream`; the gathers run on a helper stream of
 * the library, behind everything `stream` holds when the call is made and behind LKV_EV_KV_WRITTEN of the layer, into
 * two staging buffers in turn, so that the gather of one chunk (or of the next layer's call) overlaps the copy of the
 * one before it and the link stays busy back to back.  Records LKV_EV_PACKED after the last gather (on the helper
 * stream) and LKV_EV_OFFLOADED after the last copy (on `stream`): work put on `stream` after the call is ordered
 * behind the whole offload.  Does not touch tables or the free list.  Host-link copies are paced:
 * at most two per direction are queued at a time, so this call (and lkv_unpack_layer_blocks) blocks the calling
 * thread until the copy two places ahead of its own has finished (at most the duration of one chunk's copy per
 * chunk issued; staging_bytes sets the chunk size). */
lkv_status lkv_pack_layer_blocks(lkv_ctx *ctx, int32_t layer, const int32_t *block_ids, int64_t n,
                                 void *pinned_dst, void *stream);
/* Reload (Section 4: layer by layer, host to device): copies n*beta bytes from pinned_src into
 * device staging and scatters chunk i into block block_ids[i] -- the ids need not be the ones
 * the image was packed from.  Records LKV_EV_RELOADED of the layer on `stream`. */
lkv_status lkv_unpack_layer_blocks(lkv_ctx *ctx, int32_t layer, const int32_t *block_ids, int64_t n,
                                   const void *pinned_src, void *stream);

/* ---- pageable host tier (Section 4: a CPU thread moves offloaded KV from pinned to pageable memory;
 * Section 3.2.3: a transfer is cut into smaller units).  The two calls below move the same image as
 * lkv_pack_layer_blocks / lkv_unpack_layer_blocks, but to and from ORDINARY host memory: the data crosses the
 * link through a small ring of pinned units owned by the library, and CPU threads of the library copy between
 * the ring and the caller's buffer, so pinned memory stays at num_units*unit_bytes however much KV is
 * offloaded.  The calling thread blocks while all ring units are in use (that is the back-pressure of a
 * bounded ring), never for the link or the memcpy of a unit it has already handed over.  The link copies of the
 * units run on `stream`; their gather / scatter kernels run on a helper stream of the library (over two halves of
 * the device staging, so that the kernel of one unit overlaps the copy of the other), ordered behind everything
 * `stream` holds when the call is made; what the caller puts on `stream` after the call is ordered behind them. */

/* Sets the ring's shape: unit_bytes per unit (rounded down to whole blocks, at least one block, at most the
 * device staging), num_units >= 1 units of pinned memory, threads >= 1 CPU threads.  Zero keeps the default
 * (32 MiB, 4 units, 4 threads).  Allowed any time: waits for the tier's outstanding work, then rebuilds the
 * ring.  Without this call the ring is built with the defaults on first use. */
lkv_status lkv_host_tier_config(lkv_ctx *ctx, int64_t unit_bytes, int32_t num_units, int32_t threads);
/* Offload to pageable memory: as lkv_pack_layer_blocks (same waits, same events on `stream`), with host_dst
 * (n*beta bytes) ordinary host memory.  LKV_EV_OFFLOADED here means "the last unit has reached the pinned
 * ring"; the image is complete in host_dst once lkv_host_tier_synchronize(layer) or
 * lkv_event_synchronize(layer, LKV_EV_OFFLOADED) has returned.  host_dst must stay valid until then.  A
 * second offload of the same layer first waits for the first one's CPU copies. */
lkv_status lkv_offload_layer_pageable(lkv_ctx *ctx, int32_t layer, const int32_t *block_ids, int64_t n,
                                      void *host_dst, void *stream);
/* Reload from pageable memory: as lkv_unpack_layer_blocks, with host_src ordinary host memory.  Waits (host)
 * for outstanding CPU copies of an offload of the same layer, then per unit: CPU copy into a ring unit (split
 * over the library's threads and the caller), host-to-device copy, scatter.  host_src may be reused when the
 * call returns.  Records LKV_EV_RELOADED on `stream`. */
lkv_status lkv_reload_layer_pageable(lkv_ctx *ctx, int32_t layer, const int32_t *block_ids, int64_t n,
                                     const void *host_src, void *stream);
/* Blocks until the CPU copies of every pageable offload of `layer` issued so far are done (layer -1: of all
 * layers).  LKV_ERR_DEVICE if waiting for one of their device copies failed. */
lkv_status lkv_host_tier_synchronize(lkv_ctx *ctx, int32_t layer);

/* Link gate (Section 3.2.3: before a swap, check whether the host link is in use by traffic on the critical
 * path; if so wait a while and check again, unit by unit).  busy(user) is called on the calling thread before
 * every unit of all four transfer calls (a unit is a staging chunk for pack/unpack, a ring unit for the
 * pageable calls); while it returns non-zero the library sleeps delay_us microseconds and asks again, at most
 * max_checks times per unit (then the unit goes anyway, so a gate that never opens cannot stop the transfer).
 * busy == NULL removes the gate.  delay_us >= 0, max_checks >= 0. */
typedef int32_t (*lkv_link_busy_fn)(void *user);
lkv_status lkv_set_link_gate(lkv_ctx *ctx, lkv_link_busy_fn busy, void *user, int64_t delay_us, int32_t max_checks);

/* Decode attention through this layer's block table (Sections 2.1.2, 2.2, 3.2.2).  Q, O:
 * device, [num_seqs][num_q_heads][head_dim]; block_table: device, int32[num_seqs][max_blocks_per_seq]
 * (entries past ceil(context_len/bs) are ignored; every entry before that must be a block id of the pool: the
 * kernels clamp an entry outside [0, num_pool_blocks) into the pool, which gives a wrong row but touches no memory
 * outside the pool); context_lens: device, int32[num_seqs] (a value above 16*max_blocks_per_seq is cut there);
 * sequence s attends to positions 0..context_lens[s]-1; a zero context gives a zero row.
 * Waits (on `stream`) for LKV_EV_RELOADED of the layer.  A launch with long contexts (or with too few sequences to
 * fill the GPU) is split: cut into equal shares of its keys, one per compute unit, or, when decode_partition is set
 * or the batch has more than 256 sequences, into partitions of a fixed number of tokens; a second kernel merges the
 * partial results, which go through the context's split-K workspace.  This call never allocates and never synchronises: the workspace is the one lkv_create made
 * (32 MiB: enough for 256 sequences of 16384 tokens with 32 query heads) or the one the last
 * lkv_reserve_decode_workspace made; a call that needs more returns LKV_ERR_INVALID_ARG and enqueues nothing.
 * A context has ONE workspace: a split call on another stream than the context's last split call is made to wait
 * (on its stream) for that one, so calls of one context on several streams are safe, and those that split do not
 * overlap. */
lkv_status lkv_paged_decode_attention(lkv_ctx *ctx, int32_t layer, const void *Q, void *O,
                                      const int32_t *block_table, int32_t max_blocks_per_seq,
                                      const int32_t *context_lens, int32_t num_seqs, void *stream);

/* Makes the split-K workspace large enough for lkv_paged_decode_attention calls with up to num_seqs sequences and
 * tables of max_blocks_per_seq entries (never shrinks it).  Not a hot-path call: when the workspace has to grow it
 * waits for the device (earlier launches may still use the old one), frees it and allocates the new one. */
lkv_status lkv_reserve_decode_workspace(lkv_ctx *ctx, int32_t num_seqs, int32_t max_blocks_per_seq);

/* For callers that cannot allocate device memory (code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc): the same operation, arguments, kernels and results as lkv_paged_decode_attention, with the
 * split-K partial results in a fixed array that is part of the library's device code (8 MiB per GPU, held until the
 * process ends) instead of the context's workspace.  Calls no hipMalloc / hipFree and creates nothing.  A call whose
 * partial results exceed the array ((head_dim + 2) * 4 bytes for each of num_seqs * num_q_heads * partitions entries
 * of a partitioned launch, or of (num_seqs * num_kv_heads + compute units) * (num_q_heads / num_kv_heads) entries
 * of an evenly cut one, > 8 MiB) returns LKV_ERR_INVALID_ARG and enqueues nothing.  Kernel profiling (lkv_set_profiling) does not cover this call.  Every
 * call on a GPU, from any context, uses that GPU's one array: calls that overlap in time on one GPU (two streams
 * without an event between them) race on it; each call overwrites what it reads, so nothing needs clearing between
 * calls. */
lkv_status lkv_paged_decode_attention_static(lkv_ctx *ctx, int32_t layer, const void *Q, void *O,
                                             const int32_t *block_table, int32_t max_blocks_per_seq,
                                             const int32_t *context_lens, int32_t num_seqs, void *stream);

/* ------------------------------------------------------------------ ordering and statistics */
/* Makes `stream` wait for the last recorded event `ev` of `layer` (no-op if never recorded). */
lkv_status lkv_stream_wait_event(lkv_ctx *ctx, int32_t layer, int32_t ev, void *stream);
/* Blocks the host until that event has happened (for LKV_EV_OFFLOADED of a pageable offload: until the image
 * is complete in the caller's buffer). */
lkv_status lkv_event_synchronize(lkv_ctx *ctx, int32_t layer, int32_t ev);
/* Turns per-launch HIP-event timing of the library's kernels on or off (off by default).  The events are
 * attached to the kernels themselves (the begin of a launch's first kernel, the end of its last), so the times
 * are the kernels' own.  Results accumulate in lkv_stats. */
lkv_status lkv_set_profiling(lkv_ctx *ctx, int32_t on);
/* Copies min(size, sizeof(lkv_stats)) bytes of counters to out (host).  With profiling on this waits
 * for the timed launches recorded so far. */
lkv_status lkv_get_stats(lkv_ctx *ctx, lkv_stats *out, int64_t size);

#ifdef __cplusplus
}
#endif
#endif /* LKV_H */
