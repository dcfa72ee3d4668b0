/*
 * kvswap.h — C ABI of the paged KV-cache swap library for one MI355X (gfx950).
 *
 * The operations are the two the paper's hierarchical memory manager is built
 * on (Section 5, first paragraph): "preempt" moves the KV cache of a preempted
 * request out of GPU memory into host memory, "resume" reloads it when the
 * request runs again; plus the incremental write-through of Section 5.1, where
 * only KV produced since the previous offload is written to the host.  The
 * paper works at request granularity above a token-level pool (Section 3.1,
 * "Request Offload Manager" and "Hierarchical KV Cache Manager"), batches its
 * transfers and runs them on dedicated eviction / loading streams ordered by
 * events (Section 6, "KV Cache Manager").  This header fixes the byte-level
 * contract the paper leaves open.
 *
 * ---------------------------------------------------------------------------
 * Geometry
 *   L = num_layers, H = num_kv_heads, D = head_dim, B = block_size (tokens),
 *   e = bytes per element (2 for f16/bf16, 1 for fp8), N = num_blocks.
 *   chunk       = B*H*D*e bytes: the K *or* V data of one block in one layer.
 *                 A chunk is contiguous in the device pool.
 *   block_bytes = 2*L*chunk.
 *   With scales (fp8): scale_chunk = H*4 bytes per (block, layer, K|V),
 *                 block_scale_bytes = 2*L*H*4.
 *   S           = block_bytes + block_scale_bytes : one staging slot.
 *
 * Device pool addressing (bytes, all strides caller-given):
 *   chunk(l, c, p)  at pool_dev  + l*layer_stride + c*kv_stride + p*block_stride
 *   scales(l, c, p) at scale_dev + l*scale_layer_stride + c*scale_kv_stride
 *                                + p*scale_block_stride
 *   l in [0,L), c in {0 = K, 1 = V}, p in [0,N).
 *
 * Staging arena: staging_bytes / S slots of S bytes.  A request owns a
 * contiguous extent of slots [base, base+cap).  Logical block j of the request
 * lives in slot base+j:
 *   data   of (l, c) at slot_offset + (2*l + c)*chunk
 *   scales of (l, c) at slot_offset + block_bytes + (2*l + c)*H*4
 * Inside a chunk the byte order of the pool is preserved.
 * Extents are placed first-fit at the lowest free slot index, so placement is
 * a deterministic function of the call history.
 *
 * Per-request state kept by the library, keyed by request id:
 *   base, cap     staging extent
 *   staged        number of leading logical blocks whose staging copy is valid
 *   wm            watermark: number of leading FULL blocks already written
 *                 through (Section 5.1: only newer blocks need writing)
 *   swapped       set by kv_swap_out, cleared by kv_swap_in
 *
 * Conventions
 *   - Every entry point returns 0 (KV_OK) or a negative KV_E* code.  No C++
 *     exception crosses the boundary.
 *   - All-or-nothing: a call checks every request and every block id before it
 *     changes any state or enqueues any work.  KV_EHIP and KV_ENOMEM are the exception: a HIP
 *     runtime failure or an allocation failure in the middle of a call leaves bookkeeping and
 *     streams out of step.  The handle remembers it: every later call that would change state or
 *     enqueue work returns KV_EHIP without doing anything; kv_req_query, kv_io_stats_get and
 *     kv_last_hip_error still answer, and kv_pool_destroy releases everything.
 *   - Calls are asynchronous.  Swap-out / delta / move work is enqueued on the evict stream,
 *     swap-in work on the load stream, in issue order.  The library inserts every cross-stream
 *     wait the two streams need between themselves: for staging slots (a swap-in reads slots an
 *     unfinished swap-out writes; a swap-out reuses slots an unfinished swap-in still reads) and
 *     for device blocks (a swap-in is handed blocks an unfinished swap-out or move still reads;
 *     a swap-out or move reads blocks an unfinished swap-in still writes).  Section 5.3 runs
 *     eviction and loading at the same time and requires that no block or slot is reused before
 *     its previous user has finished: these waits are what keeps that true here.
 *     Each segment of a transfer (the whole call without KV_REQ_EVENTS) waits only for the newest
 *     conflicting segment of the other stream, so a swap-in may be handed the blocks of a request
 *     whose eviction has just been enqueued and fills them piece by piece behind it.
 *     Work of OTHER streams (the model's compute) is the caller's to order, through wait_event
 *     and kv_sync / kv_req_wait.
 *   - wait_event (nullable) is a hipEvent_t; the call's stream waits for it
 *     before touching the pool (ordering after the caller's compute stream).
 *   - Argument arrays are HOST pointers, read during the call, free on return.
 *   - pool_dev, scale_dev, bounce_dev are DEVICE pointers; staging_host is a
 *     pinned, device-mapped HOST pointer (hipHostMalloc / torch pin_memory),
 *     or a device pointer when KV_STAGING_DEVICE is set.  All are owned by the
 *     caller and must outlive the pool handle.  Base pointers and strides must
 *     be multiples of 16 bytes (scale pointers/strides: multiples of 4).
 *   - A handle is used by one thread at a time.
 */
#ifndef KVSWAP_H
#define KVSWAP_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct kv_pool kv_pool; /* opaque */

typedef enum { KV_F16 = 0, KV_BF16 = 1, KV_FP8_E4M3 = 2 } kv_dtype;

/* status codes */
enum {
  KV_OK = 0,
  KV_EINVAL = -1, /* null/misaligned pointer, bad geometry, bad CSR, repeated request id,
                     row length not matching the token count */
  KV_ERANGE = -2, /* physical block id outside [0, N) */
  KV_EDUP = -3,   /* the same destination block listed twice in one kv_swap_in / kv_move_blocks */
  KV_ENOENT = -4, /* request id unknown */
  KV_EEXIST = -5, /* request already swapped out (kv_swap_out twice, or delta after swap-out) */
  KV_ENOSPC = -6, /* staging arena cannot hold the extent (or cannot grow it in place) */
  KV_EHIP = -7,   /* a HIP runtime call failed; kv_last_hip_error() returns its code */
  KV_ESTATE = -8, /* token count below the watermark (a request never shrinks) */
  KV_ENOMEM = -9, /* host memory for the library's own bookkeeping could not be allocated */
  KV_E2BIG = -10  /* kv_move_blocks_noalloc: more than KV_NOALLOC_MAX_BLOCKS blocks in one call */
};

/* kv_pool_config.flags */
enum {
  KV_PATH_AUTO = 0u,      /* zero-copy, except: with a bounce buffer, transfers of 8 MiB and more
                             go through it and the copy engines (robust next to running compute) */
  KV_PATH_DMA = 1u,       /* gather into bounce_dev, then hipMemcpyAsync (needs bounce_dev) */
  KV_PATH_ZEROCOPY = 2u,  /* kernels store to / load from the mapped host arena directly */
  KV_STAGING_DEVICE = 4u, /* staging_host is device memory: the on-device gather/scatter */
  KV_PLAN_ONLY = 8u,      /* no HIP call is ever made: bookkeeping and descriptor lists only
                             (host-logic tests on machines without a GPU) */
  KV_REQ_EVENTS = 16u     /* cut every call into segments that end on request boundaries (32 MiB or
                             more each, see KV_TUNE_SEGMENT_BYTES) and record an event per segment, so
                             that each request's completion can be polled, waited for and timed, and so
                             that device-block hazards between the two streams are resolved segment by
                             segment instead of call by call */
};

/* kv_swap_out_delta flags */
enum { KV_DELTA_INCLUDE_TAIL = 1u };
/* kv_swap_in flags */
enum { KV_KEEP_STAGING = 1u };

typedef struct {
  uint32_t struct_size; /* sizeof(kv_pool_config), checked */
  int32_t num_layers, num_kv_heads, head_dim, block_size; /* L, H, D, B */
  int32_t dtype;      /* kv_dtype; only the element size matters to the copy */
  int64_t num_blocks; /* N */
  void* pool_dev;
  int64_t layer_stride, kv_stride, block_stride; /* bytes */
  void* scale_dev; /* NULL unless per-(block, layer, K|V, head) fp32 scales exist */
  int64_t scale_layer_stride, scale_kv_stride, scale_block_stride; /* bytes */
  void* staging_host;
  int64_t staging_bytes;
  void* bounce_dev; /* optional, for KV_PATH_DMA; first half serves swap-out, second swap-in */
  int64_t bounce_bytes;
  void* evict_stream; /* hipStream_t; NULL: the library creates and owns one */
  void* load_stream;  /* hipStream_t; NULL: the library creates and owns one.  Eviction and loading overlap (Section 5.3)
                         only when the two streams sit on different hardware queues.  HIP gives a process a small number of
                         them (GPU_MAX_HW_QUEUES, four by default) and lets further streams share: a process that has
                         created other streams before should pass two streams it created, and used, early */
  uint32_t flags;
} kv_pool_config;

/* Figures of the most recent swap call on a handle. */
typedef struct {
  uint32_t struct_size;
  int32_t op;       /* 1 swap_out, 2 swap_out_delta, 3 swap_in, 4 move_blocks */
  int32_t path;     /* KV_PATH_DMA or KV_PATH_ZEROCOPY (the latter also for device staging) */
  int32_t launches; /* kernel launches enqueued */
  int32_t copies;   /* hipMemcpyAsync calls enqueued (descriptor upload not counted) */
  int32_t grid;     /* workgroups of the (last) data kernel */
  int64_t blocks;   /* blocks moved */
  int64_t bytes;    /* payload bytes = blocks * S */
  double plan_us;   /* host time spent validating and building descriptors */
  double enqueue_us; /* host time spent inside HIP enqueue calls */
  float ms_total;   /* first enqueue to last completion on the stream (HIP events) */
  float ms_kernel;  /* summed duration of the data kernels (HIP events around each launch); a call that is a
                       single launch and nothing else carries no events of its own and reports ms_total */
  int32_t scatter_order; /* large scatter with both ends in HBM: 0 block by block, 1 plane by plane; -1 otherwise */
  int32_t reserved;
} kv_stats;

/* Create a handle over caller-owned memory.  Validates geometry, alignment and
 * capacity; allocates only the library's own descriptor rings and events.
 * The GPU that holds pool_dev must be the current device of the calling thread
 * (the handle's streams and descriptor memory are created there; KV_EINVAL
 * otherwise).
 * Section 3.1 (separate CPU and GPU pools), Section 6 (dedicated streams). */
int kv_pool_create(const kv_pool_config* cfg, kv_pool** out);

/* Waits for all enqueued work, then frees the handle.  Caller memory untouched. */
int kv_pool_destroy(kv_pool* p);

/* Preempt (Section 5, operation (a)).  Block tables are CSR: request i owns
 * block_ids[offsets[i] .. offsets[i+1]) in logical order; the row length must
 * equal ceil(num_tokens[i] / B).  For every request: reserve an extent of that
 * many slots if it has none (grow it in place if it is too small), copy every
 * block — all layers, K and V, scales — into slots base+j, then staged = row
 * length, wm = floor(num_tokens/B), swapped = 1.  The partial tail block is
 * copied whole.  Repeated physical ids in a table are legal (read twice).
 * Device blocks are left untouched.
 * Errors: KV_EINVAL, KV_ERANGE, KV_EEXIST (already swapped), KV_ENOSPC, KV_EHIP. */
int kv_swap_out(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                const int32_t* block_ids, const int32_t* num_tokens, void* wait_event);

/* Incremental write-through (Section 5.1; sized, ordered writes: Section 5.2).
 * Requests are served in the order given (the caller's priority order).  For
 * each: hi = floor(num_tokens/B), or ceil with KV_DELTA_INCLUDE_TAIL;
 * m = min(hi, wm + budget left) (budget 0 = unlimited; if hi <= wm nothing
 * moves); logical blocks [wm, m) are copied to slots base+wm.. ; the budget is
 * charged m - wm; staged = max(staged, m); wm = min(m, floor(num_tokens/B));
 * blocks_moved[i] (nullable) = m - old wm.  A block is never split.  The row
 * length must be >= ceil(num_tokens/B).  An unknown request gets an extent of
 * row-length slots; a known one is grown in place when the row is longer than
 * its capacity.
 * Errors: as kv_swap_out, plus KV_ESTATE when num_tokens < wm*B. */
int kv_swap_out_delta(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                      const int32_t* block_ids, const int32_t* num_tokens, int64_t block_budget,
                      uint32_t flags, int32_t* blocks_moved, void* wait_event);

/* Resume (Section 5, operation (b)).  Row i lists the freshly allocated
 * destination blocks of request i; its length must equal staged.  Slot base+j
 * is copied into block new_block_ids[offsets[i]+j] for all layers, K and V,
 * scales.  No other pool byte is written.  All destination ids of one call
 * must be distinct.  Afterwards the request is forgotten and its extent freed,
 * unless KV_KEEP_STAGING: then the extent, staged and wm stay (the host copy
 * remains a valid write-through image, Section 5.3) and swapped = 0.
 * Errors: KV_EINVAL, KV_ERANGE, KV_EDUP, KV_ENOENT, KV_EHIP. */
int kv_swap_in(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
               const int32_t* new_block_ids, uint32_t flags, void* wait_event);

/* Eviction and loading at once (Section 5.3: the two run concurrently, and blocks freed by the eviction are handed
 * to the load).  The result is that of kv_swap_out(first set) followed by kv_swap_in(second set); the destination
 * blocks of the load may be blocks of the requests being evicted.  The call is all-or-nothing as a whole: the load is
 * checked before the eviction changes anything.  A request id may appear in one set only (KV_EINVAL).  On the
 * zero-copy path the two transfers are cut into phases of KV_TUNE_PHASE_BYTES (256 MiB) and interleaved on the two
 * streams so that one eviction kernel and one load kernel always start together, each load phase waiting only for
 * the eviction phase that frees its blocks; per-request completion (kv_req_poll / kv_req_wait) follows the phases.
 * On the copy-engine path and under KV_PLAN_ONLY it is the two calls one after the other.  kv_last_stats and
 * kv_last_plan afterwards report the load.
 * Errors: those of kv_swap_out and kv_swap_in. */
int kv_evict_and_load(kv_pool* p, int32_t n_out, const uint64_t* out_ids, const int32_t* out_offsets,
                      const int32_t* out_block_ids, const int32_t* out_tokens, int32_t n_in, const uint64_t* in_ids,
                      const int32_t* in_offsets, const int32_t* in_block_ids, uint32_t in_flags, void* wait_event);

/* Blocks the calling thread until everything enqueued on this handle is done
 * (Section 6: completion is signalled through events). */
int kv_sync(kv_pool* p);

/* On-device move of whole blocks inside the pool: block src_ids[i] is copied to
 * dst_ids[i] (all layers, K, V, scales).  Destinations must be distinct and
 * must not appear among the sources.  Runs on the evict stream.  This is the
 * pool-to-pool form of the gather/scatter whose both ends are in HBM. */
int kv_move_blocks(kv_pool* p, int64_t n, const int32_t* src_ids, const int32_t* dst_ids,
                   void* wait_event);

/* kv_move_blocks for callers that cannot allocate: code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc.  Same arguments, same result in the pool, same kernel.  The call makes no hipMalloc,
 * hipFree, hipHostMalloc, event or stream creation and no host-heap allocation: its descriptors travel inside the
 * arguments of small fill launches (448 per launch) into a fixed device array that is part of the library's code
 * object (KV_NOALLOC_MAX_BLOCKS descriptors of 8 bytes = 512 KiB per GPU, held until the process ends).
 *   - n > KV_NOALLOC_MAX_BLOCKS returns KV_E2BIG and does nothing; split the list.
 *   - Runs on the evict stream after everything enqueued on either stream of this handle before it; load-stream
 *     calls made while it is unfinished wait for it as a whole (it keeps no per-block marks).
 *   - All calls on one GPU share that GPU's array.  Calls through one handle are ordered by its evict stream.
 *     Calls through DIFFERENT handles on the same GPU that overlap in time race for the array: the caller must
 *     order them (kv_sync, events).  The array keeps the last call's descriptors; each call overwrites the part
 *     it reads, nothing has to start at zero.
 *   - The call never waits for the device on the host.
 *   - kv_last_stats afterwards reports blocks, bytes, grid and host times, no stream times (no events are taken).
 * Errors: KV_EINVAL, KV_ERANGE, KV_EDUP as kv_move_blocks; KV_E2BIG; KV_EHIP. */
#define KV_NOALLOC_MAX_BLOCKS 65536
int kv_move_blocks_noalloc(kv_pool* p, int64_t n, const int32_t* src_ids, const int32_t* dst_ids,
                           void* wait_event);

/* ---- helpers (bookkeeping, statistics, tuning) ---- */

/* Reserve an extent of max_blocks slots for a request before its first delta
 * (write-through appends, so the extent must be able to hold the final length).
 * KV_EEXIST if the request is known. */
int kv_req_reserve(kv_pool* p, uint64_t req_id, int32_t max_blocks);
/* Forget a request and free its extent.  KV_ENOENT if unknown. */
int kv_req_release(kv_pool* p, uint64_t req_id);
/* Any out pointer may be NULL.  staging_offset is in bytes from staging_host. */
int kv_req_query(kv_pool* p, uint64_t req_id, int64_t* staging_offset, int32_t* cap_blocks,
                 int32_t* blocks_staged, int32_t* watermark, int32_t* swapped);
/* Write queue (Section 5.2: the KV a decode iteration produces is buffered, and after each iteration a
 * chunk sized to the next compute interval is written out, requests with larger buffers first).
 * The queue lives in the handle, so the serving loop posts only what changed and drains once per
 * iteration.
 *
 * kv_wq_post    records, for each request, its current block table (CSR as in kv_swap_out_delta), token
 *               count and priority (NULL: 0), replacing what an earlier post recorded for it.  The
 *               arrays are copied.  Errors (nothing recorded): KV_EINVAL (a row shorter than the token
 *               count needs, a request named twice, NaN priority), KV_ERANGE (block id), KV_EEXIST
 *               (request is swapped out), KV_ESTATE (fewer tokens than already written through).
 * kv_wq_drain   one kv_swap_out_delta over the queued requests in order of decreasing priority (ties:
 *               order of posting).  Budget: block_budget > 0: that many blocks; else interval_us > 0:
 *               kv_budget_blocks(p, 0, interval_us), where 0 means nothing moves; both 0: unlimited.
 *               flags as kv_swap_out_delta.  An entry whose token count a direct kv_swap_out_delta has
 *               meanwhile gone past has nothing to write and is skipped.  blocks_written, blocks_pending (full blocks still not
 *               written through, over the whole queue) and budget_used are nullable.  A planning error
 *               (KV_ENOSPC, ...) leaves queue and state unchanged.
 * kv_wq_remove  forgets a request (KV_ENOENT if it is not queued).  kv_swap_out, kv_swap_in and
 *               kv_req_release do this for the requests they name: a request's entry must not outlive its
 *               block table, and a caller that gives up blocks in another way removes or re-posts it.
 * kv_wq_pending full blocks not yet written through, and the number of requests that have some. */
int kv_wq_post(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets, const int32_t* block_ids,
               const int32_t* num_tokens, const double* priority);
int kv_wq_drain(kv_pool* p, double interval_us, int64_t block_budget, uint32_t flags, int64_t* blocks_written,
                int64_t* blocks_pending, int64_t* budget_used, void* wait_event);
int kv_wq_remove(kv_pool* p, uint64_t req_id);
int kv_wq_pending(kv_pool* p, int64_t* blocks, int32_t* requests);

/* Waits for the most recent swap call to finish, then reports it. */
int kv_last_stats(kv_pool* p, kv_stats* out);
/* Bytes of one staging slot (S) for this geometry. */
int64_t kv_slot_bytes(const kv_pool* p);
/* Descriptor list of the most recent swap call: pairs (phys_block, staging_slot)
 * in launch order.  Copies at most cap pairs; returns the number the call
 * produced.  Meant for host-logic tests under KV_PLAN_ONLY. */
int64_t kv_last_plan(kv_pool* p, int32_t* phys, int64_t* slot, int64_t cap);

/* Per-request completion (needs KV_REQ_EVENTS; Section 6: a control thread follows the transfers
 * through events; Section 5.3: blocks of a request whose eviction has finished can be reused while
 * the rest of the burst is still moving).
 * kv_req_poll: 1 when no transfer of this request is in flight (or none was ever enqueued), 0 while
 * its last enqueued segment is unfinished.  kv_req_wait blocks until then; it does not hold the
 * handle's lock while it blocks, so another thread may go on enqueuing calls meanwhile (kv_sync does
 * hold it: it is the call that stops everything).  Without KV_REQ_EVENTS both answer for the whole
 * call the request was part of. */
int kv_req_poll(kv_pool* p, uint64_t req_id);
int kv_req_wait(kv_pool* p, uint64_t req_id);
/* Completion times of the requests of the most recent swap call, in milliseconds of stream time
 * from the start of that call, in call order.  Waits for the call.  Copies at most cap entries,
 * returns how many requests the call moved data for. */
int64_t kv_last_timeline(kv_pool* p, uint64_t* req_ids, float* done_ms, int64_t cap);

/* I/O telemetry for a scheduler (Section 4.3: the memory manager exposes queue lengths and
 * transfer rates so that t_IO = evict queueing + evict + load queueing + load can be estimated;
 * Section 5.2: writes are sized to fit the next compute interval).  Index 0 = evict stream
 * (swap-out, delta), 1 = load stream (swap-in). */
typedef struct {
  uint32_t struct_size;
  int32_t inflight_calls[2]; /* calls enqueued and not yet finished */
  int64_t inflight_bytes[2]; /* their payload */
  int64_t total_calls[2];    /* finished calls accounted so far */
  int64_t total_bytes[2];
  double ewma_gbps[2];       /* payload rate of finished calls of 4 MiB and more (0: none yet) */
  double ewma_small_us[2];   /* stream time of finished calls below 4 MiB: the fixed cost (0: none yet) */
} kv_io_stats;
int kv_io_stats_get(kv_pool* p, kv_io_stats* out);

/* Blocks that a transfer enqueued now on stream `dir` (0 evict, 1 load) can move so that it
 * finishes within interval_us: floor((interval_us - fixed - inflight_bytes/rate) * rate / S),
 * never negative, with rate = ewma_gbps (32 GB/s until measured) and fixed = ewma_small_us
 * (50 us until measured).  Feed it to kv_swap_out_delta as block_budget; a result of 0 means
 * "nothing fits": do not pass it on, since a budget of 0 means unlimited there. */
int64_t kv_budget_blocks(kv_pool* p, int32_t dir, double interval_us);

/* Section 5.2 in one call: "synchronous chunked writing".  The requests are served in order of
 * decreasing priority[i] (the scheduler's buffer sizes: a request with a larger buffer is the more
 * likely victim; ties and priority == NULL: call order) under the block budget that
 * kv_budget_blocks(p, 0, interval_us) gives at this moment, so that the write ends inside the next
 * compute interval.  Otherwise as kv_swap_out_delta; blocks_moved is in the caller's order;
 * budget_used (nullable) receives the budget applied.  If nothing fits, nothing moves (the
 * arguments are still checked and extents reserved). */
int kv_swap_out_delta_timed(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                            const int32_t* block_ids, const int32_t* num_tokens, const float* priority,
                            double interval_us, uint32_t flags, int32_t* blocks_moved, int64_t* budget_used,
                            void* wait_event);

/* Launch-shape knobs: value 0 restores the default. */
enum {
  KV_TUNE_MAX_WGS_DEVICE = 1, /* workgroup cap when both ends are in HBM */
  KV_TUNE_MAX_WGS_LINK = 2,   /* workgroup cap when one end is host memory (CU budget; default 64, which saturates the
                                 link in one direction; a caller that keeps both directions busy with separate calls
                                 gains 5-7 % aggregate with 128-160) */
  KV_TUNE_KERNEL_VARIANT = 3, /* 0 default; other values select experimental kernels */
  KV_TUNE_DMA_SLICE_BLOCKS = 4, /* blocks per gather+copy slice on the DMA path */
  KV_TUNE_SEGMENT_BYTES = 5,    /* smallest segment under KV_REQ_EVENTS (default 32 MiB) */
  KV_TUNE_SCALE_LDS = 6,        /* scale side band: 0 default (LDS for the scatter), 1 word by word, 2 LDS both ways */
  KV_TUNE_SCATTER_ORDER = 8,    /* scatter of 1024 blocks and more with both ends in HBM: 0 default (the handle times
                                   both job orders on its first two such calls and keeps the faster), 1 always block
                                   by block, 2 plane by plane over descriptors sorted by destination block, whatever the size */
  KV_TUNE_PHASE_BYTES = 9,      /* kv_evict_and_load: bytes of one phase per direction (default 256 MiB) */
  KV_TUNE_PHASE_WGS_OUT = 10,   /* kv_evict_and_load: workgroups of an eviction phase (default 128) */
  KV_TUNE_PHASE_WGS_IN = 11,    /* kv_evict_and_load: workgroups of a load phase (default 128: with both directions of
                                   the link busy each kernel needs more requests in flight than alone, and the two do
                                   best with equal counts) */
  KV_TUNE_LINK_IN_WGS = 14,     /* workgroups of the scatter out of the host arena alone (0: as KV_TUNE_MAX_WGS_LINK) */
  KV_TUNE_LINK_IN_UNROLL = 15,  /* 16-byte loads in flight per lane of that scatter: 1, 2, 4, 8 (0: by chunk size) */
  KV_TUNE_HOST_STORES = 13,     /* zero-copy gather into the host arena: 0 (default) each lane writes 64 consecutive bytes with
                                   ordinary stores that L2 merges into full lines; 1 whole 128-byte lines per store instruction,
                                   non-temporal */
  KV_TUNE_KERNEL_EVENTS = 12,   /* 1: every data kernel is bracketed by its own pair of events, so that kv_stats.ms_kernel
                                   is the kernel alone also for a call that is a single launch (otherwise such a call
                                   reports its whole stream time, descriptor upload included); for measurements */
  KV_TUNE_SEGMENT_MAX_BYTES = 7 /* under KV_REQ_EVENTS: also cut a segment inside a long request once it reaches this
                                   many bytes (0, the default: only at request ends).  Smaller segments let a swap-in
                                   follow closer behind an eviction whose blocks it reuses, at one launch each */
};
int kv_pool_tune(kv_pool* p, int32_t what, int64_t value);

int kv_last_hip_error(const kv_pool* p);
const char* kv_strerror(int code);

/* ------------------------------------------------------------ measurement helpers
 * Ceilings the swap is compared against (the paper prints no bandwidth figure; Section 5.2 only asks that
 * writes use the link fully, so the link's own measured rate is the yardstick); no pool handle needed.  All four are
 * synchronous and return the mean milliseconds per iteration, or
 * a negative number for bad arguments (-1), a failed HIP resource (-2) or a failed wait (-3).
 *   kv_bench_copy        contiguous device-to-device copy kernel of `bytes` (multiple of 16 KiB) on `stream`:
 *                        the HBM copy ceiling.  grid 0: one workgroup per 4 KiB piece (the launch shape of
 *                        the on-device gather/scatter, the fastest plain copy); grid > 0: at most that many
 *                        workgroups, grid-stride, 16 KiB pieces.
 *   kv_bench_copy_scrambled  the same one-workgroup-per-4-KiB copy with the source (which 0) or the destination
 *                        (which 1) visited in runs of run_bytes in a scrambled order: the ceiling of a gather
 *                        from / a scatter into a paged pool whose chunks are that long.  run_bytes (16 bytes or
 *                        more) and bytes / run_bytes must be powers of two, bytes a multiple of 4 KiB.
 *   kv_bench_link        one contiguous hipMemcpyAsync between PINNED host memory and device memory on
 *                        `stream`; dir 0 device -> host, 1 host -> device: the host-link ceiling.
 *   kv_bench_link_bidir  both directions at once on two internal streams (dev_a -> host_a while
 *                        host_b -> dev_b); time until both copies of a pair have finished. */
double kv_bench_copy(void* dst_dev, const void* src_dev, int64_t bytes, int32_t grid, int32_t iters, void* stream);
double kv_bench_copy_scrambled(void* dst_dev, const void* src_dev, int64_t bytes, int64_t run_bytes, int32_t which,
                               int32_t iters, void* stream);
double kv_bench_link(void* host_pinned, void* dev, int64_t bytes, int32_t dir, int32_t iters, void* stream);
double kv_bench_link_bidir(void* host_a, const void* dev_a, const void* host_b, void* dev_b, int64_t bytes,
                           int32_t iters);

#ifdef __cplusplus
}
#endif
#endif /* KVSWAP_H */
