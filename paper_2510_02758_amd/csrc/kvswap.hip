// C ABI of the paged KV-cache swap for MI355X (declared in include/kvswap.h).
//
// Host side of each call: plan (planner.hpp) -> descriptor list -> one batched
// launch per direction on the evict or load stream (paper Section 6: dedicated
// streams for eviction and loading, batched transfers, event-based completion).
// Two transfer paths exist for the host link:
//   zero-copy  the gather/scatter kernel addresses the pinned host arena itself;
//   DMA        gather into a device bounce buffer, then hipMemcpyAsync of each
//              run of consecutive staging slots (and the mirror image for loads).
// With KV_STAGING_DEVICE the arena is HBM and the same kernels give the
// on-device gather/scatter.
#include "runtime.hip.inc"

// Entry of a call that changes state or enqueues work: takes the handle's lock and refuses a handle on which an
// earlier call failed half-way (KV_EHIP, KV_ENOMEM): its bookkeeping no longer describes what the streams hold.
#define KV_ENTER(p)                       \
  std::lock_guard<std::mutex> g((p)->mu); \
  if ((p)->broken) return KV_EHIP
// Every entry point is a function-try-block that ends in this handler: no exception leaves through the C boundary.
#define KV_CATCH(p) \
  catch (...) { return on_exception(p); }

// ---- the fixed descriptor array of kv_move_blocks_noalloc ----
// One array per GPU the library runs on, part of the loaded code object until the process ends
// (KV_NOALLOC_MAX_BLOCKS descriptors of 8 bytes = 512 KiB).  In host code the name `scratch` is only a stand-in
// for the symbol: the address the kernels and copies use is looked up once per device, with that device current,
// and kept in kScratchOn[device]; each GPU holds its own copy at its own address.
static __device__ __align__(256) kvswap::Desc scratch[KV_NOALLOC_MAX_BLOCKS];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
Desc* kScratchOn[kMaxDevices] = {};

// Address of `scratch` on the current device (looked up on first use); *dev_out receives the device.
hipError_t scratch_on_current_device(Desc** out, int* dev_out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidValue;
  std::lock_guard<std::mutex> g(g_scratch_mu);
  if (!kScratchOn[dev]) {
    Desc* ptr = nullptr;
    e = hipGetSymbolAddress((void**)&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidValue;
    kScratchOn[dev] = ptr;
  }
  *out = kScratchOn[dev];
  *dev_out = dev;
  return hipSuccess;
}
}  // namespace

// Everything kv_move_blocks_noalloc will need, taken once when the handle is created: the address of the
// descriptor array on this GPU, two events and the duplicate bitmap.
static int noalloc_setup(kv_pool* p) {
  hipError_t e = scratch_on_current_device(&p->na_dev, &p->device);
  if (e != hipSuccess) {
    p->last_hip = (int)e;
    return KV_EHIP;
  }
  HIPCHK(p, hipEventCreate(&p->na_fence_ev));
  HIPCHK(p, hipEventCreate(&p->na_done_ev));
  p->na_mark.assign((size_t)((p->cfg.num_blocks + 63) / 64), 0);
  return KV_OK;
}

extern "C" {

int kv_pool_create(const kv_pool_config* cfg, kv_pool** out) {
#define REJECT(why)          \
  do {                       \
    KVDBG("rejected: " why); \
    return KV_EINVAL;        \
  } while (0)
  if (!cfg || !out) return KV_EINVAL;
  *out = nullptr;
  if (cfg->struct_size != sizeof(kv_pool_config)) REJECT("struct_size does not match this library");
  const int e = elem_bytes(cfg->dtype);
  if (e == 0 || cfg->num_layers <= 0 || cfg->num_kv_heads <= 0 || cfg->head_dim <= 0 || cfg->block_size <= 0 ||
      cfg->num_blocks <= 0 || cfg->num_blocks > INT32_MAX)
    REJECT("bad dtype or non-positive geometry");
  const bool plan_only = (cfg->flags & KV_PLAN_ONLY) != 0;
  const int64_t chunk = (int64_t)cfg->block_size * cfg->num_kv_heads * cfg->head_dim * e;
  if (chunk % 16 || chunk > (1 << 30)) REJECT("chunk (B*H*D*e) must be a multiple of 16 bytes and at most 1 GiB");
  if (cfg->layer_stride <= 0 || cfg->kv_stride <= 0 || cfg->block_stride <= 0 || cfg->layer_stride % 16 ||
      cfg->kv_stride % 16 || cfg->block_stride % 16)
    REJECT("pool strides must be positive multiples of 16 bytes");
  if (!plan_only && (!cfg->pool_dev || !cfg->staging_host)) REJECT("pool_dev and staging_host are required");
  if (((uintptr_t)cfg->pool_dev | (uintptr_t)cfg->staging_host | (uintptr_t)cfg->bounce_dev) % 16)
    REJECT("pool_dev, staging_host and bounce_dev must be 16-byte aligned");
  if (cfg->staging_bytes < 0 || cfg->bounce_bytes < 0) REJECT("negative size");
  const bool scales = cfg->scale_dev != nullptr || (plan_only && cfg->scale_block_stride > 0);
  int64_t scale_chunk = 0;
  if (scales) {
    scale_chunk = (int64_t)cfg->num_kv_heads * 4;
    if (cfg->scale_layer_stride <= 0 || cfg->scale_kv_stride <= 0 || cfg->scale_block_stride <= 0 ||
        cfg->scale_layer_stride % 4 || cfg->scale_kv_stride % 4 || cfg->scale_block_stride % 4 ||
        (uintptr_t)cfg->scale_dev % 4)
      REJECT("scale pointer and strides must be positive multiples of 4 bytes");
    // keeps every staging slot 16-byte aligned
    if ((2 * cfg->num_layers * scale_chunk) % 16) REJECT("2*L*H*4 must be a multiple of 16 bytes");
  }
  if ((cfg->flags & KV_PATH_DMA) && (cfg->flags & KV_PATH_ZEROCOPY)) REJECT("both transfer paths forced");
  if ((cfg->flags & KV_PATH_DMA) && (cfg->flags & KV_STAGING_DEVICE)) REJECT("DMA path with a device arena");
#undef REJECT

  kv_pool* p = new (std::nothrow) kv_pool;
  if (!p) return KV_ENOMEM;
  try {
    p->cfg = *cfg;
    p->plan_only = plan_only;
    p->dev_staging = (cfg->flags & KV_STAGING_DEVICE) != 0;
    p->req_events = (cfg->flags & KV_REQ_EVENTS) != 0;
    p->chunk = chunk;
    p->block_bytes = 2 * (int64_t)cfg->num_layers * chunk;
    p->scale_chunk = scale_chunk;
    p->block_scale_bytes = 2 * (int64_t)cfg->num_layers * scale_chunk;
    p->S = p->block_bytes + p->block_scale_bytes;
    p->slots = cfg->staging_bytes / p->S;
    if (p->slots > INT32_MAX) p->slots = INT32_MAX;
    if (!scales) p->cfg.scale_dev = nullptr;
    p->planner.init(cfg->num_blocks, cfg->block_size, p->slots);
    if ((cfg->flags & KV_PATH_DMA) && (!cfg->bounce_dev || (cfg->bounce_bytes / 2) / p->S < 1)) {
      KVDBG("rejected: the DMA path needs a bounce buffer of at least two slots");
      delete p;
      return KV_EINVAL;
    }
    if (plan_only) {
      *out = p;
      return KV_OK;
    }

    // The kernels trust these extents: refuse a pool whose strides leave its allocation.
    const int64_t pool_need = (cfg->num_layers - 1) * cfg->layer_stride + cfg->kv_stride +
                              (cfg->num_blocks - 1) * cfg->block_stride + chunk;
    bool ok = range_ok(cfg->pool_dev, pool_need, true);
    if (!ok) KVDBG("pool strides reach %lld bytes, past the end of the allocation", (long long)pool_need);
    if (ok && scales) {
      ok = range_ok(cfg->scale_dev, (cfg->num_layers - 1) * cfg->scale_layer_stride + cfg->scale_kv_stride +
                                        (cfg->num_blocks - 1) * cfg->scale_block_stride + scale_chunk, true);
      if (!ok) KVDBG("scale strides reach past the end of the allocation");
    }
    if (ok && !range_ok(cfg->staging_host, cfg->staging_bytes, (cfg->flags & KV_STAGING_DEVICE) != 0)) {
      ok = false;
      KVDBG("staging_bytes reaches past the end of the arena allocation");
    }
    if (ok && cfg->bounce_dev && !range_ok(cfg->bounce_dev, cfg->bounce_bytes, true)) {
      ok = false;
      KVDBG("bounce_bytes reaches past the end of the bounce allocation");
    }
    if (ok) {
      hipPointerAttribute_t at;
      hipError_t er = hipPointerGetAttributes(&at, cfg->pool_dev);
      if (er != hipSuccess || at.type != hipMemoryTypeDevice) {
        ok = false;
        KVDBG("pool_dev is not device memory (hip error %d, memory type %d)", (int)er, er == hipSuccess ? (int)at.type : -1);
      }
      (void)hipGetLastError();
      // The handle's streams, events and descriptor memory belong to the device that is current now: the pool must
      // live there too.
      int cur = -1;
      if (ok && (hipGetDevice(&cur) != hipSuccess || at.device != cur)) {
        ok = false;
        KVDBG("pool_dev lives on device %d, the current device is %d: make the pool's device current first", at.device, cur);
      }
      if (ok) {
        er = hipPointerGetAttributes(&at, cfg->staging_host);
        if (er != hipSuccess) {
          ok = false;  // pageable or unknown memory cannot be a staging arena
          KVDBG("staging_host is unknown to HIP (error %d): it must be pinned memory", (int)er);
        } else if (p->dev_staging ? at.type != hipMemoryTypeDevice : at.type != hipMemoryTypeHost) {
          ok = false;
          KVDBG("staging_host has memory type %d, expected %s memory", (int)at.type, p->dev_staging ? "device" : "pinned host");
        } else {
          p->arena_dev = (char*)(at.devicePointer ? at.devicePointer : cfg->staging_host);
        }
        (void)hipGetLastError();
      }
    }
    if (!ok) {
      delete p;
      return KV_EINVAL;
    }
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess)
      p->cu_count = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    void* given[2] = {cfg->evict_stream, cfg->load_stream};
    int rc = KV_OK;
    for (int s = 0; s < 2 && !rc; s++) {
      if (given[s]) {
        p->stream[s] = (hipStream_t)given[s];
      } else {
        hipError_t er = hipStreamCreateWithFlags(&p->stream[s], hipStreamNonBlocking);
        if (er != hipSuccess) {
          p->last_hip = (int)er;
          rc = KV_EHIP;
        } else {
          p->own_stream[s] = true;
        }
      }
    }
    if (!rc) rc = grow_ring(p, ring_entries_for(cfg->num_blocks));
    if (!rc) {
      p->blk_reader.assign((size_t)cfg->num_blocks, BlkMark{0, -1});
      p->blk_writer.assign((size_t)cfg->num_blocks, BlkMark{0, -1});
    }
    if (!rc) rc = noalloc_setup(p);
    if (rc) {
      kv_pool_destroy(p);
      return rc;
    }
    *out = p;
    return KV_OK;
  } catch (...) {  // the containers of the handle could not be allocated
    (void)kv_pool_destroy(p);
    return KV_ENOMEM;
  }
}

int kv_pool_destroy(kv_pool* p) try {
  if (!p) return KV_EINVAL;
  int rc = KV_OK;
  if (!p->plan_only) {
    for (int s = 0; s < 2; s++)
      if (p->stream[s] && hipStreamSynchronize(p->stream[s]) != hipSuccess) rc = KV_EHIP;
    for (auto& c : p->calls) recycle(p, c);
    for (auto ev : p->ev_free) (void)hipEventDestroy(ev);
    if (p->ring_host) (void)hipHostFree(p->ring_host);
    if (p->ring_dev) (void)hipFree(p->ring_dev);
    if (p->na_fence_ev) (void)hipEventDestroy(p->na_fence_ev);
    if (p->na_done_ev) (void)hipEventDestroy(p->na_done_ev);
    for (int s = 0; s < 2; s++)
      if (p->own_stream[s]) (void)hipStreamDestroy(p->stream[s]);
  }
  delete p;
  return rc;
}
catch (...) {
  return KV_ENOMEM;  // nothing in here allocates beyond the event free list; the handle is not touched again
}

static int swap_out_common(kv_pool* p, int op, Plan& plan, double t0, void* wait_event) {
  p->last_plan = plan.desc;
  const double t1 = now_us();
  if (p->plan_only) {
    p->plan_stats = kv_stats{};
    fill_plan_stats(p, &p->plan_stats, op, plan.desc.size(), t1 - t0);
    return KV_OK;
  }
  // slots this call writes may still be read by an unfinished swap-in
  const uint64_t fresh_dep = pending_user(p, kEvict, plan.fresh);
  const uint64_t dep = std::max(cross_stream(p, kEvict, plan.wait_in_seq), fresh_dep);
  if (plan.desc.empty() && !wait_event) {  // nothing to enqueue
    // The call may still have taken slots (a new request below one block, a request that grew into a new partial
    // block).  Nothing is written to them now, so no stream waits here; the requests remember the reader instead,
    // and their next write-through waits for it, as after kv_req_reserve.
    if (fresh_dep)
      for (uint64_t id : plan.fresh_ids)
        if (kvswap::Req* r = p->planner.find_mut(id)) r->in_seq = std::max(r->in_seq, fresh_dep);
    p->plan_stats = kv_stats{};
    fill_plan_stats(p, &p->plan_stats, op, 0, t1 - t0);
    p->last_instant = true;
    return KV_OK;
  }
  Call* c = nullptr;
  int rc = open_call(p, kEvict, op, dep, wait_event, 0, plan.desc, &c);
  if (rc) return rc;
  fill_plan_stats(p, &c->st, op, plan.desc.size(), t1 - t0);
  rc = enqueue_transfer(p, *c, plan, true);
  if (rc) return rc;
  rc = close_call(p, *c);
  if (rc) return rc;
  for (uint64_t id : plan.touched)
    if (kvswap::Req* r = p->planner.find_mut(id)) r->out_seq = c->seq;
  c->st.enqueue_us = now_us() - t1;
  return KV_OK;
}

int kv_swap_out(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets, const int32_t* block_ids,
                const int32_t* num_tokens, void* wait_event) try {
  if (!p) return KV_EINVAL;
  KV_ENTER(p);
  const double t0 = now_us();
  Plan plan;
  int rc = p->planner.plan_swap_out(n, req_ids, offsets, block_ids, num_tokens, &plan);
  if (rc) return rc;
  for (int32_t i = 0; i < n; i++) p->wq.erase(req_ids[i]);  // a swapped-out request has nothing left to write through
  return swap_out_common(p, 1, plan, t0, wait_event);
}
KV_CATCH(p)

int kv_swap_out_delta(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                      const int32_t* block_ids, const int32_t* num_tokens, int64_t block_budget, uint32_t flags,
                      int32_t* blocks_moved, void* wait_event) try {
  if (!p) return KV_EINVAL;
  KV_ENTER(p);
  const double t0 = now_us();
  Plan plan;
  int rc = p->planner.plan_delta(n, req_ids, offsets, block_ids, num_tokens, block_budget, flags, blocks_moved,
                                 &plan);
  if (rc) return rc;
  return swap_out_common(p, 2, plan, t0, wait_event);
}
KV_CATCH(p)

int kv_swap_in(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
               const int32_t* new_block_ids, uint32_t flags, void* wait_event) try {
  if (!p) return KV_EINVAL;
  KV_ENTER(p);
  const double t0 = now_us();
  Plan plan;
  int rc = p->planner.plan_swap_in(n, req_ids, offsets, new_block_ids, flags, &plan);
  if (rc) return rc;
  for (int32_t i = 0; i < n; i++) p->wq.erase(req_ids[i]);  // their tables have just changed
  p->last_plan = plan.desc;
  const double t1 = now_us();
  if (p->plan_only) {
    p->plan_stats = kv_stats{};
    fill_plan_stats(p, &p->plan_stats, 3, plan.desc.size(), t1 - t0);
    return KV_OK;
  }
  const uint64_t dep = cross_stream(p, kLoad, plan.wait_out_seq);
  if (plan.desc.empty() && !wait_event) {
    p->plan_stats = kv_stats{};
    fill_plan_stats(p, &p->plan_stats, 3, 0, t1 - t0);
    p->last_instant = true;
    return KV_OK;
  }
  Call* c = nullptr;
  rc = open_call(p, kLoad, 3, dep, wait_event, 1, plan.desc, &c);
  if (rc) return rc;
  fill_plan_stats(p, &c->st, 3, plan.desc.size(), t1 - t0);
  rc = enqueue_transfer(p, *c, plan, false);
  if (rc) return rc;
  rc = close_call(p, *c);
  if (rc) return rc;
  for (uint64_t id : plan.touched)
    if (kvswap::Req* r = p->planner.find_mut(id)) r->in_seq = c->seq;
  for (auto& f : plan.freed) p->pending.push_back({f.first, f.first + f.second, c->seq});
  c->st.enqueue_us = now_us() - t1;
  return KV_OK;
}
KV_CATCH(p)

// Section 5.3 in one call: kv_swap_out of the first set followed by kv_swap_in of the second, planned together so that
// the two transfers can be interleaved phase by phase on the two streams (see enqueue_in_phase).  Other paths than
// zero-copy get the two calls one after the other, which the per-segment ordering already overlaps.
int kv_evict_and_load(kv_pool* p, int32_t n_out, const uint64_t* out_ids, const int32_t* out_offsets,
                      const int32_t* out_block_ids, const int32_t* out_tokens, int32_t n_in, const uint64_t* in_ids,
                      const int32_t* in_offsets, const int32_t* in_block_ids, uint32_t in_flags, void* wait_event) try {
  if (!p) return KV_EINVAL;
  if (n_out < 0 || n_in < 0 || (n_out > 0 && !out_ids) || (n_in > 0 && !in_ids)) return KV_EINVAL;
  {
    std::lock_guard<std::mutex> g(p->mu);
    if (p->broken) return KV_EHIP;
    // a request is evicted or loaded, not both
    std::unordered_map<uint64_t, int> seen;
    for (int32_t i = 0; i < n_out; i++) seen.emplace(out_ids[i], 0);
    for (int32_t i = 0; i < n_in; i++)
      if (seen.count(in_ids[i])) return KV_EINVAL;
    // the load is checked before the eviction changes anything: the call is all-or-nothing as a whole
    int rc = p->planner.check_swap_in(n_in, in_ids, in_offsets, in_block_ids);
    if (rc) return rc;
    const bool in_phase = !p->plan_only && !use_dma(p, 1u << 30) && n_out > 0 && n_in > 0;
    if (in_phase) {
      const double t0 = now_us();
      Plan po, pi;
      rc = p->planner.plan_swap_out(n_out, out_ids, out_offsets, out_block_ids, out_tokens, &po);
      if (rc) return rc;
      rc = p->planner.plan_swap_in(n_in, in_ids, in_offsets, in_block_ids, in_flags, &pi);
      if (rc) {  // cannot happen after check_swap_in; if it does, the eviction's bookkeeping is already committed
        p->broken = true;
        return rc;
      }
      for (int32_t i = 0; i < n_out; i++) p->wq.erase(out_ids[i]);
      for (int32_t i = 0; i < n_in; i++) p->wq.erase(in_ids[i]);
      p->last_plan = pi.desc;  // as after the two calls made one after the other: the load's list
      const double t1 = now_us();
      if (!po.desc.empty() && !pi.desc.empty()) {
        const uint64_t dep_out = std::max(cross_stream(p, kEvict, po.wait_in_seq), pending_user(p, kEvict, po.fresh));
        const uint64_t dep_in = cross_stream(p, kLoad, pi.wait_out_seq);
        Call *co = nullptr, *ci = nullptr;
        rc = open_call(p, kEvict, 1, dep_out, wait_event, 0, po.desc, &co);
        if (rc) return rc;
        rc = open_call(p, kLoad, 3, dep_in, wait_event, 1, pi.desc, &ci, /*do_retire=*/false);
        if (rc) return rc;
        fill_plan_stats(p, &co->st, 1, po.desc.size(), t1 - t0);
        fill_plan_stats(p, &ci->st, 3, pi.desc.size(), t1 - t0);
        rc = enqueue_in_phase(p, *co, po, *ci, pi);
        if (rc) return rc;
        if ((rc = close_call(p, *co)) || (rc = close_call(p, *ci))) return rc;
        for (uint64_t id : po.touched)
          if (kvswap::Req* r = p->planner.find_mut(id)) r->out_seq = co->seq;
        for (uint64_t id : pi.touched)
          if (kvswap::Req* r = p->planner.find_mut(id)) r->in_seq = ci->seq;
        for (auto& f : pi.freed) p->pending.push_back({f.first, f.first + f.second, ci->seq});
        co->st.enqueue_us = ci->st.enqueue_us = now_us() - t1;
        return KV_OK;
      }
      // one side moves nothing: the plans are committed, enqueue them the ordinary way
      rc = swap_out_common(p, 1, po, t0, wait_event);
      if (rc) return rc;
      if (pi.desc.empty() && !wait_event) return KV_OK;
      const uint64_t dep_in = cross_stream(p, kLoad, pi.wait_out_seq);
      Call* c = nullptr;
      rc = open_call(p, kLoad, 3, dep_in, wait_event, 1, pi.desc, &c);
      if (rc) return rc;
      fill_plan_stats(p, &c->st, 3, pi.desc.size(), t1 - t0);
      if ((rc = enqueue_transfer(p, *c, pi, false)) || (rc = close_call(p, *c))) return rc;
      for (uint64_t id : pi.touched)
        if (kvswap::Req* r = p->planner.find_mut(id)) r->in_seq = c->seq;
      for (auto& f : pi.freed) p->pending.push_back({f.first, f.first + f.second, c->seq});
      return KV_OK;
    }
  }
  // plan-only handles, the copy-engine path, and calls with an empty side: the two calls one after the other
  int rc = kv_swap_out(p, n_out, out_ids, out_offsets, out_block_ids, out_tokens, wait_event);
  if (rc) return rc;
  return kv_swap_in(p, n_in, in_ids, in_offsets, in_block_ids, in_flags, wait_event);
}
KV_CATCH(p)

int kv_move_blocks(kv_pool* p, int64_t n, const int32_t* src_ids, const int32_t* dst_ids, void* wait_event) try {
  if (!p) return KV_EINVAL;
  KV_ENTER(p);
  const double t0 = now_us();
  Plan plan;
  int rc = p->planner.plan_move(n, src_ids, dst_ids, &plan);
  if (rc) return rc;
  p->last_plan = plan.desc;
  const double t1 = now_us();
  if (p->plan_only || (plan.desc.empty() && !wait_event)) {
    p->plan_stats = kv_stats{};
    fill_plan_stats(p, &p->plan_stats, 4, plan.desc.size(), t1 - t0);
    p->last_instant = true;
    return KV_OK;
  }
  Call* c = nullptr;
  rc = open_call(p, kEvict, 4, 0, wait_event, 2, plan.desc, &c);
  if (rc) return rc;
  fill_plan_stats(p, &c->st, 4, plan.desc.size(), t1 - t0);
  c->st.path = KV_PATH_ZEROCOPY;
  rc = enqueue_kernel(p, *c, 2, plan.desc.data(), plan.desc.size(), nullptr, 0, /*sole=*/true);
  if (rc) return rc;
  mark_blocks(p, *c, 2, plan.desc.data(), plan.desc.size(), -1);
  rc = close_call(p, *c);
  if (rc) return rc;
  c->st.enqueue_us = now_us() - t1;
  return KV_OK;
}
KV_CATCH(p)

// kv_move_blocks for callers that cannot allocate.  Uses only what kv_pool_create set up: no hipMalloc, hipFree,
// hipHostMalloc, event or stream creation, and no host heap either (the descriptors travel inside kernel
// arguments, duplicates are found with the handle's bitmap).  The kernel is the one kv_move_blocks launches; it
// reads its descriptors from the library's fixed device array instead of the growable ring.
int kv_move_blocks_noalloc(kv_pool* p, int64_t n, const int32_t* src_ids, const int32_t* dst_ids, void* wait_event) try {
  if (!p) return KV_EINVAL;
  KV_ENTER(p);
  const double t0 = now_us();
  if (n < 0) return KV_EINVAL;
  if (n > KV_NOALLOC_MAX_BLOCKS) return KV_E2BIG;
  if (n > 0 && (!src_ids || !dst_ids)) return KV_EINVAL;
  const int64_t N = p->cfg.num_blocks;
  for (int64_t i = 0; i < n; i++)
    if (src_ids[i] < 0 || src_ids[i] >= N || dst_ids[i] < 0 || dst_ids[i] >= N) return KV_ERANGE;
  if (p->na_mark.empty() && n > 0) p->na_mark.assign((size_t)((N + 63) / 64), 0);  // plan-only handles: first use
  // destinations must be distinct and must not be sources: sources set their bit (twice is fine), then every
  // destination must find its bit clear and sets it
  bool dup = false;
  uint64_t* mark = p->na_mark.data();
  for (int64_t i = 0; i < n; i++) mark[src_ids[i] >> 6] |= 1ull << (src_ids[i] & 63);
  for (int64_t i = 0; i < n; i++) {
    uint64_t& w = mark[dst_ids[i] >> 6];
    const uint64_t bit = 1ull << (dst_ids[i] & 63);
    if (w & bit) dup = true;
    w |= bit;
  }
  for (int64_t i = 0; i < n; i++) {  // all zero again for the next call
    mark[src_ids[i] >> 6] = 0;
    mark[dst_ids[i] >> 6] = 0;
  }
  if (dup) return KV_EDUP;
  p->plan_stats = kv_stats{};
  fill_plan_stats(p, &p->plan_stats, 4, (size_t)n, now_us() - t0);
  p->plan_stats.path = KV_PATH_ZEROCOPY;
  p->last_instant = true;  // no call record: kv_last_stats reports the plan figures
  if (p->plan_only || (n == 0 && !wait_event)) return KV_OK;

  hipStream_t st = p->stream[kEvict];
  // after everything the load stream has been given so far (it may still write blocks this move reads, or read
  // blocks it overwrites), and after the caller's event
  HIPCHK(p, hipEventRecord(p->na_fence_ev, p->stream[kLoad]));
  HIPCHK(p, hipStreamWaitEvent(st, p->na_fence_ev, 0));
  hipEvent_t callers = (hipEvent_t)wait_event;
  if (callers) HIPCHK(p, hipStreamWaitEvent(st, callers, 0));
  if (n > 0) {
    // The descriptors go into the fixed array in batches that travel as kernel arguments: nothing on the host has to
    // outlive this call, so it never waits for an earlier one.  The array keeps the previous call's descriptors:
    // [0, n) is overwritten here, in stream order behind the previous call's kernel, and nothing beyond n is read.
    (void)hipGetLastError();
    DescPack pack;
    for (int64_t at = 0; at < n; at += kDescPack) {
      const int m = (int)std::min<int64_t>(kDescPack, n - at);
      for (int i = 0; i < m; i++) pack.d[i] = {src_ids[at + i], dst_ids[at + i]};
      hipLaunchKernelGGL(kv_desc_fill_kernel, dim3(1), dim3(512), 0, st, p->na_dev, at, m, pack);
    }
    HIPCHK(p, hipGetLastError());
    MoveArgs a;
    int u = 1;
    const int grid = build_move_args(p, 2, (size_t)n, nullptr, 0, false, &a, &u);
    a.desc = p->na_dev;
    (void)hipGetLastError();
    launch_move<2>(u, grid, 0, st, a);
    HIPCHK(p, hipGetLastError());
    p->plan_stats.launches = 1;
    p->plan_stats.grid = grid;
  }
  HIPCHK(p, hipEventRecord(p->na_done_ev, st));
  p->na_pending = true;
  p->plan_stats.enqueue_us = now_us() - t0 - p->plan_stats.plan_us;
  return KV_OK;
}
KV_CATCH(p)

int kv_sync(kv_pool* p) try {
  if (!p) return KV_EINVAL;
  KV_ENTER(p);
  if (p->plan_only) return KV_OK;
  for (int s = 0; s < 2; s++) HIPCHK(p, hipStreamSynchronize(p->stream[s]));
  retire(p);
  return KV_OK;
}
KV_CATCH(p)

int kv_req_reserve(kv_pool* p, uint64_t req_id, int32_t max_blocks) try {
  if (!p) return KV_EINVAL;
  KV_ENTER(p);
  int rc = p->planner.reserve(req_id, max_blocks);
  if (rc || p->plan_only) return rc;
  // The extent may lie on slots that an unfinished swap-in of their previous owner still reads: whatever
  // this request writes there first has to wait for it, exactly as for an extent taken inside a swap-out.
  const auto run = p->planner.last_fresh();
  const uint64_t dep = pending_user(p, kEvict, {run});  // the extent's first use is a write on the evict stream
  if (dep)
    if (kvswap::Req* r = p->planner.find_mut(req_id)) r->in_seq = dep;
  return KV_OK;
}
KV_CATCH(p)

int kv_req_release(kv_pool* p, uint64_t req_id) try {
  if (!p) return KV_EINVAL;
  KV_ENTER(p);
  kvswap::Req was;
  int rc = p->planner.release(req_id, &was);
  if (!rc) p->wq.erase(req_id);
  if (rc || p->plan_only) return rc;
  // the slots may still be in use by unfinished work of either stream: later users wait for it
  for (uint64_t s : {was.in_seq, was.out_seq})
    if (s && was.cap && !seq_done(p, s)) p->pending.push_back({was.base, was.base + was.cap, s});
  return KV_OK;
}
KV_CATCH(p)

int kv_req_query(kv_pool* p, uint64_t req_id, int64_t* staging_offset, int32_t* cap_blocks, int32_t* blocks_staged,
                 int32_t* watermark, int32_t* swapped) try {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  const kvswap::Req* r = p->planner.find(req_id);
  if (!r) return KV_ENOENT;
  if (staging_offset) *staging_offset = r->base * p->S;
  if (cap_blocks) *cap_blocks = r->cap;
  if (blocks_staged) *blocks_staged = r->staged;
  if (watermark) *watermark = r->wm;
  if (swapped) *swapped = r->swapped ? 1 : 0;
  return KV_OK;
}
KV_CATCH(p)

int kv_last_stats(kv_pool* p, kv_stats* out) try {
  if (!p || !out) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  if (p->plan_only || p->last_instant || p->calls.empty()) {
    *out = p->plan_stats;
    out->struct_size = sizeof(kv_stats);
    return KV_OK;
  }
  Call& c = p->calls.back();
  if (c.end) {
    HIPCHK(p, hipEventSynchronize(c.end));
    float ms = 0.f;
    HIPCHK(p, hipEventElapsedTime(&ms, c.start, c.end));
    c.st.ms_total = ms;
    float ks = 0.f;
    for (auto& k : c.kev) {
      HIPCHK(p, hipEventElapsedTime(&ms, k.first, k.second));
      ks += ms;
    }
    // a call that is one launch and nothing else carries no kernel events: its own events bracket the kernel
    c.st.ms_kernel = c.kev.empty() && c.st.launches == 1 && c.st.copies == 0 ? c.st.ms_total : ks;
  }
  *out = c.st;
  return KV_OK;
}
KV_CATCH(p)

int64_t kv_slot_bytes(const kv_pool* p) { return p ? p->S : 0; }

// (call, event) that completes the request's last transfer; call == nullptr: nothing in flight
static hipEvent_t req_event(kv_pool* p, uint64_t req_id) {
  auto it = p->req_where.find(req_id);
  if (it == p->req_where.end()) return nullptr;
  Call* c = find_call(p, it->second.first);
  if (!c) return nullptr;
  const int sg = it->second.second;
  return sg >= 0 && sg < (int)c->seg_ev.size() ? c->seg_ev[(size_t)sg] : c->end;
}

int kv_req_poll(kv_pool* p, uint64_t req_id) try {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  if (p->plan_only) return 1;
  hipEvent_t ev = req_event(p, req_id);
  if (!ev) return 1;
  hipError_t e = hipEventQuery(ev);
  if (e == hipSuccess) return 1;
  (void)hipGetLastError();
  if (e == hipErrorNotReady) return 0;
  p->last_hip = (int)e;
  p->broken = true;
  return KV_EHIP;
}
KV_CATCH(p)

int kv_req_wait(kv_pool* p, uint64_t req_id) try {
  if (!p) return KV_EINVAL;
  hipEvent_t ev;
  {
    std::lock_guard<std::mutex> g(p->mu);
    if (p->plan_only) return KV_OK;
    ev = req_event(p, req_id);
  }
  if (!ev) return KV_OK;
  // The wait runs without the handle's lock: a thread that waits for one request does not hold up the thread
  // that enqueues the next calls.  An event returns to the free list only after its work has finished; should
  // another call record it again meanwhile, this wait ends later than it had to, never earlier than the
  // request's own transfer.
  const hipError_t e = hipEventSynchronize(ev);
  if (e != hipSuccess) {
    std::lock_guard<std::mutex> g(p->mu);
    p->last_hip = (int)e;
    p->broken = true;
    (void)hipGetLastError();
    return KV_EHIP;
  }
  return KV_OK;
}
KV_CATCH(p)

int64_t kv_last_timeline(kv_pool* p, uint64_t* req_ids, float* done_ms, int64_t cap) try {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  if (p->plan_only || p->last_instant || p->calls.empty()) return 0;
  Call& c = p->calls.back();
  if (!c.end) return 0;
  HIPCHK(p, hipEventSynchronize(c.end));
  const int64_t n = (int64_t)c.req_seg.size();
  for (int64_t i = 0; i < n && i < cap; i++) {
    const int sg = c.req_seg[(size_t)i].second;
    hipEvent_t ev = sg >= 0 && sg < (int)c.seg_ev.size() ? c.seg_ev[(size_t)sg] : c.end;
    float ms = 0.f;
    HIPCHK(p, hipEventElapsedTime(&ms, c.start, ev));
    if (req_ids) req_ids[i] = c.req_seg[(size_t)i].first;
    if (done_ms) done_ms[i] = ms;
  }
  return n;
}
KV_CATCH(p)

static void io_snapshot(kv_pool* p, kv_io_stats* o) {
  std::memset(o, 0, sizeof(*o));
  o->struct_size = sizeof(kv_io_stats);
  if (!p->plan_only) {
    retire(p);
    for (auto& c : p->calls) {
      if (!c.end || c.st.op == 4) continue;
      if (hipEventQuery(c.end) == hipSuccess) {
        account(p, c);  // the newest call stays in the queue for kv_last_stats even when finished
        continue;
      }
      (void)hipGetLastError();
      o->inflight_calls[c.stream]++;
      o->inflight_bytes[c.stream] += c.st.bytes;
    }
  }
  for (int s = 0; s < 2; s++) {
    o->total_calls[s] = p->tot_calls[s];
    o->total_bytes[s] = p->tot_bytes[s];
    o->ewma_gbps[s] = p->ewma_gbps[s];
    o->ewma_small_us[s] = p->ewma_small_us[s];
  }
}

int kv_io_stats_get(kv_pool* p, kv_io_stats* out) try {
  if (!p || !out) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  io_snapshot(p, out);
  return KV_OK;
}
KV_CATCH(p)

static int64_t budget_blocks_locked(kv_pool* p, int32_t dir, double interval_us);

int64_t kv_budget_blocks(kv_pool* p, int32_t dir, double interval_us) try {
  if (!p || (dir != 0 && dir != 1) || !(interval_us >= 0)) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  return budget_blocks_locked(p, dir, interval_us);
}
KV_CATCH(p)

int kv_swap_out_delta_timed(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                            const int32_t* block_ids, const int32_t* num_tokens, const float* priority,
                            double interval_us, uint32_t flags, int32_t* blocks_moved, int64_t* budget_used,
                            void* wait_event) try {
  if (!p || !(interval_us >= 0)) return KV_EINVAL;
  if (n < 0 || (n > 0 && (!req_ids || !offsets || !num_tokens))) return KV_EINVAL;
  KV_ENTER(p);
  const double t0 = now_us();
  const int64_t budget = budget_blocks_locked(p, 0, interval_us);
  if (budget_used) *budget_used = budget;
  // priority order, stable
  std::vector<int32_t> order((size_t)n);
  for (int32_t i = 0; i < n; i++) order[(size_t)i] = i;
  if (priority)
    std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return priority[a] > priority[b]; });
  for (int32_t i = 0; i < n; i++)
    if (offsets[i + 1] < offsets[i] || offsets[0] < 0) return KV_EINVAL;
  std::vector<uint64_t> ids((size_t)n);
  std::vector<int32_t> off((size_t)n + 1, 0), tok((size_t)n), blk, moved((size_t)n, 0);
  for (int32_t k = 0; k < n; k++) {
    const int32_t i = order[(size_t)k];
    ids[(size_t)k] = req_ids[i];
    tok[(size_t)k] = num_tokens[i];
    const int32_t len = offsets[i + 1] - offsets[i];
    if (len > 0 && !block_ids) return KV_EINVAL;
    blk.insert(blk.end(), block_ids + offsets[i], block_ids + offsets[i] + len);
    off[(size_t)k + 1] = off[(size_t)k] + len;
  }
  Plan plan;
  int rc = p->planner.plan_delta(n, ids.data(), off.data(), blk.data(), tok.data(), budget, flags, moved.data(), &plan,
                                 /*limited_even_if_zero=*/true);
  if (rc) return rc;
  if (blocks_moved)
    for (int32_t k = 0; k < n; k++) blocks_moved[order[(size_t)k]] = moved[(size_t)k];
  return swap_out_common(p, 2, plan, t0, wait_event);
}
KV_CATCH(p)

int kv_wq_post(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets, const int32_t* block_ids,
               const int32_t* num_tokens, const double* priority) try {
  if (!p || n < 0 || (n > 0 && (!req_ids || !offsets || !num_tokens))) return KV_EINVAL;
  KV_ENTER(p);
  const int64_t B = p->cfg.block_size, N = p->cfg.num_blocks;
  if (n > 0 && offsets[0] < 0) return KV_EINVAL;
  for (int32_t i = 0; i < n; i++) {
    const int64_t row = (int64_t)offsets[i + 1] - offsets[i], len = num_tokens[i];
    if (row < 0 || len < 0 || row < (len + B - 1) / B) return KV_EINVAL;
    if (row > 0 && !block_ids) return KV_EINVAL;
    if (priority && !(priority[i] == priority[i])) return KV_EINVAL;  // NaN has no place in an order
    for (int32_t j = 0; j < i; j++)
      if (req_ids[j] == req_ids[i]) return KV_EINVAL;
    for (int64_t j = offsets[i]; j < offsets[i + 1]; j++)
      if (block_ids[j] < 0 || block_ids[j] >= N) return KV_ERANGE;
    const kvswap::Req* r = p->planner.find(req_ids[i]);
    if (r && r->swapped) return KV_EEXIST;
    if (r && len < (int64_t)r->wm * B) return KV_ESTATE;
  }
  for (int32_t i = 0; i < n; i++) {
    kv_pool::WqEntry& e = p->wq[req_ids[i]];
    e.blocks.assign(block_ids + offsets[i], block_ids + offsets[i + 1]);
    e.tokens = num_tokens[i];
    e.priority = priority ? priority[i] : 0.0;
    e.order = ++p->wq_order;
  }
  return KV_OK;
}
KV_CATCH(p)

int kv_wq_remove(kv_pool* p, uint64_t req_id) try {
  if (!p) return KV_EINVAL;
  KV_ENTER(p);
  return p->wq.erase(req_id) ? KV_OK : KV_ENOENT;
}
KV_CATCH(p)

// Full blocks the queued requests have not written through yet.
static void wq_count(kv_pool* p, int64_t* blocks, int32_t* requests) {
  int64_t nb = 0;
  int32_t nr = 0;
  for (auto& kvp : p->wq) {
    const kvswap::Req* r = p->planner.find(kvp.first);
    const int64_t d = kvp.second.tokens / p->cfg.block_size - (r ? r->wm : 0);
    if (d > 0) {
      nb += d;
      nr++;
    }
  }
  if (blocks) *blocks = nb;
  if (requests) *requests = nr;
}

int kv_wq_pending(kv_pool* p, int64_t* blocks, int32_t* requests) try {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  wq_count(p, blocks, requests);
  return KV_OK;
}
KV_CATCH(p)

int kv_wq_drain(kv_pool* p, double interval_us, int64_t block_budget, uint32_t flags, int64_t* blocks_written,
                int64_t* blocks_pending, int64_t* budget_used, void* wait_event) try {
  if (!p || !(interval_us >= 0) || block_budget < 0) return KV_EINVAL;
  KV_ENTER(p);
  const double t0 = now_us();
  const bool timed = block_budget == 0 && interval_us > 0;
  const int64_t budget = timed ? budget_blocks_locked(p, 0, interval_us) : block_budget;
  if (budget_used) *budget_used = budget;
  std::vector<std::pair<uint64_t, const kv_pool::WqEntry*>> order;
  order.reserve(p->wq.size());
  for (auto& kvp : p->wq) {
    // An entry posted before a direct delta went past it has nothing left to write: it is skipped, not an error.
    const kvswap::Req* r = p->planner.find(kvp.first);
    if (r && kvp.second.tokens < (int64_t)r->wm * p->cfg.block_size) continue;
    order.push_back({kvp.first, &kvp.second});
  }
  std::sort(order.begin(), order.end(), [](const auto& a, const auto& b) {
    if (a.second->priority != b.second->priority) return a.second->priority > b.second->priority;
    return a.second->order < b.second->order;
  });
  const int32_t n = (int32_t)order.size();
  std::vector<uint64_t> ids((size_t)n);
  std::vector<int32_t> off((size_t)n + 1, 0), tok((size_t)n), blk, moved((size_t)n, 0);
  for (int32_t k = 0; k < n; k++) {
    const kv_pool::WqEntry& e = *order[(size_t)k].second;
    ids[(size_t)k] = order[(size_t)k].first;
    tok[(size_t)k] = e.tokens;
    blk.insert(blk.end(), e.blocks.begin(), e.blocks.end());
    off[(size_t)k + 1] = (int32_t)blk.size();
  }
  Plan plan;
  int rc = p->planner.plan_delta(n, ids.data(), off.data(), blk.data(), tok.data(), budget, flags, moved.data(), &plan,
                                 /*limited_even_if_zero=*/timed);
  if (rc) return rc;
  int64_t total = 0;
  for (int32_t k = 0; k < n; k++) total += moved[(size_t)k];
  if (blocks_written) *blocks_written = total;
  wq_count(p, blocks_pending, nullptr);
  return swap_out_common(p, 2, plan, t0, wait_event);
}
KV_CATCH(p)

static int64_t budget_blocks_locked(kv_pool* p, int32_t dir, double interval_us) {
  kv_io_stats io;
  io_snapshot(p, &io);
  const double rate = io.ewma_gbps[dir] > 0 ? io.ewma_gbps[dir] : 32.0;           // GB/s = bytes per ns
  const double fixed = io.ewma_small_us[dir] > 0 ? io.ewma_small_us[dir] : 50.0;  // us
  const double queued_us = (double)io.inflight_bytes[dir] / (rate * 1e3);
  const double left_us = interval_us - fixed - queued_us;
  if (left_us <= 0) return 0;
  return (int64_t)(left_us * rate * 1e3 / (double)p->S);
}

int64_t kv_last_plan(kv_pool* p, int32_t* phys, int64_t* slot, int64_t cap) try {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  const int64_t n = (int64_t)p->last_plan.size();
  for (int64_t i = 0; i < n && i < cap; i++) {
    if (phys) phys[i] = p->last_plan[(size_t)i].a;
    if (slot) slot[i] = (int64_t)(uint32_t)p->last_plan[(size_t)i].b;
  }
  return n;
}
KV_CATCH(p)

int kv_pool_tune(kv_pool* p, int32_t what, int64_t value) try {
  if (!p || value < 0) return KV_EINVAL;
  KV_ENTER(p);
  switch (what) {
    case KV_TUNE_MAX_WGS_DEVICE:
      p->max_wgs_device = std::min<int64_t>(value, 1 << 30);
      return KV_OK;
    case KV_TUNE_MAX_WGS_LINK:
      p->max_wgs_link = std::min<int64_t>(value, 1 << 30);
      return KV_OK;
    case KV_TUNE_KERNEL_VARIANT:
      if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8 && value != 101 && value != 102 && value != 104)
        return KV_EINVAL;
      p->variant = value;
      return KV_OK;
    case KV_TUNE_DMA_SLICE_BLOCKS:
      p->dma_slice = value;
      return KV_OK;
    case KV_TUNE_SCALE_LDS:
      if (value > 2) return KV_EINVAL;
      p->scale_lds_knob = value;
      return KV_OK;
    case KV_TUNE_SEGMENT_BYTES:
      p->segment_bytes = value ? value : 32ll << 20;
      return KV_OK;
    case KV_TUNE_SEGMENT_MAX_BYTES:
      p->segment_max_bytes = value;
      return KV_OK;
    case KV_TUNE_LINK_IN_WGS:
      p->link_in_wgs = std::min<int64_t>(value, 1 << 30);
      return KV_OK;
    case KV_TUNE_LINK_IN_UNROLL:
      if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return KV_EINVAL;
      p->link_in_unroll = value;
      return KV_OK;
    case KV_TUNE_HOST_STORES:
      if (value > 1) return KV_EINVAL;
      p->host_stores_nt = value;
      return KV_OK;
    case KV_TUNE_KERNEL_EVENTS:
      p->kernel_events = value ? 1 : 0;
      return KV_OK;
    case KV_TUNE_PHASE_BYTES:
      p->phase_bytes = value ? value : 256ll << 20;
      return KV_OK;
    case KV_TUNE_PHASE_WGS_OUT:
      p->phase_wgs_out = value;
      return KV_OK;
    case KV_TUNE_PHASE_WGS_IN:
      p->phase_wgs_in = value;
      return KV_OK;
    case KV_TUNE_SCATTER_ORDER:
      if (value > 2) return KV_EINVAL;
      p->scatter_order = value;
      return KV_OK;
    default:
      return KV_EINVAL;
  }
}
KV_CATCH(p)

int kv_last_hip_error(const kv_pool* p) { return p ? p->last_hip.load() : 0; }

const char* kv_strerror(int code) {
  switch (code) {
    case KV_OK: return "ok";
    case KV_EINVAL: return "invalid argument";
    case KV_ERANGE: return "block id out of range";
    case KV_EDUP: return "duplicate destination block";
    case KV_ENOENT: return "unknown request";
    case KV_EEXIST: return "request already swapped out or already known";
    case KV_ENOSPC: return "staging arena full";
    case KV_EHIP: return "HIP runtime error";
    case KV_ESTATE: return "token count below the watermark";
    case KV_ENOMEM: return "out of host memory for the library's bookkeeping";
    case KV_E2BIG: return "more blocks than the fixed descriptor array of the allocation-free entry point holds";
    default: return "unknown status";
  }
}

// ---- measurement helpers: ceilings the swap is compared against ----

// Contiguous device-to-device copy of `bytes` (multiple of 16 KiB) with the lane shape of the gather.
// grid == 0: one workgroup per 4 KiB piece, one 16-byte load per lane, the launch shape of the on-device
// gather/scatter and the fastest plain copy measured on MI355X; grid > 0: at most that many workgroups,
// four loads per lane, grid-stride.  Runs `iters` times on `stream`; returns the mean milliseconds per
// copy, or < 0.
double kv_bench_copy(void* dst_dev, const void* src_dev, int64_t bytes, int32_t grid, int32_t iters, void* stream) {
  if (!dst_dev || !src_dev || bytes <= 0 || bytes % 16384 || grid < 0 || iters <= 0) return -1.0;
  if (!range_ok(dst_dev, bytes, true) || !range_ok(src_dev, bytes, true)) return -1.0;
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return -2.0;
  constexpr int64_t kMaxGrid = ((int64_t)1 << 32) / 256 - 1;
  auto once = [&]() {
    if (grid == 0) {
      const int64_t pieces = bytes / 4096;
      hipLaunchKernelGGL((kv_copy_kernel<1>), dim3((unsigned)std::min(pieces, kMaxGrid)), dim3(256), 0, st,
                         (const char*)src_dev, (char*)dst_dev, pieces);
    } else {
      const int64_t pieces = bytes / 16384;
      hipLaunchKernelGGL((kv_copy_kernel<4>), dim3((unsigned)std::min<int64_t>(pieces, grid)), dim3(256), 0, st,
                         (const char*)src_dev, (char*)dst_dev, pieces);
    }
  };
  once();
  (void)hipEventRecord(a, st);
  for (int i = 0; i < iters; i++) once();
  (void)hipEventRecord(b, st);
  float ms = -1.f;
  if (hipEventSynchronize(b) != hipSuccess || hipEventElapsedTime(&ms, a, b) != hipSuccess) ms = -3.f * iters;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return (double)ms / iters;
}

// The same copy with one side visited in runs of run_bytes in a scrambled order (a fixed bijection on the run
// index): what a gather from (which 0: source scrambled) or a scatter into (which 1: destination scrambled) a
// paged pool looks like to the memory system, with the lane shape and the launch shape of the on-device kernels
// and nothing else in the way.  run_bytes is a power of two from 16 bytes up, bytes / run_bytes a power of two,
// bytes a multiple of 4 KiB.  Returns the mean milliseconds per copy, or < 0.
double kv_bench_copy_scrambled(void* dst_dev, const void* src_dev, int64_t bytes, int64_t run_bytes, int32_t which,
                               int32_t iters, void* stream) {
  if (!dst_dev || !src_dev || bytes <= 0 || bytes % 4096 || run_bytes < 16 || iters <= 0 || (which != 0 && which != 1)) return -1.0;
  const int64_t runs = bytes / run_bytes;
  if ((run_bytes & (run_bytes - 1)) || runs * run_bytes != bytes || runs < 1 || (runs & (runs - 1))) return -1.0;
  if (!range_ok(dst_dev, bytes, true) || !range_ok(src_dev, bytes, true)) return -1.0;
  int shift = 0;
  while ((16ll << shift) < run_bytes) shift++;
  const int64_t chunks = runs;
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return -2.0;
  constexpr int64_t kMaxGrid = ((int64_t)1 << 32) / 256 - 1;
  const int64_t pieces = bytes / 4096;
  auto once = [&]() {
    hipLaunchKernelGGL(kv_copy_scrambled_kernel, dim3((unsigned)std::min(pieces, kMaxGrid)), dim3(256), 0, st,
                       (const char*)src_dev, (char*)dst_dev, pieces, shift, chunks - 1, (int)which);
  };
  once();
  (void)hipEventRecord(a, st);
  for (int i = 0; i < iters; i++) once();
  (void)hipEventRecord(b, st);
  float ms = -1.f;
  if (hipEventSynchronize(b) != hipSuccess || hipEventElapsedTime(&ms, a, b) != hipSuccess) ms = -3.f * iters;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return (double)ms / iters;
}

// One contiguous hipMemcpyAsync between pinned host and device memory, timed with events:
// the host-link ceiling.  dir 0: device -> host, 1: host -> device.  Returns mean ms per copy.
double kv_bench_link(void* host_pinned, void* dev, int64_t bytes, int32_t dir, int32_t iters, void* stream) {
  if (!host_pinned || !dev || bytes <= 0 || iters <= 0 || (dir != 0 && dir != 1)) return -1.0;
  if (!range_ok(dev, bytes) || !range_ok(host_pinned, bytes)) return -1.0;
  hipStream_t st = (hipStream_t)stream;
  hipEvent_t a, b;
  if (hipEventCreate(&a) != hipSuccess || hipEventCreate(&b) != hipSuccess) return -2.0;
  auto once = [&]() {
    return dir == 0 ? hipMemcpyAsync(host_pinned, dev, (size_t)bytes, hipMemcpyDeviceToHost, st)
                    : hipMemcpyAsync(dev, host_pinned, (size_t)bytes, hipMemcpyHostToDevice, st);
  };
  (void)once();
  (void)hipEventRecord(a, st);
  for (int i = 0; i < iters; i++) (void)once();
  (void)hipEventRecord(b, st);
  float ms = -1.f;
  if (hipEventSynchronize(b) != hipSuccess || hipEventElapsedTime(&ms, a, b) != hipSuccess) ms = -3.f * iters;
  (void)hipEventDestroy(a);
  (void)hipEventDestroy(b);
  return (double)ms / iters;
}

// Both directions at once: `iters` copies device -> host (dev_a -> host_a) on one stream while as many
// run host -> device (host_b -> dev_b) on another; the four buffers must not overlap.  Returns the mean
// milliseconds until BOTH of a pair have finished (host clock around the whole batch), or < 0.
double kv_bench_link_bidir(void* host_a, const void* dev_a, const void* host_b, void* dev_b, int64_t bytes,
                           int32_t iters) {
  if (!host_a || !dev_a || !host_b || !dev_b || bytes <= 0 || iters <= 0) return -1.0;
  if (!range_ok(dev_a, bytes) || !range_ok(dev_b, bytes) || !range_ok(host_a, bytes) || !range_ok(host_b, bytes))
    return -1.0;
  hipStream_t up = nullptr, down = nullptr;
  if (hipStreamCreateWithFlags(&down, hipStreamNonBlocking) != hipSuccess) return -2.0;
  if (hipStreamCreateWithFlags(&up, hipStreamNonBlocking) != hipSuccess) {
    (void)hipStreamDestroy(down);
    return -2.0;
  }
  auto pair = [&]() {
    (void)hipMemcpyAsync(host_a, dev_a, (size_t)bytes, hipMemcpyDeviceToHost, down);
    (void)hipMemcpyAsync(dev_b, host_b, (size_t)bytes, hipMemcpyHostToDevice, up);
  };
  pair();  // warm-up
  double ms = -3.0;
  if (hipStreamSynchronize(down) == hipSuccess && hipStreamSynchronize(up) == hipSuccess) {
    const auto t0 = std::chrono::steady_clock::now();
    for (int i = 0; i < iters; i++) pair();
    const bool ok = hipStreamSynchronize(down) == hipSuccess && hipStreamSynchronize(up) == hipSuccess;
    const auto t1 = std::chrono::steady_clock::now();
    if (ok) ms = std::chrono::duration<double, std::milli>(t1 - t0).count() / iters;
  }
  (void)hipStreamDestroy(down);
  (void)hipStreamDestroy(up);
  return ms;
}

}  // extern "C"
