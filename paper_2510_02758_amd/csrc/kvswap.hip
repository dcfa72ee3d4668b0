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
#include <hip/hip_runtime.h>

#include <chrono>
#include <climits>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <unordered_map>
#include <vector>

#include "planner.hpp"

#include "kernels.hip.inc"

using kvswap::Desc;
using kvswap::Plan;

namespace {

constexpr int kEvict = 0, kLoad = 1;

struct Call {
  uint64_t seq = 0;
  int stream = kEvict;
  hipEvent_t start = nullptr, end = nullptr;
  std::vector<std::pair<hipEvent_t, hipEvent_t>> kev;
  std::vector<hipEvent_t> seg_ev;                  // one per segment under KV_REQ_EVENTS
  std::vector<std::pair<uint64_t, int>> req_seg;   // (request id, segment that completes it; -1: the whole call)
  kv_stats st{};
  bool accounted = false;  // already folded into the telemetry
};

struct RingSeg {
  size_t begin, end;
  uint64_t seq;
};

// Last in-flight reader / writer of a device block: low 32 bits of the call's sequence number
// (0: none) and the segment of that call that touches the block (-1: the call as a whole).
struct BlkMark {
  uint32_t seq;
  int32_t seg;
};

struct PendingRelease {
  int64_t lo, hi;
  uint64_t seq;  // load-stream call that still reads these slots
};

// KVSWAP_DEBUG=1 in the environment makes rejected configurations say why on stderr.
bool debug_on() {
  static const bool on = [] {
    const char* e = std::getenv("KVSWAP_DEBUG");
    return e && *e && *e != '0';
  }();
  return on;
}
#define KVDBG(...)                                   \
  do {                                               \
    if (debug_on()) {                                \
      std::fprintf(stderr, "[kvswap] " __VA_ARGS__); \
      std::fputc('\n', stderr);                      \
    }                                                \
  } while (0)

double now_us() {
  using namespace std::chrono;
  return duration<double, std::micro>(steady_clock::now().time_since_epoch()).count();
}

}  // namespace

struct kv_pool {
  kv_pool_config cfg{};
  int64_t chunk = 0, block_bytes = 0, scale_chunk = 0, block_scale_bytes = 0, S = 0, slots = 0;
  bool plan_only = false, dev_staging = false;
  char* arena_dev = nullptr;  // the arena as the kernels address it
  kvswap::Planner planner;
  std::mutex mu;

  hipStream_t stream[2] = {nullptr, nullptr};
  bool own_stream[2] = {false, false};

  Desc* ring_host = nullptr;
  Desc* ring_dev = nullptr;
  size_t ring_cap = 0, ring_head = 0;
  std::deque<RingSeg> ring_inflight;

  std::vector<hipEvent_t> ev_free;
  std::deque<Call> calls;  // oldest first; the newest is kept for kv_last_stats
  uint64_t seq = 0;
  std::vector<PendingRelease> pending;
  std::vector<BlkMark> blk_reader, blk_writer;  // per device block, see block_hazard()
  std::unordered_map<uint64_t, std::pair<uint64_t, int>> req_where;  // request -> (call seq, segment) of its last transfer
  bool req_events = false;
  int64_t segment_bytes = 32ll << 20;
  int64_t segment_max_bytes = 0;  // > 0: a segment is also cut inside a request once it reaches this size

  // write queue (kv_wq_*): the running requests' latest tables, drained in priority order
  struct WqEntry {
    std::vector<int32_t> blocks;
    int32_t tokens = 0;
    double priority = 0;
    uint64_t order = 0;  // position in the most recent post: ties keep post order
  };
  std::unordered_map<uint64_t, WqEntry> wq;
  uint64_t wq_order = 0;
  std::vector<Desc> last_plan;
  kv_stats plan_stats{};  // figures of a call that enqueued nothing
  bool last_instant = false;
  int last_hip = 0;

  // telemetry, updated when finished calls are retired
  int64_t tot_calls[2] = {0, 0}, tot_bytes[2] = {0, 0};
  double ewma_gbps[2] = {0, 0}, ewma_small_us[2] = {0, 0};

  int64_t max_wgs_device = 0, max_wgs_link = 0, variant = 0, dma_slice = 0, scale_lds_knob = 0;
  int cu_count = 256;
};

#define HIPCHK(p, expr)                         \
  do {                                          \
    hipError_t e_ = (expr);                     \
    if (e_ != hipSuccess) {                     \
      (p)->last_hip = (int)e_;                  \
      return KV_EHIP;                           \
    }                                           \
  } while (0)

namespace {

int elem_bytes(int dtype) {
  switch (dtype) {
    case KV_F16:
    case KV_BF16:
      return 2;
    case KV_FP8_E4M3:
      return 1;
    default:
      return 0;
  }
}

// true unless HIP knows the allocation and [ptr, ptr+need) leaves it
bool range_ok(const void* ptr, int64_t need) {
  hipDeviceptr_t base = nullptr;
  size_t size = 0;
  if (hipMemGetAddressRange(&base, &size, (hipDeviceptr_t)ptr) != hipSuccess) {
    (void)hipGetLastError();
    return true;
  }
  return (const char*)ptr + need <= (const char*)base + size;
}

int get_event(kv_pool* p, hipEvent_t* out) {
  if (!p->ev_free.empty()) {
    *out = p->ev_free.back();
    p->ev_free.pop_back();
    return KV_OK;
  }
  HIPCHK(p, hipEventCreate(out));
  return KV_OK;
}

void recycle(kv_pool* p, Call& c) {
  if (c.start) p->ev_free.push_back(c.start);
  if (c.end) p->ev_free.push_back(c.end);
  for (auto& k : c.kev) {
    p->ev_free.push_back(k.first);
    p->ev_free.push_back(k.second);
  }
  c.kev.clear();
  for (auto e : c.seg_ev) p->ev_free.push_back(e);
  c.seg_ev.clear();
  for (auto& rs : c.req_seg) {
    auto it = p->req_where.find(rs.first);
    if (it != p->req_where.end() && it->second.first == c.seq) p->req_where.erase(it);
  }
  c.req_seg.clear();
  c.start = c.end = nullptr;
}

Call* find_call(kv_pool* p, uint64_t seq) {
  for (auto& c : p->calls)
    if (c.seq == seq) return &c;
  return nullptr;
}

// Is the call with this sequence number finished?  Retired calls are.
bool seq_done(kv_pool* p, uint64_t seq) {
  if (seq == 0) return true;
  Call* c = find_call(p, seq);
  if (!c || !c->end) return true;
  hipError_t e = hipEventQuery(c->end);
  if (e == hipSuccess) return true;
  (void)hipGetLastError();
  return false;
}

constexpr int64_t kSmallCallBytes = 4ll << 20;
constexpr double kEwmaWeight = 0.25;

// A finished call leaves the queue: fold its stream time into the running estimates.
void account(kv_pool* p, Call& c) {
  if (c.accounted || !c.start || !c.end || c.st.op == 4) return;
  c.accounted = true;
  float ms = 0.f;
  if (hipEventElapsedTime(&ms, c.start, c.end) != hipSuccess || ms <= 0.f) {
    (void)hipGetLastError();
    return;
  }
  const int s = c.stream;
  p->tot_calls[s]++;
  p->tot_bytes[s] += c.st.bytes;
  if (c.st.bytes >= kSmallCallBytes) {
    const double gbps = (double)c.st.bytes / ((double)ms * 1e6);
    p->ewma_gbps[s] = p->ewma_gbps[s] > 0 ? (1 - kEwmaWeight) * p->ewma_gbps[s] + kEwmaWeight * gbps : gbps;
  } else if (c.st.bytes > 0) {
    const double us = (double)ms * 1e3;
    p->ewma_small_us[s] = p->ewma_small_us[s] > 0 ? (1 - kEwmaWeight) * p->ewma_small_us[s] + kEwmaWeight * us : us;
  }
}

// Drop finished calls from the front, always keeping the newest for the statistics.
void retire(kv_pool* p) {
  while (p->calls.size() > 1) {
    Call& c = p->calls.front();
    if (c.end && hipEventQuery(c.end) != hipSuccess) {
      (void)hipGetLastError();
      break;
    }
    account(p, c);
    recycle(p, c);
    p->calls.pop_front();
  }
  while (!p->ring_inflight.empty() && !find_call(p, p->ring_inflight.front().seq)) p->ring_inflight.pop_front();
  size_t w = 0;
  for (size_t i = 0; i < p->pending.size(); i++)
    if (find_call(p, p->pending[i].seq)) p->pending[w++] = p->pending[i];
  p->pending.resize(w);
}

int wait_seq_on_host(kv_pool* p, uint64_t seq) {
  Call* c = find_call(p, seq);
  if (c && c->end) HIPCHK(p, hipEventSynchronize(c->end));
  return KV_OK;
}

int grow_ring(kv_pool* p, size_t need) {
  for (int s = 0; s < 2; s++) HIPCHK(p, hipStreamSynchronize(p->stream[s]));
  p->ring_inflight.clear();
  if (p->ring_host) HIPCHK(p, hipHostFree(p->ring_host));
  if (p->ring_dev) HIPCHK(p, hipFree(p->ring_dev));
  p->ring_host = nullptr;
  p->ring_dev = nullptr;
  size_t cap = p->ring_cap ? p->ring_cap : (size_t)1 << 16;
  while (cap < need) cap *= 2;
  HIPCHK(p, hipHostMalloc((void**)&p->ring_host, cap * sizeof(Desc), hipHostMallocDefault));
  HIPCHK(p, hipMalloc((void**)&p->ring_dev, cap * sizeof(Desc)));
  p->ring_cap = cap;
  p->ring_head = 0;
  return KV_OK;
}

// Reserve n consecutive descriptors in both rings; waits (on the host) for earlier work whose
// descriptors still occupy that part: other calls through their end event, earlier launches of
// this same call (a call cut into more slices than the ring holds) through its stream.
int ring_reserve(kv_pool* p, size_t n, uint64_t seq, hipStream_t st, size_t* at) {
  if (n > p->ring_cap / 2) {
    int rc = grow_ring(p, n * 4);
    if (rc) return rc;
  }
  if (p->ring_head + n > p->ring_cap) p->ring_head = 0;
  const size_t b = p->ring_head, e = b + n;
  bool own_synced = false;
  for (auto& s : p->ring_inflight) {
    if (!(s.begin < e && b < s.end)) continue;
    if (s.seq != seq) {
      int rc = wait_seq_on_host(p, s.seq);
      if (rc) return rc;
    } else {
      if (!own_synced) HIPCHK(p, hipStreamSynchronize(st));
      own_synced = true;
      s.begin = s.end = 0;  // consumed: its kernel and its descriptor upload have run
    }
  }
  p->ring_inflight.push_back({b, e, seq});
  p->ring_head = e;
  *at = b;
  return KV_OK;
}

template <int MODE, int KIND, bool LEAN>
void launch_move_u(int u, int grid, hipStream_t st, const MoveArgs& a) {
  const size_t lds = a.scale_lds ? (size_t)a.scale_words * 4 : 0;
  switch (u) {
    case 1:
      hipLaunchKernelGGL((kv_move_kernel<MODE, 1, KIND, LEAN>), dim3(grid), dim3(256), lds, st, a);
      break;
    case 2:
      hipLaunchKernelGGL((kv_move_kernel<MODE, 2, KIND, LEAN>), dim3(grid), dim3(256), lds, st, a);
      break;
    case 8:
      hipLaunchKernelGGL((kv_move_kernel<MODE, 8, KIND, LEAN>), dim3(grid), dim3(256), lds, st, a);
      break;
    default:
      hipLaunchKernelGGL((kv_move_kernel<MODE, 4, KIND, LEAN>), dim3(grid), dim3(256), lds, st, a);
      break;
  }
}

// kind: 0 HBM arena, 1 host arena (link-bound), 2 bounce buffer.  The lean build of the kernel serves
// every launch that has neither small chunks nor scales.
template <int MODE>
void launch_move(int u, int grid, int kind, hipStream_t st, const MoveArgs& a) {
  const bool lean = !a.cpj && !a.scale_words;
  if (MODE == 2) {
    lean ? launch_move_u<MODE, 0, true>(u, grid, st, a) : launch_move_u<MODE, 0, false>(u, grid, st, a);
  } else if (kind == 1) {
    lean ? launch_move_u<MODE, 1, true>(u, grid, st, a) : launch_move_u<MODE, 1, false>(u, grid, st, a);
  } else if (kind == 2) {
    lean ? launch_move_u<MODE, 2, true>(u, grid, st, a) : launch_move_u<MODE, 2, false>(u, grid, st, a);
  } else {
    lean ? launch_move_u<MODE, 0, true>(u, grid, st, a) : launch_move_u<MODE, 0, false>(u, grid, st, a);
  }
}

// Loads in flight per lane.  Both ends in HBM: one 16-byte load per lane and one workgroup per
// 4 KiB piece measured fastest on MI355X (the hardware dispatcher keeps every CU fed and the
// job order stays the address order of the contiguous side).  Host link: fewer, fatter
// workgroups, since the link and not the CUs is the limit.
int pick_unroll(const kv_pool* p, bool link) {
  if (p->variant == 1 || p->variant == 2 || p->variant == 4 || p->variant == 8) return (int)p->variant;
  if (!link) return 1;
  if (p->chunk < 4096) return 4;  // groups of small chunks: four 4 KiB groups per workgroup pass
  if (p->chunk >= 16384) return 4;
  if (p->chunk >= 8192) return 2;
  return 1;
}

// Very short descriptor lists (a preemption after write-through moves one tail block per victim)
// travel inside the kernel arguments: no upload in front of the kernel, no ring space.
constexpr size_t kInlineDescMax = sizeof(MoveArgs::inl) / sizeof(Desc);

// Hand n descriptors to the device and launch one data kernel over them on stream `st`.
// mode 0 gather, 1 scatter, 2 move.  `contig` is the contiguous side.  `sole`: this is the only
// launch of its call, so the call's own start and end events already bracket it and the pair of
// kernel events (a marker packet each) is left out.
int enqueue_kernel(kv_pool* p, Call& call, int mode, const Desc* desc, size_t n, char* contig, int kind,
                   bool sole = false) {
  if (n == 0) return KV_OK;
  const bool link = kind == 1;
  hipStream_t st = p->stream[call.stream];
  size_t at = 0;
  int rc = KV_OK;
  const bool inline_desc = n <= kInlineDescMax;
  if (!inline_desc) {
    rc = ring_reserve(p, n, call.seq, st, &at);
    if (rc) return rc;
    std::memcpy(p->ring_host + at, desc, n * sizeof(Desc));
    HIPCHK(p, hipMemcpyAsync(p->ring_dev + at, p->ring_host + at, n * sizeof(Desc), hipMemcpyHostToDevice, st));
  }

  const int u = pick_unroll(p, link);
  const int64_t piece = 256 * 16 * (int64_t)u;
  MoveArgs a;
  a.pool = (char*)p->cfg.pool_dev;
  a.ls = p->cfg.layer_stride;
  a.ks = p->cfg.kv_stride;
  a.bs = p->cfg.block_stride;
  a.scale = (char*)p->cfg.scale_dev;
  a.sls = p->cfg.scale_layer_stride;
  a.sks = p->cfg.scale_kv_stride;
  a.sbs = p->cfg.scale_block_stride;
  a.contig = contig;
  a.S = p->S;
  a.block_bytes = p->block_bytes;
  a.desc = p->ring_dev + at;
  a.use_inl = inline_desc ? 1 : 0;
  std::memset(a.inl, 0, sizeof(a.inl));
  if (inline_desc) std::memcpy(a.inl, desc, n * sizeof(Desc));
  a.chunk = (int32_t)p->chunk;
  a.ppc = (int32_t)((p->chunk + piece - 1) / piece);
  a.jobs_per_block = 2 * p->cfg.num_layers * a.ppc;
  a.L2 = 2 * p->cfg.num_layers;
  a.lpc = a.cpj = 0;
  if (p->chunk < 4096) {  // several chunks per job
    a.lpc = (int32_t)(p->chunk / 16);
    a.cpj = 256 / a.lpc;
    const int per_job = a.cpj * u;
    a.jobs_per_block = (a.L2 + per_job - 1) / per_job;
  }
  a.H = p->cfg.num_kv_heads;
  a.scale_words = p->cfg.scale_dev ? 2 * p->cfg.num_layers * p->cfg.num_kv_heads : 0;
  // Scale side band through LDS (knob 1 = never, 2 = whenever it fits 64 KiB).  Default: for the
  // scatter only.  On a scale-heavy pool (512-byte chunks, 128-byte scale pieces) staging lifts the
  // scatter from 5.07 to 5.58 TB/s on-device and the swap-in from 53.3 to 55.1 GB/s, because the
  // staging side is then read as 16-byte vectors; the gather gains nothing (4.66 vs 4.58 TB/s).
  const bool lds_fits = a.scale_words && mode != 2 && (int64_t)a.scale_words * 4 <= 65536;
  a.scale_lds = lds_fits && (p->scale_lds_knob == 2 || (p->scale_lds_knob == 0 && mode == 1)) ? 1 : 0;
  a.n_data_jobs = (int64_t)n * a.jobs_per_block;
  a.n_jobs = a.n_data_jobs + (a.scale_words ? (int64_t)n : 0);

  // default caps: host link 64 workgroups, grid-stride (the link saturates there and three
  // quarters of the CUs stay free for the model); HBM to HBM one workgroup per job, up to the
  // largest grid whose thread count still fits 32 bits (64 GiB per launch at 4 KiB a job; the
  // kernel strides over what is beyond)
  constexpr int64_t kMaxGrid = ((int64_t)1 << 32) / 256 - 1;
  int64_t cap = link ? (p->max_wgs_link ? p->max_wgs_link : 64) : (p->max_wgs_device ? p->max_wgs_device : kMaxGrid);
  const int grid = (int)std::min<int64_t>(a.n_jobs, std::min(cap, kMaxGrid));

  hipEvent_t k0 = nullptr, k1 = nullptr;
  if (!sole) {
    if ((rc = get_event(p, &k0)) || (rc = get_event(p, &k1))) return rc;
    HIPCHK(p, hipEventRecord(k0, st));
  }
  if (mode == 0)
    launch_move<0>(u, grid, kind, st, a);
  else if (mode == 1)
    launch_move<1>(u, grid, kind, st, a);
  else
    launch_move<2>(u, grid, 0, st, a);
  HIPCHK(p, hipGetLastError());
  if (!sole) {
    HIPCHK(p, hipEventRecord(k1, st));
    call.kev.push_back({k0, k1});
  }
  call.st.launches++;
  call.st.grid = grid;
  return KV_OK;
}

// Path choice.  Alone, the zero-copy kernels are the fastest way over the link in both directions
// and the only one that needs no bounce traffic.  Next to a kernel that saturates HBM and the CUs
// they lose up to a fifth of their rate and make that kernel stall, while gather + copy engine
// keeps its rate and leaves the other kernel alone.  So KV_PATH_AUTO uses the copy engines when
// the caller supplied a bounce buffer (a serving loop that overlaps swaps with compute) and the
// transfer is large enough for the extra launches not to matter, and zero-copy otherwise.
constexpr int64_t kAutoDmaMinBytes = 32ll << 20;

bool use_dma(const kv_pool* p, size_t blocks) {
  if (p->dev_staging) return false;
  if (p->cfg.flags & KV_PATH_DMA) return true;
  if (p->cfg.flags & KV_PATH_ZEROCOPY) return false;
  const int64_t half_slots = p->cfg.bounce_dev ? (p->cfg.bounce_bytes / 2) / p->S : 0;
  return half_slots >= 1 && (int64_t)blocks * p->S >= kAutoDmaMinBytes;
}

void mark_blocks(kv_pool* p, const Call& c, int mode, const Desc* desc, size_t n, int seg);
hipEvent_t block_hazard(kv_pool* p, int stream, int mode, const Desc* desc, size_t n);

// Move the planned blocks between pool and arena.  out = true: pool -> arena.
// Under KV_REQ_EVENTS the descriptor list is cut into segments that end where a request ends
// (each at least segment_bytes long) and, with segment_max_bytes set, also inside a long request;
// every segment is launched on its own and followed by an event, so a request is known to be
// complete while the rest of the burst still moves.  Device-block hazards against the other
// stream are resolved per segment: a segment waits only for the newest segment of the other
// stream that touches ITS blocks, which lets a swap-in refill the blocks of a request whose
// eviction is still in flight, piece by piece behind it (Section 5.3).
int enqueue_transfer(kv_pool* p, Call& call, const Plan& plan, bool out) {
  const std::vector<Desc>& desc = plan.desc;
  char* arena = (char*)p->cfg.staging_host;
  const size_t n = desc.size();
  const bool dma = use_dma(p, n);
  call.st.path = dma ? KV_PATH_DMA : KV_PATH_ZEROCOPY;
  hipStream_t st = p->stream[call.stream];

  std::vector<size_t> seg_end;
  if (p->req_events) {
    const size_t min_blocks = (size_t)std::max<int64_t>(1, (p->segment_bytes + p->S - 1) / p->S);
    const size_t max_blocks =
        p->segment_max_bytes > 0 ? (size_t)std::max<int64_t>(1, p->segment_max_bytes / p->S) : 0;
    size_t begin = 0;
    for (size_t r = 0; r < plan.req_end.size(); r++) {
      const size_t e = plan.req_end[r].second;
      if (max_blocks)
        while (e - begin > max_blocks) {
          begin += max_blocks;
          seg_end.push_back(begin);
        }
      if (e - begin >= min_blocks || r + 1 == plan.req_end.size()) {
        seg_end.push_back(e);
        begin = e;
      }
    }
  }
  if (seg_end.empty() || seg_end.back() != n) seg_end.push_back(n);

  const int64_t half_slots = dma ? (p->cfg.bounce_bytes / 2) / p->S : 0;
  char* bounce = dma ? (char*)p->cfg.bounce_dev + (out ? 0 : (p->cfg.bounce_bytes / 2 / 16) * 16) : nullptr;
  int64_t slice = half_slots;
  if (dma && p->dma_slice > 0) slice = std::min<int64_t>(slice, p->dma_slice);
  std::vector<Desc> kd;
  size_t s0 = 0, next_req = 0;
  hipEvent_t waited = nullptr;
  for (size_t sg = 0; sg < seg_end.size(); sg++) {
    const size_t s1 = seg_end[sg];
    hipEvent_t hazard = block_hazard(p, call.stream, out ? 0 : 1, desc.data() + s0, s1 - s0);
    if (hazard && hazard != waited) {
      HIPCHK(p, hipStreamWaitEvent(st, hazard, 0));
      waited = hazard;
    }
    if (!dma) {
      int rc = enqueue_kernel(p, call, out ? 0 : 1, desc.data() + s0, s1 - s0, p->arena_dev, p->dev_staging ? 0 : 1,
                              /*sole=*/seg_end.size() == 1);
      if (rc) return rc;
    } else {
      for (size_t a0 = s0; a0 < s1; a0 += (size_t)slice) {
        const size_t a1 = std::min(s1, a0 + (size_t)slice);
        kd.resize(a1 - a0);
        for (size_t i = a0; i < a1; i++) kd[i - a0] = {desc[i].a, (int32_t)(i - a0)};
        if (out) {
          int rc = enqueue_kernel(p, call, 0, kd.data(), kd.size(), bounce, 2);
          if (rc) return rc;
        }
        // one copy per run of consecutive staging slots
        for (size_t i = a0; i < a1;) {
          size_t j = i + 1;
          while (j < a1 && (uint32_t)desc[j].b == (uint32_t)desc[j - 1].b + 1) j++;
          char* h = arena + (int64_t)(uint32_t)desc[i].b * p->S;
          char* d = bounce + (int64_t)(i - a0) * p->S;
          const size_t bytes = (j - i) * (size_t)p->S;
          if (out)
            HIPCHK(p, hipMemcpyAsync(h, d, bytes, hipMemcpyDeviceToHost, st));
          else
            HIPCHK(p, hipMemcpyAsync(d, h, bytes, hipMemcpyHostToDevice, st));
          call.st.copies++;
          i = j;
        }
        if (!out) {
          int rc = enqueue_kernel(p, call, 1, kd.data(), kd.size(), bounce, 2);
          if (rc) return rc;
        }
      }
    }
    int seg_index = -1;
    if (p->req_events) {
      hipEvent_t ev;
      int rc = get_event(p, &ev);
      if (rc) return rc;
      HIPCHK(p, hipEventRecord(ev, st));
      call.seg_ev.push_back(ev);
      seg_index = (int)call.seg_ev.size() - 1;
    }
    mark_blocks(p, call, out ? 0 : 1, desc.data() + s0, s1 - s0, seg_index);
    while (next_req < plan.req_end.size() && plan.req_end[next_req].second <= s1) {
      const uint64_t id = plan.req_end[next_req].first;
      call.req_seg.push_back({id, seg_index});
      p->req_where[id] = {call.seq, seg_index};
      next_req++;
    }
    s0 = s1;
  }
  return KV_OK;
}

// Device-block hazards between the two streams.  A new call on `stream` that READS block b must
// come after an unfinished call of the other stream that WRITES b; one that WRITES b must come
// after unfinished readers and writers of b on the other stream.  Calls of one stream finish in
// order, so the newest (call, segment) among the conflicting marks is the one event to wait for.
// mode: 0 gather (reads desc.a), 1 scatter (writes desc.a), 2 move (reads a, writes b).
hipEvent_t block_hazard(kv_pool* p, int stream, int mode, const Desc* desc, size_t n) {
  if (p->blk_reader.empty() || n == 0) return nullptr;
  // unfinished calls of the other stream, oldest first
  std::vector<Call*> other;
  for (auto& c : p->calls)
    if (c.stream != stream && c.end && c.seq != 0) {
      if (hipEventQuery(c.end) != hipSuccess) {
        (void)hipGetLastError();
        other.push_back(&c);
      }
    }
  if (other.empty()) return nullptr;
  int best_call = -1, best_seg = -2;
  auto consider = [&](const BlkMark& m) {
    if (!m.seq) return;
    for (int i = (int)other.size() - 1; i >= 0; i--)
      if ((uint32_t)other[(size_t)i]->seq == m.seq) {
        // -1 means "the whole call": later than any of its segments
        const int seg = m.seg < 0 ? INT32_MAX : m.seg;
        if (i > best_call || (i == best_call && seg > best_seg)) {
          best_call = i;
          best_seg = seg;
        }
        return;
      }
  };
  for (size_t k = 0; k < n; k++) {
    const Desc& d = desc[k];
    if (mode == 0) {
      consider(p->blk_writer[(size_t)d.a]);
    } else if (mode == 1) {
      consider(p->blk_reader[(size_t)d.a]);
      consider(p->blk_writer[(size_t)d.a]);
    } else {
      consider(p->blk_writer[(size_t)d.a]);
      consider(p->blk_reader[(size_t)d.b]);
      consider(p->blk_writer[(size_t)d.b]);
    }
  }
  if (best_call < 0) return nullptr;
  Call* c = other[(size_t)best_call];
  if (best_seg != INT32_MAX && best_seg >= 0 && best_seg < (int)c->seg_ev.size()) return c->seg_ev[(size_t)best_seg];
  return c->end;
}

void mark_blocks(kv_pool* p, const Call& c, int mode, const Desc* desc, size_t n, int seg) {
  if (p->blk_reader.empty()) return;
  const BlkMark m{(uint32_t)c.seq, seg};
  for (size_t i = 0; i < n; i++) {
    if (mode == 0) {
      p->blk_reader[(size_t)desc[i].a] = m;
    } else if (mode == 1) {
      p->blk_writer[(size_t)desc[i].a] = m;
    } else {
      p->blk_reader[(size_t)desc[i].a] = m;
      p->blk_writer[(size_t)desc[i].b] = m;
    }
  }
}

// Open a call record: cross-stream waits, caller's event, start event.  mode 2 (move) resolves its
// device-block hazards here, for the whole call; transfers (mode 0 / 1) do it per segment in
// enqueue_transfer.  Events of unfinished calls are only recycled by retire(), which never runs
// between open_call and close_call, so an event block_hazard() returns stays valid until the wait on
// it has been enqueued.
int open_call(kv_pool* p, int stream, int op, uint64_t wait_seq, void* wait_event, int mode,
              const std::vector<Desc>& desc, Call** out) {
  retire(p);
  p->last_instant = false;
  hipEvent_t blk_dep = mode == 2 ? block_hazard(p, stream, mode, desc.data(), desc.size()) : nullptr;
  if (blk_dep) HIPCHK(p, hipStreamWaitEvent(p->stream[stream], blk_dep, 0));
  p->calls.emplace_back();
  Call& c = p->calls.back();
  c.seq = ++p->seq;
  c.stream = stream;
  c.st.struct_size = sizeof(kv_stats);
  c.st.op = op;
  hipStream_t st = p->stream[stream];
  if (wait_seq) {
    Call* dep = find_call(p, wait_seq);
    if (dep && dep->stream != stream && dep->end) HIPCHK(p, hipStreamWaitEvent(st, dep->end, 0));
  }
  if (wait_event) HIPCHK(p, hipStreamWaitEvent(st, (hipEvent_t)wait_event, 0));
  int rc;
  if ((rc = get_event(p, &c.start)) || (rc = get_event(p, &c.end))) return rc;
  HIPCHK(p, hipEventRecord(c.start, st));
  *out = &c;
  return KV_OK;
}

int close_call(kv_pool* p, Call& c) {
  HIPCHK(p, hipEventRecord(c.end, p->stream[c.stream]));
  return KV_OK;
}

// The call with this sequence number, if it is unfinished and runs on another stream than `stream`
// (work of the same stream is ordered by the stream itself); 0 otherwise.
uint64_t cross_stream(kv_pool* p, int stream, uint64_t seq) {
  if (!seq) return 0;
  Call* c = find_call(p, seq);
  if (!c || c->stream == stream || seq_done(p, seq)) return 0;
  return seq;
}

// Newest unfinished call of another stream that still uses any slot in the given runs (slots of released
// extents and of swap-ins that gave their extent up).  Candidates of the caller's own stream are skipped
// one by one, so that a newer same-stream entry cannot hide an older one of the other stream.
uint64_t pending_user(kv_pool* p, int stream, const std::vector<std::pair<int64_t, int64_t>>& runs) {
  uint64_t s = 0;
  for (auto& r : runs)
    for (auto& q : p->pending)
      if (q.lo < r.first + r.second && r.first < q.hi) s = std::max(s, cross_stream(p, stream, q.seq));
  return s;
}

void fill_plan_stats(kv_pool* p, kv_stats* st, int op, size_t blocks, double plan_us) {
  st->struct_size = sizeof(kv_stats);
  st->op = op;
  st->blocks = (int64_t)blocks;
  st->bytes = (int64_t)blocks * p->S;
  st->plan_us = plan_us;
}

}  // namespace

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
  if (!p) return KV_EINVAL;
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
  bool ok = range_ok(cfg->pool_dev, pool_need);
  if (!ok) KVDBG("pool strides reach %lld bytes, past the end of the allocation", (long long)pool_need);
  if (ok && scales) {
    ok = range_ok(cfg->scale_dev, (cfg->num_layers - 1) * cfg->scale_layer_stride + cfg->scale_kv_stride +
                                      (cfg->num_blocks - 1) * cfg->scale_block_stride + scale_chunk);
    if (!ok) KVDBG("scale strides reach past the end of the allocation");
  }
  if (ok && !range_ok(cfg->staging_host, cfg->staging_bytes)) {
    ok = false;
    KVDBG("staging_bytes reaches past the end of the arena allocation");
  }
  if (ok && cfg->bounce_dev && !range_ok(cfg->bounce_dev, cfg->bounce_bytes)) {
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
  if (!rc) rc = grow_ring(p, (size_t)1 << 16);
  if (!rc) {
    p->blk_reader.assign((size_t)cfg->num_blocks, BlkMark{0, -1});
    p->blk_writer.assign((size_t)cfg->num_blocks, BlkMark{0, -1});
  }
  if (rc) {
    kv_pool_destroy(p);
    return rc;
  }
  *out = p;
  return KV_OK;
}

int kv_pool_destroy(kv_pool* p) {
  if (!p) return KV_EINVAL;
  int rc = KV_OK;
  if (!p->plan_only) {
    for (int s = 0; s < 2; s++)
      if (p->stream[s] && hipStreamSynchronize(p->stream[s]) != hipSuccess) rc = KV_EHIP;
    for (auto& c : p->calls) recycle(p, c);
    for (auto ev : p->ev_free) (void)hipEventDestroy(ev);
    if (p->ring_host) (void)hipHostFree(p->ring_host);
    if (p->ring_dev) (void)hipFree(p->ring_dev);
    for (int s = 0; s < 2; s++)
      if (p->own_stream[s]) (void)hipStreamDestroy(p->stream[s]);
  }
  delete p;
  return rc;
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
  const uint64_t dep = std::max(cross_stream(p, kEvict, plan.wait_in_seq), pending_user(p, kEvict, plan.fresh));
  if (plan.desc.empty() && !wait_event) {  // nothing to enqueue
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
                const int32_t* num_tokens, void* wait_event) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  const double t0 = now_us();
  Plan plan;
  int rc = p->planner.plan_swap_out(n, req_ids, offsets, block_ids, num_tokens, &plan);
  if (rc) return rc;
  for (int32_t i = 0; i < n; i++) p->wq.erase(req_ids[i]);  // a swapped-out request has nothing left to write through
  return swap_out_common(p, 1, plan, t0, wait_event);
}

int kv_swap_out_delta(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                      const int32_t* block_ids, const int32_t* num_tokens, int64_t block_budget, uint32_t flags,
                      int32_t* blocks_moved, void* wait_event) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  const double t0 = now_us();
  Plan plan;
  int rc = p->planner.plan_delta(n, req_ids, offsets, block_ids, num_tokens, block_budget, flags, blocks_moved,
                                 &plan);
  if (rc) return rc;
  return swap_out_common(p, 2, plan, t0, wait_event);
}

int kv_swap_in(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
               const int32_t* new_block_ids, uint32_t flags, void* wait_event) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
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

int kv_move_blocks(kv_pool* p, int64_t n, const int32_t* src_ids, const int32_t* dst_ids, void* wait_event) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
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

int kv_sync(kv_pool* p) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  if (p->plan_only) return KV_OK;
  for (int s = 0; s < 2; s++) HIPCHK(p, hipStreamSynchronize(p->stream[s]));
  retire(p);
  return KV_OK;
}

int kv_req_reserve(kv_pool* p, uint64_t req_id, int32_t max_blocks) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
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

int kv_req_release(kv_pool* p, uint64_t req_id) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  kvswap::Req was;
  int rc = p->planner.release(req_id, &was);
  if (!rc) p->wq.erase(req_id);
  if (rc || p->plan_only) return rc;
  // the slots may still be in use by unfinished work of either stream: later users wait for it
  for (uint64_t s : {was.in_seq, was.out_seq})
    if (s && was.cap && !seq_done(p, s)) p->pending.push_back({was.base, was.base + was.cap, s});
  return KV_OK;
}

int kv_req_query(kv_pool* p, uint64_t req_id, int64_t* staging_offset, int32_t* cap_blocks, int32_t* blocks_staged,
                 int32_t* watermark, int32_t* swapped) {
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

int kv_last_stats(kv_pool* p, kv_stats* out) {
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

int kv_req_poll(kv_pool* p, uint64_t req_id) {
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
  return KV_EHIP;
}

int kv_req_wait(kv_pool* p, uint64_t req_id) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  if (p->plan_only) return KV_OK;
  hipEvent_t ev = req_event(p, req_id);
  if (ev) HIPCHK(p, hipEventSynchronize(ev));
  return KV_OK;
}

int64_t kv_last_timeline(kv_pool* p, uint64_t* req_ids, float* done_ms, int64_t cap) {
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

int kv_io_stats_get(kv_pool* p, kv_io_stats* out) {
  if (!p || !out) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  io_snapshot(p, out);
  return KV_OK;
}

static int64_t budget_blocks_locked(kv_pool* p, int32_t dir, double interval_us);

int64_t kv_budget_blocks(kv_pool* p, int32_t dir, double interval_us) {
  if (!p || (dir != 0 && dir != 1) || !(interval_us >= 0)) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  return budget_blocks_locked(p, dir, interval_us);
}

int kv_swap_out_delta_timed(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets,
                            const int32_t* block_ids, const int32_t* num_tokens, const float* priority,
                            double interval_us, uint32_t flags, int32_t* blocks_moved, int64_t* budget_used,
                            void* wait_event) {
  if (!p || !(interval_us >= 0)) return KV_EINVAL;
  if (n < 0 || (n > 0 && (!req_ids || !offsets || !num_tokens))) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
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

int kv_wq_post(kv_pool* p, int32_t n, const uint64_t* req_ids, const int32_t* offsets, const int32_t* block_ids,
               const int32_t* num_tokens, const double* priority) {
  if (!p || n < 0 || (n > 0 && (!req_ids || !offsets || !num_tokens))) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
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

int kv_wq_remove(kv_pool* p, uint64_t req_id) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  return p->wq.erase(req_id) ? KV_OK : KV_ENOENT;
}

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

int kv_wq_pending(kv_pool* p, int64_t* blocks, int32_t* requests) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  wq_count(p, blocks, requests);
  return KV_OK;
}

int kv_wq_drain(kv_pool* p, double interval_us, int64_t block_budget, uint32_t flags, int64_t* blocks_written,
                int64_t* blocks_pending, int64_t* budget_used, void* wait_event) {
  if (!p || !(interval_us >= 0) || block_budget < 0) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  const double t0 = now_us();
  const bool timed = block_budget == 0 && interval_us > 0;
  const int64_t budget = timed ? budget_blocks_locked(p, 0, interval_us) : block_budget;
  if (budget_used) *budget_used = budget;
  std::vector<std::pair<uint64_t, const kv_pool::WqEntry*>> order;
  order.reserve(p->wq.size());
  for (auto& kvp : p->wq) order.push_back({kvp.first, &kvp.second});
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

int64_t kv_last_plan(kv_pool* p, int32_t* phys, int64_t* slot, int64_t cap) {
  if (!p) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  const int64_t n = (int64_t)p->last_plan.size();
  for (int64_t i = 0; i < n && i < cap; i++) {
    if (phys) phys[i] = p->last_plan[(size_t)i].a;
    if (slot) slot[i] = (int64_t)(uint32_t)p->last_plan[(size_t)i].b;
  }
  return n;
}

int kv_pool_tune(kv_pool* p, int32_t what, int64_t value) {
  if (!p || value < 0) return KV_EINVAL;
  std::lock_guard<std::mutex> g(p->mu);
  switch (what) {
    case KV_TUNE_MAX_WGS_DEVICE:
      p->max_wgs_device = std::min<int64_t>(value, 1 << 30);
      return KV_OK;
    case KV_TUNE_MAX_WGS_LINK:
      p->max_wgs_link = std::min<int64_t>(value, 1 << 30);
      return KV_OK;
    case KV_TUNE_KERNEL_VARIANT:
      if (value != 0 && value != 1 && value != 2 && value != 4 && value != 8) return KV_EINVAL;
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
    default:
      return KV_EINVAL;
  }
}

int kv_last_hip_error(const kv_pool* p) { return p ? p->last_hip : 0; }

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
  if (!range_ok(dst_dev, bytes) || !range_ok(src_dev, bytes)) return -1.0;
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
