// The swap library's host runtime AND its kernel source on the CPU, against the C oracle.
//
// Built by tests/test_native_sanitizers.py with a host compiler, AddressSanitizer + UBSan and the stand-in HIP
// runtime of tests/native/mockhip: kvswap.hip (with runtime.hip.inc and kernels.hip.inc) is compiled unchanged;
// streams are queues whose operations run when the stand-in's executor picks them, so this driver chooses how
// far the "device" lags behind the host and which of the two streams is starved.  A seeded serving history
// (growth with budgeted write-through, cold and warm preemption of one or several requests, resumption with and
// without keeping the host image, compaction moves, releases, re-reservations, write-queue rounds, calls that
// must be refused) is played through the C ABI with
// no synchronisation inside a chunk; blocks and slots given up by one call go to the next at once.  After every
// chunk pool, scales and arena must equal what the oracle reaches by running the same calls one after the other,
// and the per-request state must agree.  A missing wait between the streams shows up as a byte difference, a
// wait that can never be satisfied as a reported deadlock, an out-of-bounds access of a kernel or of the host
// code as a sanitizer error.
//
// With a third argument a second thread polls the handle (request state, statistics, queue length) all through
// every chunk: built with ThreadSanitizer this checks that every entry point takes the handle's lock, and the
// comparison with the oracle that such readers change nothing.
//
// "hipfail": in one chunk some HIP call inside the library fails (the stand-in's failure injection); "nomem": some
// allocation made while a library call runs throws std::bad_alloc.  Either the library absorbs it and the history
// goes on equal to the oracle, or the call returns KV_EHIP / KV_ENOMEM; from then on the handle must refuse every
// call that changes state, still answer queries, and kv_pool_destroy must release everything (LeakSanitizer).
//
// usage: runtime_on_mock_hip <seed> <chunks> [poller|hipfail|nomem]
// DRIVER_TRACE=1 in the environment prints every call with its block tables, MOCKHIP_TRACE=1 the moment an injected
// failure fires; a mismatch in the pool names the first differing layer, K or V, and block.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <atomic>
#include <cstdio>
#include <thread>
#include <map>
#include <random>
#include <vector>

#include "kvswap.h"
extern "C" {
#include "../../oracle/kv_oracle.h"
}

// ---- allocation failures, only while a library call runs ----
static bool g_in_lib = false;
static long g_new_fail_in = 0;
static bool g_new_fired = false;
#if defined(__has_feature) && __has_feature(thread_sanitizer)
// ThreadSanitizer brings its own operator new: the "nomem" mode is not available in that build
#else
void* operator new(std::size_t n) {
  if (g_in_lib && g_new_fail_in > 0 && --g_new_fail_in == 0) {
    g_new_fired = true;
    throw std::bad_alloc();
  }
  if (void* q = std::malloc(n ? n : 1)) return q;
  throw std::bad_alloc();
}
void* operator new[](std::size_t n) { return operator new(n); }
void* operator new(std::size_t n, const std::nothrow_t&) noexcept {
  try {
    return operator new(n);
  } catch (...) {
    return nullptr;
  }
}
void* operator new[](std::size_t n, const std::nothrow_t& t) noexcept { return operator new(n, t); }
void operator delete(void* q) noexcept { std::free(q); }
void operator delete(void* q, std::size_t) noexcept { std::free(q); }
void operator delete[](void* q) noexcept { std::free(q); }
void operator delete[](void* q, std::size_t) noexcept { std::free(q); }
void operator delete(void* q, const std::nothrow_t&) noexcept { std::free(q); }
void operator delete[](void* q, const std::nothrow_t&) noexcept { std::free(q); }
#endif
static int leave_lib(int rc) {
  g_in_lib = false;
  return rc;
}
#define LIB(call) (g_in_lib = true, leave_lib(call))
// The same for the entry points that only enqueue: they must come back without having waited for the device (the
// descriptor ring is sized so that a burst never finds it full; nothing else in them waits).
static int leave_async(int rc, long waits_before, const char* what) {
  g_in_lib = false;
  if (mockhip::host_waits() != waits_before) {
    std::fprintf(stderr, "MISMATCH: %s waited for the device on the host\n", what);
    std::exit(1);
  }
  return rc;
}
#define LIB_ASYNC(call) (g_in_lib = true, leave_async(call, mockhip::host_waits(), #call))

namespace {

struct Failed {  // the armed failure has surfaced as this status of a library call
  int rc;
};

[[noreturn]] void die(const char* what, int chunk, int step) {
  std::fprintf(stderr, "MISMATCH in chunk %d at step %d: %s\n", chunk, step, what);
  std::exit(1);
}

struct Geo {
  int L, H, D, B, e, dtype;
  int64_t N, chunk, block_bytes, scale_chunk, S, ls, ks, bs, sls, sks, sbs;
};

}  // namespace

int main(int argc, char** argv) {
  const uint64_t seed = argc > 1 ? std::strtoull(argv[1], nullptr, 10) : 1;
  const int chunks = argc > 2 ? std::atoi(argv[2]) : 8;
  const std::string extra = argc > 3 ? argv[3] : "";
  const bool poller = extra == "poller", hipfail = extra == "hipfail", nomem = extra == "nomem";
  std::mt19937_64 rng(seed * 7919 + 13);
  auto rnd = [&](int64_t lo, int64_t hi) { return lo + (int64_t)(rng() % (uint64_t)(hi - lo + 1)); };
  mockhip::reset(seed);

  // ---- configuration of this run, all from the seed ----
  Geo g;
  bool scales = seed % 4 == 3;
  if (seed >= 192) {
    // beyond the 192 fixed combinations: a geometry of its own per seed, so that the kernels' piece arithmetic
    // (pieces per chunk, chunks per job, ragged last pieces, scale words) meets shapes nobody wrote down
    for (;;) {
      const int e = (int)rnd(1, 2);
      g = {(int)rnd(1, 4), (int)rnd(1, 8), 8 * (int)rnd(1, 16), (int)rnd(1, 24), e, e == 1 ? KV_FP8_E4M3 : (rnd(0, 1) ? KV_F16 : KV_BF16),
           0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0};
      const int64_t chunk = (int64_t)g.B * g.H * g.D * g.e;
      if (chunk % 16 || chunk > 20480) continue;
      scales = e == 1 && (g.L * g.H) % 2 == 0 && rnd(0, 2) != 0;
      break;
    }
  } else
  switch (seed % 4) {
    case 0: g = {2, 2, 8, 2, 2, KV_F16, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}; break;       // 64-byte chunks: several per job
    case 1: g = {1, 4, 64, 8, 2, KV_BF16, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}; break;     // 4 KiB chunks: one piece each
    case 2: g = {2, 4, 72, 16, 2, KV_F16, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}; break;     // 9 KiB chunks: ragged pieces
    default: g = {3, 4, 32, 4, 1, KV_FP8_E4M3, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0}; break; // fp8, 512-byte chunks, scales
  }
  g.N = rnd(90, 140);
  g.chunk = (int64_t)g.B * g.H * g.D * g.e;
  g.block_bytes = 2 * g.L * g.chunk;
  g.scale_chunk = scales ? g.H * 4 : 0;
  g.S = g.block_bytes + 2 * g.L * g.scale_chunk;
  const bool padded = (seed / 4) % 2 == 1;
  g.bs = g.chunk + (padded ? 48 : 0);
  g.ks = g.N * g.bs + (padded ? 32 : 0);
  g.ls = 2 * g.ks + (padded ? 64 : 0);
  g.sbs = g.scale_chunk + (padded ? 8 : 0);
  g.sks = g.N * g.sbs + (padded ? 4 : 0);
  g.sls = 2 * g.sks + (padded ? 12 : 0);
  const int mode = (int)((seed / 8) % 3);            // 0 zero-copy, 1 copy engines, 2 device arena
  const bool events = (seed / 24) % 2 == 1;
  const int policy = (int)((seed / 48) % 4);         // random, starve evict, starve load, lazy
  const int64_t slots = 70;
  const int R = 9, cap_max = 20;

  const size_t pool_bytes = (size_t)(g.L * g.ls), scale_bytes = (size_t)(scales ? g.L * g.sls : 16);
  const size_t stag_bytes = (size_t)(slots * g.S + 24);
  std::vector<uint8_t> pool_a(pool_bytes), scale_a(scale_bytes), stag_a(stag_bytes, 0xA5);
  for (auto& b : pool_a) b = (uint8_t)rng();
  for (auto& b : scale_a) b = (uint8_t)rng();
  uint8_t *pool_b = nullptr, *scale_b = nullptr, *stag_b = nullptr, *bounce = nullptr;
  if (hipMalloc((void**)&pool_b, pool_bytes) || hipMalloc((void**)&scale_b, scale_bytes)) return 3;
  if (mode == 2 ? hipMalloc((void**)&stag_b, stag_bytes) : hipHostMalloc((void**)&stag_b, stag_bytes, 0)) return 3;
  const int64_t bounce_slots = rnd(1, 5);
  if (mode == 1 && hipMalloc((void**)&bounce, (size_t)(2 * bounce_slots * g.S))) return 3;
  std::memcpy(pool_b, pool_a.data(), pool_bytes);
  std::memcpy(scale_b, scale_a.data(), scale_bytes);
  std::memset(stag_b, 0xA5, stag_bytes);

  ora_config oc;
  std::memset(&oc, 0, sizeof(oc));
  oc.L = g.L; oc.H = g.H; oc.D = g.D; oc.B = g.B; oc.elem_bytes = g.e; oc.N = g.N;
  oc.pool = pool_a.data(); oc.layer_stride = g.ls; oc.kv_stride = g.ks; oc.block_stride = g.bs;
  oc.scale = scales ? scale_a.data() : nullptr;
  oc.s_layer_stride = g.sls; oc.s_kv_stride = g.sks; oc.s_block_stride = g.sbs;
  oc.staging = stag_a.data(); oc.staging_bytes = (int64_t)stag_a.size();
  ora_state* ora = ora_create(&oc);
  if (!ora || ora_slot_bytes(ora) != g.S) die("oracle set-up", -1, -1);

  hipStream_t evict, load, compute;  // compute: the "model", which writes KV into the pool on a stream of its own
  hipStreamCreateWithFlags(&evict, hipStreamNonBlocking);
  hipStreamCreateWithFlags(&load, hipStreamNonBlocking);
  hipStreamCreateWithFlags(&compute, hipStreamNonBlocking);
  hipEvent_t ev_evict, ev_load, ev_compute;
  hipEventCreate(&ev_evict);
  hipEventCreate(&ev_load);
  hipEventCreate(&ev_compute);
  kv_pool_config kc;
  std::memset(&kc, 0, sizeof(kc));
  kc.struct_size = sizeof(kc);
  kc.num_layers = g.L; kc.num_kv_heads = g.H; kc.head_dim = g.D; kc.block_size = g.B; kc.dtype = g.dtype;
  kc.num_blocks = g.N; kc.pool_dev = pool_b; kc.layer_stride = g.ls; kc.kv_stride = g.ks; kc.block_stride = g.bs;
  kc.scale_dev = scales ? scale_b : nullptr;
  kc.scale_layer_stride = g.sls; kc.scale_kv_stride = g.sks; kc.scale_block_stride = g.sbs;
  kc.staging_host = stag_b; kc.staging_bytes = (int64_t)stag_bytes;
  kc.bounce_dev = bounce; kc.bounce_bytes = bounce ? 2 * bounce_slots * g.S : 0;
  kc.evict_stream = evict; kc.load_stream = load;
  kc.flags = (mode == 0 ? KV_PATH_ZEROCOPY : mode == 1 ? KV_PATH_DMA : KV_STAGING_DEVICE) | (events ? KV_REQ_EVENTS : 0);
  kv_pool* kp = nullptr;
  if (kv_pool_create(&kc, &kp) != KV_OK) die("kv_pool_create", -1, -1);
  // Scale side band: the library's default (through LDS for the scatter only), never, or always.  A launch with
  // LDS runs its lanes as fibers; a ThreadSanitizer build cannot do that and keeps to the path without LDS.
  const int64_t lds_knob = mockhip::fibers_available() ? (int64_t)(seed % 3) : 1;
  if (kv_pool_tune(kp, KV_TUNE_SCALE_LDS, lds_knob) != KV_OK) die("tune", -1, -1);
  if (events) {
    kv_pool_tune(kp, KV_TUNE_SEGMENT_BYTES, rnd(1, 3) * g.S);
    if (rnd(0, 1)) kv_pool_tune(kp, KV_TUNE_SEGMENT_MAX_BYTES, rnd(1, 4) * g.S);
  }
  kv_pool_tune(kp, KV_TUNE_PHASE_BYTES, rnd(1, 3) * g.S);  // eviction and loading in one call: phases of one to three blocks
  if (rnd(0, 1)) kv_pool_tune(kp, KV_TUNE_PHASE_WGS_IN, rnd(1, 6));
  if (rnd(0, 2) == 0) kv_pool_tune(kp, KV_TUNE_MAX_WGS_LINK, rnd(1, 5));
  if (mode == 0 && rnd(0, 1)) kv_pool_tune(kp, KV_TUNE_HOST_STORES, 1);  // the other lane layout of the gather into the host arena
  if (rnd(0, 2) == 0) kv_pool_tune(kp, KV_TUNE_MAX_WGS_DEVICE, rnd(1, 7));
  if (mode == 1 && rnd(0, 1)) kv_pool_tune(kp, KV_TUNE_DMA_SLICE_BLOCKS, rnd(1, 3));
  if (mode == 2 && rnd(0, 1)) kv_pool_tune(kp, KV_TUNE_SCATTER_ORDER, 2);  // the plane-by-plane build of the scatter
  if (seed < 192 && seed % 4 == 1 && mode != 0 && rnd(0, 1)) kv_pool_tune(kp, KV_TUNE_KERNEL_VARIANT, 101);  // 4 KiB chunks: the pipelined build
  if (seed >= 192 && rnd(0, 1)) {  // loads in flight per lane: every build of the kernel
    const int64_t u[7] = {1, 2, 4, 8, 101, 102, 104};  // 10x: resident pipelined workgroups, where the chunk allows
    if (kv_pool_tune(kp, KV_TUNE_KERNEL_VARIANT, u[rnd(0, 6)]) != KV_OK) die("tune", -1, -1);
  }

  // ---- the serving history ----
  std::vector<int32_t> free_list((size_t)g.N);
  for (int64_t i = 0; i < g.N; i++) free_list[(size_t)i] = (int32_t)i;
  std::shuffle(free_list.begin(), free_list.end(), rng);
  std::vector<std::vector<int32_t>> table((size_t)R + 1);
  std::vector<int32_t> length((size_t)R + 1, 0);
  std::vector<int> state((size_t)R + 1, 0);  // 0 idle, 1 running, 2 out
  std::vector<uint64_t> trace_ids;  // what the last csr() built, for DRIVER_TRACE
  std::vector<int32_t> trace_off, trace_blk;
  std::vector<int> cap((size_t)R + 1, 0);    // extent sizes differ, so that a new extent can lie over parts of several old ones
  long calls = 0;

  const bool trace = std::getenv("DRIVER_TRACE") != nullptr;
  auto both = [&](int rc_lib, int rc_ora, const char* what, int chunk, int step) {
    if (trace) {
      std::fprintf(stderr, "[%d.%d] %s:", chunk, step, what);
      for (size_t i = 0; i + 1 < trace_off.size(); i++) {
        std::fprintf(stderr, " r%llu{", (unsigned long long)trace_ids[i]);
        for (int32_t j = trace_off[i]; j < trace_off[i + 1]; j++) std::fprintf(stderr, "%d ", trace_blk[(size_t)j]);
        std::fprintf(stderr, "}");
      }
      std::fprintf(stderr, "\n");
      trace_ids.clear(); trace_off.clear(); trace_blk.clear();
    }
    if ((rc_lib == KV_EHIP && mockhip::failure_fired()) || (rc_lib == KV_ENOMEM && g_new_fired)) throw Failed{rc_lib};
    if (rc_lib != rc_ora || rc_lib != 0) {
      std::fprintf(stderr, "%s: library %d oracle %d (hip error %d, injected failure fired: %d)\n", what, rc_lib, rc_ora,
                   kv_last_hip_error(kp), (int)mockhip::failure_fired());
      die("return code", chunk, step);
    }
    calls++;
  };
  auto csr = [&](const std::vector<int>& rs, std::vector<uint64_t>& ids, std::vector<int32_t>& off,
                 std::vector<int32_t>& blk, std::vector<int32_t>& tok) {
    ids.clear(); off.assign(1, 0); blk.clear(); tok.clear();
    for (int r : rs) {
      ids.push_back((uint64_t)r);
      blk.insert(blk.end(), table[(size_t)r].begin(), table[(size_t)r].end());
      off.push_back((int32_t)blk.size());
      tok.push_back(length[(size_t)r]);
    }
    trace_ids = ids; trace_off = off; trace_blk = blk;
  };
  // a reservation may find no run of free slots long enough: both sides must say so, and nothing has changed then
  auto reserve = [&](int r, int64_t n, const char* what, int chunk, int step) {
    const int rc_lib = LIB(kv_req_reserve(kp, (uint64_t)r, n)), rc_ora = ora_req_reserve(ora, (uint64_t)r, n);
    if ((rc_lib == KV_EHIP && mockhip::failure_fired()) || (rc_lib == KV_ENOMEM && g_new_fired)) throw Failed{rc_lib};
    if (rc_lib != rc_ora || (rc_lib != 0 && rc_lib != KV_ENOSPC)) {
      std::fprintf(stderr, "%s: library %d oracle %d\n", what, rc_lib, rc_ora);
      die("return code", chunk, step);
    }
    calls++;
    return rc_lib == 0;
  };
  auto give_up = [&](int r) {
    free_list.insert(free_list.end(), table[(size_t)r].begin(), table[(size_t)r].end());
    table[(size_t)r].clear();
  };

  const int fail_chunk = hipfail || nomem ? (int)rnd(0, chunks - 1) : -1;
  const long fail_at = hipfail ? (long)rnd(1, 60) : (long)rnd(1, 300);
  bool handled = false;
  int handled_rc = 0;
  try {
  for (int chunk = 0; chunk < chunks; chunk++) {
    if (chunk == fail_chunk) {
      if (hipfail) mockhip::fail_after(fail_at, 999);
      if (nomem) g_new_fail_in = fail_at;
    }
    // who lags in this chunk
    const int pol = policy == 0 ? mockhip::kRandom : policy == 3 ? mockhip::kLazy : (chunk + policy) % 2 ? mockhip::kStarve0 : mockhip::kStarve1;
    mockhip::set_policy(pol, pol == mockhip::kStarve0 ? evict : pol == mockhip::kStarve1 ? load : nullptr);
    std::vector<int32_t> held;
    // Once the model has written on its own stream, the calls that WRITE pool blocks (swap-in, move) name the
    // model's latest event, as an engine does when it hands blocks the model has touched to another owner.
    void* after_model = nullptr;
    if (chunk == 0) {
      // A fixed opening on the empty arena: request 1 (slots 0..3) is swapped out and resumed without keeping its image,
      // so its slots are still being read by the load stream; request 2 (slots 4..6) is swapped out AFTER that and
      // released, so its slots are still being written by the evict stream; request 3 then reserves slots 0..6 and
      // writes them at once.  That write has to wait for the older call on the other stream, not for the newer one
      // on its own.
      std::vector<uint64_t> ids;
      std::vector<int32_t> off, blk, tok;
      auto fill = [&](int r, int n) {
        if (!reserve(r, n, "opening reserve", 0, -1)) die("opening reserve", 0, -1);
        cap[(size_t)r] = n; state[(size_t)r] = 1; length[(size_t)r] = (int32_t)(n * g.B);
        for (int j = 0; j < n; j++) { table[(size_t)r].push_back(free_list.back()); free_list.pop_back(); }
      };
      auto cold_out = [&](int r) {
        csr({r}, ids, off, blk, tok);
        both(LIB_ASYNC(kv_swap_out(kp, 1, ids.data(), off.data(), blk.data(), tok.data(), nullptr)),
             ora_swap_out(ora, 1, ids.data(), off.data(), blk.data(), tok.data()), "opening swap_out", 0, -1);
        give_up(r);
        state[(size_t)r] = 2;
      };
      // Before that, twice: a write-through call that takes slots and moves nothing.  Request 4 is swapped out and resumed
      // without keeping its image, so the load stream still reads its old slots.  (a) Request 5, unknown so far, is written
      // through below one block: it gets the extent request 4 gave up and nothing is enqueued.  (b) Request 6 sits in the
      // slot before another such extent and grows into a new partial block: its extent grows over it in place, again with
      // nothing to enqueue.  The next delta of either completes the block and writes the slot: it must wait for the swap-in.
      if (g.B >= 2) {
        std::vector<int32_t> ma(1), mb(1);
        auto delta_of = [&](int r, int blocks, int32_t tokens, const char* what) {
          while ((int)table[(size_t)r].size() < blocks) { table[(size_t)r].push_back(free_list.back()); free_list.pop_back(); }
          length[(size_t)r] = tokens;
          csr({r}, ids, off, blk, tok);
          both(LIB_ASYNC(kv_swap_out_delta(kp, 1, ids.data(), off.data(), blk.data(), tok.data(), 0, 0, mb.data(), nullptr)),
               ora_swap_out_delta(ora, 1, ids.data(), off.data(), blk.data(), tok.data(), 0, 0, ma.data()), what, 0, -1);
          if (ma != mb) die("blocks_moved", 0, -1);
        };
        auto out_and_back = [&](int r, int n) {  // afterwards the load stream reads the n slots the request has just given up
          fill(r, n);
          cold_out(r);
          for (int j = 0; j < n; j++) { table[(size_t)r].push_back(free_list.back()); free_list.pop_back(); }
          csr({r}, ids, off, blk, tok);
          both(LIB_ASYNC(kv_swap_in(kp, 1, ids.data(), off.data(), blk.data(), 0, nullptr)), ora_swap_in(ora, 1, ids.data(), off.data(), blk.data(), 0),
               "opening swap_in", 0, -1);
          held.insert(held.end(), table[(size_t)r].begin(), table[(size_t)r].end());
          table[(size_t)r].clear();
          length[(size_t)r] = 0; state[(size_t)r] = 0;
        };
        auto finish = [&](int r) {
          give_up(r);
          length[(size_t)r] = 0; state[(size_t)r] = 0;
          both(LIB(kv_req_release(kp, (uint64_t)r)), ora_req_release(ora, (uint64_t)r), "opening release", 0, -1);
        };
        // (a)
        out_and_back(4, 2);                                           // slots 0..1
        delta_of(5, 1, 1, "delta below one block");                   // takes slot 0, moves nothing
        if (mb[0] != 0) die("a delta below one block moved something", 0, -1);
        delta_of(5, 1, (int32_t)g.B, "delta that completes the block");  // writes slot 0
        finish(5);
        // (b)
        delta_of(6, 1, (int32_t)g.B, "delta of one full block");      // slot 0
        out_and_back(4, 2);                                           // slots 1..2
        delta_of(6, 2, (int32_t)g.B + 1, "growth into a partial block");  // the extent grows over slot 1, nothing moves
        if (mb[0] != 0) die("growth into a partial block moved something", 0, -1);
        delta_of(6, 2, 2 * (int32_t)g.B, "delta that completes the second block");  // writes slot 1
        finish(6);
      }
      fill(1, 4);
      fill(2, 3);
      cold_out(1);
      for (int j = 0; j < 4; j++) { table[1].push_back(free_list.back()); free_list.pop_back(); }
      csr({1}, ids, off, blk, tok);
      both(LIB_ASYNC(kv_swap_in(kp, 1, ids.data(), off.data(), blk.data(), 0, nullptr)), ora_swap_in(ora, 1, ids.data(), off.data(), blk.data(), 0),
           "opening swap_in", 0, -1);
      held.insert(held.end(), table[1].begin(), table[1].end());  // kept out of circulation until the chunk's comparison: what the swap-in wrote must still be there
      table[1].clear();
      length[1] = 0; state[1] = 0;
      cold_out(2);
      give_up(2);
      length[2] = 0; state[2] = 0;
      both(LIB(kv_req_release(kp, 2)), ora_req_release(ora, 2), "opening release", 0, -1);
      fill(3, 7);
      csr({3}, ids, off, blk, tok);
      std::vector<int32_t> ma(1), mb(1);
      both(LIB_ASYNC(kv_swap_out_delta(kp, 1, ids.data(), off.data(), blk.data(), tok.data(), 0, 0, mb.data(), nullptr)),
           ora_swap_out_delta(ora, 1, ids.data(), off.data(), blk.data(), tok.data(), 0, 0, ma.data()), "opening delta", 0, -1);
      if (ma != mb) die("blocks_moved", 0, -1);
    }
    std::atomic<bool> stop{false};
    std::atomic<long> polls{0};
    std::thread side;
    if (poller)
      side = std::thread([&] {
        uint64_t x = seed * 977 + (uint64_t)chunk;
        while (!stop.load()) {
          x = x * 6364136223846793005ull + 1442695040888963407ull;
          const uint64_t r = 1 + (x >> 33) % (uint64_t)R;
          int64_t o, blocks;
          int32_t a, b, c, d, reqs;
          kv_io_stats io;
          kv_stats st;
          std::memset(&io, 0, sizeof(io)); io.struct_size = sizeof(io);
          std::memset(&st, 0, sizeof(st)); st.struct_size = sizeof(st);
          switch ((x >> 20) % 6) {
            case 0: (void)kv_req_poll(kp, r); break;
            case 1: (void)kv_req_query(kp, r, &o, &a, &b, &c, &d); break;
            case 2: (void)kv_io_stats_get(kp, &io); break;
            case 3: (void)kv_last_stats(kp, &st); break;
            case 4: if (kv_req_wait(kp, r) != KV_OK) die("kv_req_wait", chunk, -2); break;
            default: (void)kv_wq_pending(kp, &blocks, &reqs); break;
          }
          polls++;
          std::this_thread::yield();
        }
      });
    for (int step = 0; step < 45; step++) {
      std::vector<int> running, out, idle;
      for (int r = 1; r <= R; r++) (state[(size_t)r] == 1 ? running : state[(size_t)r] == 2 ? out : idle).push_back(r);
      std::vector<uint64_t> ids;
      std::vector<int32_t> off, blk, tok;
      if (rnd(0, 7) == 0 && !hipfail && !nomem) {
        // the application leaves an error of its own behind in the thread (a time asked of an event that was never
        // recorded): the library must not take it for a failure of its next launch
        hipEvent_t never;
        float ms;
        hipEventCreate(&never);
        (void)hipEventElapsedTime(&ms, never, never);
        hipEventDestroy(never);
      }
      int op = (int)rnd(0, 14);
      if (op == 0 && !idle.empty() && free_list.size() > 8) {  // start
        const int r = idle[(size_t)rnd(0, (int64_t)idle.size() - 1)];
        cap[(size_t)r] = (int)rnd(3, cap_max);
        if (!reserve(r, cap[(size_t)r], "reserve", chunk, step)) continue;
        state[(size_t)r] = 1; length[(size_t)r] = 0; table[(size_t)r].clear();
        running.assign(1, r);
        op = 1;
      }
      if ((op == 1 || op == 2) && !running.empty()) {  // grow + budgeted write-through
        std::shuffle(running.begin(), running.end(), rng);
        std::vector<int> rs(running.begin(), running.begin() + rnd(1, (int64_t)running.size()));
        std::vector<int> with;
        for (int r : rs) {
          const int32_t want = (int32_t)std::min<int64_t>(length[(size_t)r] + rnd(1, 3 * g.B), (int64_t)cap[(size_t)r] * g.B);
          while ((int64_t)table[(size_t)r].size() * g.B < want && !free_list.empty()) {
            table[(size_t)r].push_back(free_list.back());
            free_list.pop_back();
          }
          length[(size_t)r] = (int32_t)std::min<int64_t>(want, (int64_t)table[(size_t)r].size() * g.B);
          if (!table[(size_t)r].empty()) with.push_back(r);
        }
        if (!with.empty()) {
          csr(with, ids, off, blk, tok);
          const int64_t budget = rnd(0, 5);
          std::vector<int32_t> ma(with.size(), -1), mb(with.size(), -1);
          both(LIB_ASYNC(kv_swap_out_delta(kp, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data(), budget, 0, mb.data(), nullptr)),
               ora_swap_out_delta(ora, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data(), budget, 0, ma.data()),
               "delta", chunk, step);
          if (ma != mb) die("blocks_moved", chunk, step);
        }
      } else if ((op == 3 || op == 4 || op == 5) && !running.empty()) {  // preempt: warm, cold, several at once
        std::shuffle(running.begin(), running.end(), rng);
        std::vector<int> rs;
        for (int r : running)
          if (!table[(size_t)r].empty() && (int)rs.size() < (op == 5 ? 3 : 1)) rs.push_back(r);
        if (rs.empty()) continue;
        csr(rs, ids, off, blk, tok);
        if (op == 4) {
          both(LIB_ASYNC(kv_swap_out(kp, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data(), nullptr)),
               ora_swap_out(ora, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data()), "swap_out", chunk, step);
        } else {
          std::vector<int32_t> ma(rs.size()), mb(rs.size());
          both(LIB_ASYNC(kv_swap_out_delta(kp, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data(), 0, KV_DELTA_INCLUDE_TAIL, mb.data(), nullptr)),
               ora_swap_out_delta(ora, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data(), 0, KV_DELTA_INCLUDE_TAIL, ma.data()),
               "tail delta", chunk, step);
        }
        for (int r : rs) { give_up(r); state[(size_t)r] = 2; }
      } else if ((op == 6 || op == 7) && !out.empty()) {  // resume one or several, with or without the host image
        std::shuffle(out.begin(), out.end(), rng);
        std::vector<int> rs;
        size_t need = 0;
        for (int r : out) {
          const size_t nb = (size_t)((length[(size_t)r] + g.B - 1) / g.B);
          if ((int)rs.size() < (op == 7 ? 3 : 1) && need + nb <= free_list.size()) { rs.push_back(r); need += nb; }
        }
        if (rs.empty()) continue;
        for (int r : rs) {
          const size_t nb = (size_t)((length[(size_t)r] + g.B - 1) / g.B);
          for (size_t j = 0; j < nb; j++) { table[(size_t)r].push_back(free_list.back()); free_list.pop_back(); }  // LIFO
        }
        csr(rs, ids, off, blk, tok);
        const bool keep = rnd(0, 9) < 7;
        both(LIB_ASYNC(kv_swap_in(kp, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), keep ? KV_KEEP_STAGING : 0, after_model)),
             ora_swap_in(ora, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), keep ? KV_KEEP_STAGING : 0), "swap_in", chunk, step);
        for (int r : rs) {
          state[(size_t)r] = 1;
          if (!keep && (rnd(0, 9) < 4 || !reserve(r, cap[(size_t)r], "re-reserve", chunk, step))) {
            // the request ends here, by choice or for want of room (the swap-in has already dropped its record):
            // its old slots stay in use by that swap-in until whoever reserves them next
            give_up(r);
            length[(size_t)r] = 0; state[(size_t)r] = 0;
          }
        }
      } else if (op == 14 && !running.empty() && !out.empty()) {
        // Eviction and loading in one call: one or two running requests are evicted cold while one or two others come
        // back, and the blocks the evicted ones give up are the first the resumed ones are handed.
        std::shuffle(running.begin(), running.end(), rng);
        std::shuffle(out.begin(), out.end(), rng);
        std::vector<int> ev, ld;
        for (int r : running)
          if (!table[(size_t)r].empty() && (int)ev.size() < (int)rnd(1, 2)) ev.push_back(r);
        if (ev.empty()) continue;
        std::vector<int32_t> avail;
        for (int r : ev) avail.insert(avail.end(), table[(size_t)r].begin(), table[(size_t)r].end());
        if (rnd(0, 1)) std::shuffle(avail.begin(), avail.end(), rng);  // in any order: a load phase may need a late eviction phase
        size_t room = avail.size() + free_list.size(), need_blocks = 0;
        for (int r : out) {
          const size_t nb = (size_t)((length[(size_t)r] + g.B - 1) / g.B);
          if ((int)ld.size() < 2 && need_blocks + nb <= room) { ld.push_back(r); need_blocks += nb; }
        }
        if (ld.empty()) continue;
        std::vector<uint64_t> ids2;
        std::vector<int32_t> off2, blk2, tok2;
        csr(ev, ids, off, blk, tok);
        size_t used = 0;
        for (int r : ld) {
          const size_t nb = (size_t)((length[(size_t)r] + g.B - 1) / g.B);
          for (size_t q = 0; q < nb; q++) {
            if (used < avail.size()) table[(size_t)r].push_back(avail[used++]);
            else { table[(size_t)r].push_back(free_list.back()); free_list.pop_back(); }
          }
        }
        csr(ld, ids2, off2, blk2, tok2);
        const bool keep = rnd(0, 9) < 7;
        const uint32_t fl = keep ? KV_KEEP_STAGING : 0;
        int rc_ora = ora_swap_out(ora, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data());
        if (rc_ora == 0) rc_ora = ora_swap_in(ora, (int32_t)ids2.size(), ids2.data(), off2.data(), blk2.data(), fl);
        both(LIB_ASYNC(kv_evict_and_load(kp, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data(), (int32_t)ids2.size(),
                                   ids2.data(), off2.data(), blk2.data(), fl, after_model)),
             rc_ora, "evict and load", chunk, step);
        for (int r : ev) { table[(size_t)r].clear(); state[(size_t)r] = 2; }
        free_list.insert(free_list.end(), avail.begin() + (long)used, avail.end());  // what the load did not take
        for (int r : ld) {
          state[(size_t)r] = 1;
          if (!keep && (rnd(0, 9) < 4 || !reserve(r, cap[(size_t)r], "re-reserve", chunk, step))) {
            give_up(r);
            length[(size_t)r] = 0; state[(size_t)r] = 0;
          }
        }
      } else if (op == 8 && !running.empty()) {  // compaction move
        const int r = running[(size_t)rnd(0, (int64_t)running.size() - 1)];
        const size_t k = std::min<size_t>({table[(size_t)r].size(), free_list.size(), (size_t)rnd(1, 4)});
        if (!k) continue;
        std::vector<int32_t> src(table[(size_t)r].begin(), table[(size_t)r].begin() + (long)k), dst;
        for (size_t j = 0; j < k; j++) { dst.push_back(free_list.back()); free_list.pop_back(); }
        if (rnd(0, 1)) {
          // the entry point for callers that cannot allocate: same result, and the HIP runtime is asked for no memory,
          // event or stream while it runs (the stand-in's own queues use the host heap, so that is not counted)
          const long res0 = mockhip::resource_calls();
          both(LIB_ASYNC(kv_move_blocks_noalloc(kp, (int64_t)k, src.data(), dst.data(), after_model)),
               ora_move_blocks(ora, (int64_t)k, src.data(), dst.data()), "move without allocation", chunk, step);
          if (mockhip::resource_calls() != res0) die("kv_move_blocks_noalloc allocated", chunk, step);
        } else
        both(LIB_ASYNC(kv_move_blocks(kp, (int64_t)k, src.data(), dst.data(), after_model)), ora_move_blocks(ora, (int64_t)k, src.data(), dst.data()),
             "move", chunk, step);
        std::copy(dst.begin(), dst.end(), table[(size_t)r].begin());
        free_list.insert(free_list.end(), src.begin(), src.end());
      } else if (op == 9 && running.size() + out.size() > 0) {  // finish
        std::vector<int> live(running);
        live.insert(live.end(), out.begin(), out.end());
        const int r = live[(size_t)rnd(0, (int64_t)live.size() - 1)];
        give_up(r);
        length[(size_t)r] = 0; state[(size_t)r] = 0;
        both(LIB(kv_req_release(kp, (uint64_t)r)), ora_req_release(ora, (uint64_t)r), "release", chunk, step);
      } else if (op == 11 && !running.empty()) {  // the write queue: post every running request, drain under a budget
        std::vector<int> with;
        for (int r : running)
          if (!table[(size_t)r].empty()) with.push_back(r);
        if (with.empty()) continue;
        std::shuffle(with.begin(), with.end(), rng);
        csr(with, ids, off, blk, tok);
        std::vector<double> prio(with.size());
        for (auto& x : prio) x = (double)rnd(0, 3);  // few levels: ties keep the order of the post
        both(LIB_ASYNC(kv_wq_post(kp, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data(), prio.data())), 0, "wq_post", chunk, step);
        // what the queue promises: the same as one delta over the posted requests, highest priority first
        std::vector<int> order(with.size());
        for (size_t i = 0; i < order.size(); i++) order[i] = (int)i;
        std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return prio[(size_t)a] > prio[(size_t)b]; });
        std::vector<int> sorted;
        for (int i : order) sorted.push_back(with[(size_t)i]);
        csr(sorted, ids, off, blk, tok);
        std::vector<int32_t> ma(sorted.size(), 0);
        int64_t written = -1, pending = -1, used = -1, expect = 0;
        if (rnd(0, 3) == 0) {
          // budget from a time interval: the library derives it from its own rate estimates and says what it used
          const int rc = LIB_ASYNC(kv_wq_drain(kp, (double)rnd(1, 3000), 0, 0, &written, &pending, &used, nullptr));
          if ((rc == KV_EHIP && mockhip::failure_fired()) || (rc == KV_ENOMEM && g_new_fired)) throw Failed{rc};
          if (rc != KV_OK || used < 0) die("timed wq_drain", chunk, step);
          calls++;
          if (used == 0) {  // the interval is shorter than the fixed cost of a call: nothing may have moved
            if (written != 0) die("timed wq_drain: moved blocks without a budget", chunk, step);
            continue;
          }
          if (ora_swap_out_delta(ora, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data(), used, 0, ma.data()) != 0)
            die("timed wq_drain: oracle", chunk, step);
        } else {
          const int64_t budget = rnd(1, 6);
          both(LIB_ASYNC(kv_wq_drain(kp, 0.0, budget, 0, &written, &pending, &used, nullptr)),
               ora_swap_out_delta(ora, (int32_t)ids.size(), ids.data(), off.data(), blk.data(), tok.data(), budget, 0, ma.data()),
               "wq_drain", chunk, step);
          if (used != budget) die("wq_drain: budget", chunk, step);
        }
        for (int32_t m : ma) expect += m;
        if (written != expect) die("wq_drain: blocks written", chunk, step);
      } else if (op == 13 && !running.empty() && !hipfail && !nomem) {
        // The model overwrites a chunk of a request's last block on its own stream, after whatever the swap streams
        // still do; the write-through that follows names the model's event and must carry the new bytes.
        std::shuffle(running.begin(), running.end(), rng);
        const int r = running[0];
        if (table[(size_t)r].empty()) continue;
        const int32_t b = table[(size_t)r].back();
        const int l = (int)rnd(0, g.L - 1), c = (int)rnd(0, 1);
        const size_t at = (size_t)(l * g.ls + c * g.ks + (int64_t)b * g.bs);
        std::vector<uint8_t> fresh((size_t)g.chunk);
        for (auto& x : fresh) x = (uint8_t)rng();
        std::memcpy(pool_a.data() + at, fresh.data(), fresh.size());  // the oracle's pool has it at once
        hipEventRecord(ev_evict, evict);
        hipEventRecord(ev_load, load);
        hipStreamWaitEvent(compute, ev_evict, 0);
        hipStreamWaitEvent(compute, ev_load, 0);
        uint8_t* dst = pool_b + at;
        mockhip::enqueue(compute, [dst, fresh]() { std::memcpy(dst, fresh.data(), fresh.size()); });
        hipEventRecord(ev_compute, compute);
        after_model = ev_compute;
        csr({r}, ids, off, blk, tok);
        std::vector<int32_t> ma(1), mb(1);
        both(LIB_ASYNC(kv_swap_out_delta(kp, 1, ids.data(), off.data(), blk.data(), tok.data(), 0, KV_DELTA_INCLUDE_TAIL, mb.data(), ev_compute)),
             ora_swap_out_delta(ora, 1, ids.data(), off.data(), blk.data(), tok.data(), 0, KV_DELTA_INCLUDE_TAIL, ma.data()),
             "delta after the model", chunk, step);
        if (ma != mb) die("blocks_moved", chunk, step);
      } else if (op == 12) {  // calls that must be refused, with the same code on both sides and nothing changed
        auto same = [&](int rc_lib, int rc_ora, const char* what) {
          if ((rc_lib == KV_EHIP && mockhip::failure_fired()) || (rc_lib == KV_ENOMEM && g_new_fired)) throw Failed{rc_lib};
          if (rc_lib != rc_ora || rc_lib == 0) {
            std::fprintf(stderr, "%s: library %d oracle %d\n", what, rc_lib, rc_ora);
            die("refusal", chunk, step);
          }
          calls++;
        };
        const int which = (int)rnd(0, 4);
        if (which == 4) {  // more blocks than the allocation-free move takes in one call: refused before anything is looked at
          static std::vector<int32_t> many((size_t)KV_NOALLOC_MAX_BLOCKS + 1, 0);
          const int rc = LIB(kv_move_blocks_noalloc(kp, (int64_t)many.size(), many.data(), many.data(), nullptr));
          if ((rc == KV_EHIP && mockhip::failure_fired()) || (rc == KV_ENOMEM && g_new_fired)) throw Failed{rc};
          if (rc != KV_E2BIG) die("kv_move_blocks_noalloc accepted more blocks than its array holds", chunk, step);
          calls++;
        }
        if (which == 0 && !out.empty() && length[(size_t)out[0]] > g.B && free_list.size() > 4) {  // one destination twice
          const int r = out[0];
          const size_t nb = (size_t)((length[(size_t)r] + g.B - 1) / g.B);
          std::vector<int32_t> dst(nb, free_list.back());
          uint64_t id = (uint64_t)r;
          int32_t o2[2] = {0, (int32_t)nb};
          same(LIB_ASYNC(kv_swap_in(kp, 1, &id, o2, dst.data(), 0, nullptr)), ora_swap_in(ora, 1, &id, o2, dst.data(), 0), "duplicate destination");
        } else if (which == 1 && !running.empty() && !table[(size_t)running[0]].empty()) {  // a block id outside the pool
          const int r = running[0];
          csr({r}, ids, off, blk, tok);
          blk.back() = (int32_t)g.N;
          same(LIB_ASYNC(kv_swap_out(kp, 1, ids.data(), off.data(), blk.data(), tok.data(), nullptr)),
               ora_swap_out(ora, 1, ids.data(), off.data(), blk.data(), tok.data()), "block id out of range");
        } else if (which == 2 && free_list.size() > 2) {  // resuming a request nobody has heard of
          uint64_t id = 999;
          int32_t o2[2] = {0, 1}, dst[1] = {free_list.back()};
          same(LIB_ASYNC(kv_swap_in(kp, 1, &id, o2, dst, 0, nullptr)), ora_swap_in(ora, 1, &id, o2, dst, 0), "swap-in of an unknown request");
        } else if (which == 3 && !out.empty()) {  // writing through what is out
          const int r = out[0];
          int64_t o = 0;
          int32_t c = 0, st = 0, w = 0, sw = 0;
          if (ora_req_query(ora, (uint64_t)r, &o, &c, &st, &w, &sw) != 0 || !sw) continue;  // preempted warm: a delta is still legal
          const size_t nb = (size_t)((length[(size_t)r] + g.B - 1) / g.B);
          std::vector<int32_t> src(nb, 0);
          uint64_t id = (uint64_t)r;
          int32_t o2[2] = {0, (int32_t)nb}, t2[1] = {length[(size_t)r]}, ma[1], mb[1];
          same(LIB_ASYNC(kv_swap_out_delta(kp, 1, &id, o2, src.data(), t2, 0, 0, mb, nullptr)),
               ora_swap_out_delta(ora, 1, &id, o2, src.data(), t2, 0, 0, ma), "delta of a swapped-out request");
        }
      } else if (op == 10 && events && !running.empty()) {  // a control thread's poll: must not disturb anything
        const int rc = LIB(kv_req_poll(kp, (uint64_t)running[0]));
        if ((rc == KV_EHIP && mockhip::failure_fired()) || (rc == KV_ENOMEM && g_new_fired)) throw Failed{rc};
        if (rc != 0 && rc != 1) die("kv_req_poll", chunk, step);
      }
    }
    if (poller) {
      while (polls.load() < 50) std::this_thread::yield();  // the reader has really run beside the history
      stop = true;
      side.join();
    }
    {
      const int rc = LIB(kv_sync(kp));
      if ((rc == KV_EHIP && mockhip::failure_fired()) || (rc == KV_ENOMEM && g_new_fired)) throw Failed{rc};
      if (rc != KV_OK) die("kv_sync", chunk, -1);
    }
    mockhip::fail_after(0, 0);  // an armed failure that this chunk did not reach stays unused
    g_new_fail_in = 0;
    hipStreamSynchronize(compute);
    if (std::memcmp(pool_a.data(), pool_b, pool_bytes)) {
      size_t at = 0;
      while (pool_a[at] == pool_b[at]) at++;
      const int64_t l = (int64_t)at / g.ls, c = ((int64_t)at % g.ls) / g.ks, b = (((int64_t)at % g.ls) % g.ks) / g.bs;
      std::fprintf(stderr, "first difference at byte %zu: layer %lld, %s, block %lld\n", at, (long long)l, c ? "V" : "K", (long long)b);
      die("pool bytes", chunk, -1);
    }
    if (std::memcmp(stag_a.data(), stag_b, stag_bytes)) die("arena bytes", chunk, -1);
    if (scales && std::memcmp(scale_a.data(), scale_b, scale_bytes)) die("scale bytes", chunk, -1);
    free_list.insert(free_list.end(), held.begin(), held.end());
    for (int r = 1; r <= R; r++) {
      int64_t oa = -1, ob = -1;
      int32_t ca = -1, sa = -1, wa = -1, xa = -1, cb = -1, sb = -1, wb = -1, xb = -1;
      const int qa = ora_req_query(ora, (uint64_t)r, &oa, &ca, &sa, &wa, &xa);
      const int qb = kv_req_query(kp, (uint64_t)r, &ob, &cb, &sb, &wb, &xb);
      if (qa != qb || (qa == 0 && (oa != ob || ca != cb || sa != sb || wa != wb || xa != xb))) die("request state", chunk, r);
    }
  }
  } catch (const Failed& f) {
    // The call in which the failure surfaced has returned KV_EHIP or KV_ENOMEM.  From here on the handle refuses
    // whatever would change state or enqueue work, still answers queries, and can be destroyed.
    handled = true;
    handled_rc = f.rc;
    mockhip::fail_after(0, 0);
    g_new_fail_in = 0;
    if (f.rc == KV_EHIP && kv_last_hip_error(kp) != 999) die("kv_last_hip_error after an injected failure", -1, -1);
    uint64_t id = 1;
    int32_t off1[2] = {0, 1}, blk1[2] = {0, 1}, tok1[1] = {1}, moved1[1];
    int64_t a = 0, b = 0, c = 0;
    if (kv_req_reserve(kp, 1000, 1) != KV_EHIP || kv_req_release(kp, 1) != KV_EHIP ||
        kv_swap_out(kp, 1, &id, off1, blk1, tok1, nullptr) != KV_EHIP ||
        kv_swap_out_delta(kp, 1, &id, off1, blk1, tok1, 0, 0, moved1, nullptr) != KV_EHIP ||
        kv_swap_in(kp, 1, &id, off1, blk1, 0, nullptr) != KV_EHIP || kv_move_blocks(kp, 1, blk1, blk1 + 1, nullptr) != KV_EHIP ||
        kv_move_blocks_noalloc(kp, 1, blk1, blk1 + 1, nullptr) != KV_EHIP ||
        kv_evict_and_load(kp, 1, &id, off1, blk1, tok1, 0, nullptr, nullptr, nullptr, 0, nullptr) != KV_EHIP ||
        kv_wq_post(kp, 1, &id, off1, blk1, tok1, nullptr) != KV_EHIP || kv_wq_drain(kp, 0, 4, 0, &a, &b, &c, nullptr) != KV_EHIP ||
        kv_sync(kp) != KV_EHIP || kv_pool_tune(kp, KV_TUNE_MAX_WGS_LINK, 8) != KV_EHIP)
      die("a call was accepted by a handle that had failed", -1, -1);
    kv_io_stats io;
    int32_t x;
    const int q = kv_req_query(kp, 1, &a, &x, &x, &x, &x);
    if (kv_io_stats_get(kp, &io) != KV_OK || (q != KV_OK && q != KV_ENOENT)) die("queries after a failure", -1, -1);
  }
  if (kv_pool_destroy(kp) != KV_OK) die("kv_pool_destroy", -1, -1);
  ora_destroy(ora);
  hipStreamDestroy(evict);
  hipStreamDestroy(load);
  hipStreamDestroy(compute);
  hipEventDestroy(ev_evict);
  hipEventDestroy(ev_load);
  hipEventDestroy(ev_compute);
  hipFree(pool_b); hipFree(scale_b);
  mode == 2 ? hipFree(stag_b) : hipHostFree(stag_b);
  if (bounce) hipFree(bounce);
  if (handled) {
    std::printf("seed %llu: failure handled: the call returned %d, the handle then refused further work and was destroyed\n",
                (unsigned long long)seed, handled_rc);
    return 0;
  }
  std::printf("seed %llu: %ld calls, %ld device operations, L %d H %d D %d B %d e %d%s mode %d events %d policy %d: equal to the oracle\n",
              (unsigned long long)seed, calls, mockhip::executed_ops(), g.L, g.H, g.D, g.B, g.e, scales ? " +scales" : "", mode,
              (int)events, policy);
  return calls > 40 ? 0 : 2;
}
