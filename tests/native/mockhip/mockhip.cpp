// Implementation of the host-only HIP stand-in (see hip/hip_runtime.h in this directory).
#include <hip/hip_runtime.h>

#include <cstdio>
#include <deque>
#include <map>
#include <mutex>
#include <random>
#include <vector>

unsigned int lds[16384];  // "extern __shared__ unsigned int lds[]" of the kernel source

namespace mockhip {

Idx threadIdx_, blockIdx_, gridDim_, blockDim_;

struct Event {
  uint64_t recorded = 0;   // generation of the latest hipEventRecord
  uint64_t completed = 0;  // newest generation whose record operation has executed
  double t = 0;            // clock value when that happened
};
struct Op {
  int kind;  // 0 function, 1 record, 2 wait
  std::function<void()> fn;
  Event* ev;
  uint64_t gen;
};
struct Stream {
  std::deque<Op> q;
};
struct Alloc {
  size_t size;
  int type;
};

static std::vector<Stream*> streams;
static std::map<char*, Alloc> allocs;
static std::mt19937_64 rng(1);
static int policy = kRandom;
static Stream* starved = nullptr;
static double clock_ms = 0;
static long n_exec = 0, n_deadlock = 0;
static hipError_t last_error = hipSuccess;
static Stream null_stream;
// One lock around the whole stand-in: the program under test may call from several threads.  A blocking wait
// takes it once per step of the "GPU", so that other threads get in between the steps as they would on hardware.
static std::recursive_mutex api_mu;
#define API_LOCK std::lock_guard<std::recursive_mutex> api_guard(api_mu)

static long fail_in = 0;
static int fail_code = 0;
static bool fail_fired = false;

static Stream* S(hipStream_t s) { return s ? s : &null_stream; }

// true when this call is the one chosen to fail
static bool injected() {
  if (fail_in <= 0 || --fail_in > 0) return false;
  fail_fired = true;
  last_error = fail_code;
  return true;
}

static bool runnable(Stream* s) {
  if (s->q.empty()) return false;
  const Op& o = s->q.front();
  return o.kind != 2 || o.ev->completed >= o.gen;
}

static void run_head(Stream* s) {
  Op o = std::move(s->q.front());
  s->q.pop_front();
  clock_ms += 0.001;
  n_exec++;
  if (o.kind == 0) {
    o.fn();
  } else if (o.kind == 1) {
    if (o.gen > o.ev->completed) {
      o.ev->completed = o.gen;
      o.ev->t = clock_ms;
    }
  }
}

// one step of the "GPU": false when nothing can run
static bool step() {
  std::vector<Stream*> ready, preferred;
  std::vector<Stream*> all = streams;
  all.push_back(&null_stream);
  for (Stream* s : all)
    if (runnable(s)) {
      ready.push_back(s);
      if (s != starved) preferred.push_back(s);
    }
  if (ready.empty()) return false;
  std::vector<Stream*>& pick = (policy == kStarve0 || policy == kStarve1) && !preferred.empty() ? preferred : ready;
  run_head(pick[(size_t)(rng() % pick.size())]);
  return true;
}

template <class Pred>
static void drive(Pred done) {
  for (;;) {
    API_LOCK;
    if (done()) return;
    if (!step()) {
      n_deadlock++;
      std::fprintf(stderr, "mockhip: DEADLOCK: a wait can never be satisfied\n");
      std::abort();
    }
  }
}

// after an enqueueing call the device makes some progress, or none
static void progress() {
  int k = 0;
  if (policy == kRandom) k = (int)(rng() % 4);
  if (policy == kStarve0 || policy == kStarve1) k = (int)(rng() % 3);
  for (int i = 0; i < k; i++)
    if (!step()) break;
}

void reset(uint64_t seed) {
  API_LOCK;
  rng.seed(seed);
  policy = kRandom;
  starved = nullptr;
}
void set_policy(int p, Stream* s) {
  API_LOCK;
  policy = p;
  starved = s;
}
static void push_fn(Stream* s, std::function<void()> fn) {
  S(s)->q.push_back({0, std::move(fn), nullptr, 0});
  progress();
}
void enqueue(Stream* s, std::function<void()> fn) {
  API_LOCK;
  if (injected()) return;  // a failed launch: hipGetLastError() reports it
  push_fn(s, std::move(fn));
}
void fail_after(long n, int code) {
  API_LOCK;
  fail_in = n;
  fail_code = code;
  fail_fired = false;
}
bool failure_fired() {
  API_LOCK;
  return fail_fired;
}
long executed_ops() {
  API_LOCK;
  return n_exec;
}
long deadlocks() {
  API_LOCK;
  return n_deadlock;
}

}  // namespace mockhip

using namespace mockhip;

hipError_t hipGetLastError() {
  API_LOCK;
  hipError_t e = last_error;
  last_error = hipSuccess;
  return e;
}
hipError_t hipGetDevice(int* dev) { *dev = 0; return hipSuccess; }
hipError_t hipGetDeviceProperties(hipDeviceProp_t* prop, int) { prop->multiProcessorCount = 256; return hipSuccess; }

static hipError_t alloc_any(void** p, size_t n, int type) {
  API_LOCK;
  char* m = (char*)std::malloc(n ? n : 1);
  if (!m) return last_error = hipErrorOutOfMemory;
  std::memset(m, 0xCD, n);
  allocs[m] = {n, type};
  *p = m;
  return hipSuccess;
}
static hipError_t free_any(void* p) {
  API_LOCK;
  auto it = allocs.find((char*)p);
  if (it == allocs.end()) return last_error = hipErrorInvalidValue;
  allocs.erase(it);
  std::free(p);
  return hipSuccess;
}
hipError_t hipMalloc(void** p, size_t n) { return alloc_any(p, n, hipMemoryTypeDevice); }
hipError_t hipFree(void* p) { return free_any(p); }
hipError_t hipHostMalloc(void** p, size_t n, unsigned) { return alloc_any(p, n, hipMemoryTypeHost); }
hipError_t hipHostFree(void* p) { return free_any(p); }

static const std::pair<char* const, Alloc>* find_alloc(const void* p) {
  auto it = allocs.upper_bound((char*)p);
  if (it == allocs.begin()) return nullptr;
  --it;
  if ((const char*)p >= it->first + it->second.size && !((const char*)p == it->first)) return nullptr;
  return &*it;
}
hipError_t hipMemGetAddressRange(hipDeviceptr_t* base, size_t* size, hipDeviceptr_t p) {
  API_LOCK;
  auto* a = find_alloc(p);
  if (!a) return last_error = hipErrorInvalidValue;
  *base = a->first;
  *size = a->second.size;
  return hipSuccess;
}
hipError_t hipPointerGetAttributes(hipPointerAttribute_t* at, const void* p) {
  API_LOCK;
  auto* a = find_alloc(p);
  if (!a) return last_error = hipErrorInvalidValue;
  at->type = a->second.type;
  at->devicePointer = (void*)p;
  at->hostPointer = a->second.type == hipMemoryTypeHost ? (void*)p : nullptr;
  return hipSuccess;
}

hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) {
  API_LOCK;
  *s = new Stream;
  streams.push_back(*s);
  return hipSuccess;
}
hipError_t hipStreamDestroy(hipStream_t s) {
  API_LOCK;
  drive([&] { return s->q.empty(); });
  for (size_t i = 0; i < streams.size(); i++)
    if (streams[i] == s) streams.erase(streams.begin() + (long)i);
  if (starved == s) starved = nullptr;
  delete s;
  return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t s) {
  {
    API_LOCK;
    if (injected()) return fail_code;
  }
  Stream* st = S(s);
  drive([&] { return st->q.empty(); });
  return hipSuccess;
}
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned) {
  API_LOCK;
  if (injected()) return fail_code;
  if (e->recorded == 0) return hipSuccess;  // never recorded: nothing to wait for
  S(s)->q.push_back({2, nullptr, e, e->recorded});
  progress();
  return hipSuccess;
}
hipError_t hipEventCreate(hipEvent_t* e) {
  API_LOCK;
  if (injected()) return fail_code;
  *e = new Event;
  return hipSuccess;
}
hipError_t hipEventDestroy(hipEvent_t e) {
  API_LOCK;
  // operations that still name the event are a use after free in the program under test
  for (Stream* s : streams)
    for (Op& o : s->q)
      if (o.ev == e) {
        std::fprintf(stderr, "mockhip: event destroyed while a queued operation uses it\n");
        std::abort();
      }
  delete e;
  return hipSuccess;
}
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s) {
  API_LOCK;
  if (injected()) return fail_code;
  e->recorded++;
  S(s)->q.push_back({1, nullptr, e, e->recorded});
  progress();
  return hipSuccess;
}
hipError_t hipEventQuery(hipEvent_t e) {
  API_LOCK;
  if (injected()) return fail_code;
  return e->completed >= e->recorded ? hipSuccess : hipErrorNotReady;
}
hipError_t hipEventSynchronize(hipEvent_t e) {
  uint64_t gen;
  {
    API_LOCK;
    if (injected()) return fail_code;
    gen = e->recorded;
  }
  drive([&] { return e->completed >= gen; });
  return hipSuccess;
}
hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b) {
  API_LOCK;
  if (a->completed < a->recorded || b->completed < b->recorded || !a->recorded || !b->recorded)
    return last_error = hipErrorNotReady;
  *ms = (float)(b->t - a->t);
  return hipSuccess;
}
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind, hipStream_t s) {
  API_LOCK;
  if (injected()) return fail_code;
  push_fn(s, [=]() { std::memcpy(dst, src, n); });
  return hipSuccess;
}
