// Implementation of the host-only HIP stand-in (see hip/hip_runtime.h in this directory).
#include <atomic>
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
  if (std::getenv("MOCKHIP_TRACE")) std::fprintf(stderr, "mockhip: injected failure fires now\n");
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
static std::atomic<long> n_resource{0};
long resource_calls() { return n_resource.load(); }
static thread_local long n_host_waits = 0;
long host_waits() { return n_host_waits; }

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
  n_resource++;
  char* m = (char*)std::malloc(n ? n : 1);
  if (!m) return last_error = hipErrorOutOfMemory;
  std::memset(m, 0xCD, n);
  allocs[m] = {n, type};
  *p = m;
  return hipSuccess;
}
static hipError_t free_any(void* p) {
  API_LOCK;
  n_resource++;
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
  at->device = 0;
  at->devicePointer = (void*)p;
  at->hostPointer = a->second.type == hipMemoryTypeHost ? (void*)p : nullptr;
  return hipSuccess;
}

hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) {
  API_LOCK;
  n_resource++;
  *s = new Stream;
  streams.push_back(*s);
  return hipSuccess;
}
hipError_t hipStreamDestroy(hipStream_t s) {
  API_LOCK;
  n_resource++;
  drive([&] { return s->q.empty(); });
  for (size_t i = 0; i < streams.size(); i++)
    if (streams[i] == s) streams.erase(streams.begin() + (long)i);
  if (starved == s) starved = nullptr;
  delete s;
  return hipSuccess;
}
hipError_t hipStreamSynchronize(hipStream_t s) {
  n_host_waits++;
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
  n_resource++;
  if (injected()) return fail_code;
  *e = new Event;
  return hipSuccess;
}
hipError_t hipEventDestroy(hipEvent_t e) {
  API_LOCK;
  n_resource++;
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
  n_host_waits++;
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

// ---- workgroups with barriers: one fiber per lane ----
#if defined(__has_feature)
#if __has_feature(address_sanitizer)
#define MOCKHIP_ASAN 1
#include <sanitizer/common_interface_defs.h>
#endif
#if __has_feature(thread_sanitizer)
#define MOCKHIP_TSAN 1
#endif
#endif

#if defined(__x86_64__) && !defined(MOCKHIP_TSAN)
#define MOCKHIP_FIBERS 1
// Switch of stacks without a system call (swapcontext saves the signal mask on every switch, which makes a
// launch of some thousand workgroups take seconds): the callee-saved registers go onto the old stack, the
// stack pointers are exchanged, the registers of the new stack come back.
extern "C" void mockhip_switch(void** save_sp, void* new_sp);
asm(R"(
  .text
  .globl mockhip_switch
  .type mockhip_switch,@function
mockhip_switch:
  pushq %rbp
  pushq %rbx
  pushq %r12
  pushq %r13
  pushq %r14
  pushq %r15
  movq %rsp, (%rdi)
  movq %rsi, %rsp
  popq %r15
  popq %r14
  popq %r13
  popq %r12
  popq %rbx
  popq %rbp
  ret
  .size mockhip_switch, .-mockhip_switch
)");
#endif

namespace mockhip {
namespace {

constexpr size_t kLaneStack = 128 << 10;
struct Fibers {
  std::vector<void*> sp;   // saved stack pointer of each parked lane
  std::vector<char*> stack;
  std::vector<int> state;  // 0 runnable, 1 parked at the barrier, 2 finished
  void* sched_sp = nullptr;
  const void* sched_bottom = nullptr;
  size_t sched_size = 0;
  int cur = -1;
  const std::function<void()>* body = nullptr;
  ~Fibers() {
    for (char* p : stack) std::free(p);
  }
};
Fibers fb;

#ifdef MOCKHIP_FIBERS
// The sanitizer has to be told about every change of stack, or it takes the fiber's frames for garbage.
void leave(void** save, const void* bottom, size_t size) {
#ifdef MOCKHIP_ASAN
  __sanitizer_start_switch_fiber(save, bottom, size);
#else
  (void)save; (void)bottom; (void)size;
#endif
}
void arrive(void* save, const void** old_bottom, size_t* old_size) {
#ifdef MOCKHIP_ASAN
  __sanitizer_finish_switch_fiber(save, old_bottom, old_size);
#else
  (void)save; (void)old_bottom; (void)old_size;
#endif
}

[[noreturn]] void lane_main() {
  arrive(nullptr, &fb.sched_bottom, &fb.sched_size);
  (*fb.body)();
  fb.state[(size_t)fb.cur] = 2;
  leave(nullptr, fb.sched_bottom, fb.sched_size);  // nullptr: this fiber's frames are gone for good
  mockhip_switch(&fb.sp[(size_t)fb.cur], fb.sched_sp);
  std::abort();  // a finished lane is never resumed
}
#endif

}  // namespace

bool fibers_available() {
#ifdef MOCKHIP_FIBERS
  return true;
#else
  return false;
#endif
}

void barrier() {
#ifdef MOCKHIP_FIBERS
  if (fb.cur < 0) return;  // a launch without LDS: lanes run one after the other and its kernels have no barrier
  const int me = fb.cur;
  fb.state[(size_t)me] = 1;
  void* save = nullptr;
  leave(&save, fb.sched_bottom, fb.sched_size);
  mockhip_switch(&fb.sp[(size_t)me], fb.sched_sp);
  arrive(save, nullptr, nullptr);
#endif
}

void run_grid(dim3 g, dim3 b, size_t lds_bytes, const std::function<void()>& lane) {
  gridDim_ = {g.x, g.y, g.z};
  blockDim_ = {b.x, b.y, b.z};
  if (lds_bytes == 0) {
    for (unsigned bx = 0; bx < g.x; bx++)
      for (unsigned tx = 0; tx < b.x; tx++) {
        blockIdx_ = {bx, 0, 0};
        threadIdx_ = {tx, 0, 0};
        lane();
      }
    return;
  }
  if (!fibers_available() || lds_bytes > sizeof(lds)) {
    std::fprintf(stderr, "mockhip: a launch with %zu bytes of LDS cannot be emulated in this build\n", lds_bytes);
    std::abort();
  }
#ifdef MOCKHIP_FIBERS
  const size_t n = b.x;
  if (fb.stack.size() < n) {
    fb.sp.resize(n);
    fb.state.resize(n);
    fb.stack.reserve(n);  // first, so that a push_back that cannot allocate does not drop a stack it was just handed
    while (fb.stack.size() < n) fb.stack.push_back((char*)std::malloc(kLaneStack));  // reused by every later launch
  }
  fb.body = &lane;
  for (unsigned bx = 0; bx < g.x; bx++) {
    for (size_t t = 0; t < n; t++) {
      // a fresh stack: six register slots, the entry point, and the slot a caller's return address would take
      void** top = (void**)(((uintptr_t)fb.stack[t] + kLaneStack) & ~(uintptr_t)15);
      top[-1] = nullptr;
      top[-2] = (void*)&lane_main;
      for (int i = 3; i <= 8; i++) top[-i] = nullptr;
      fb.sp[t] = (void*)(top - 8);
      fb.state[t] = 0;
    }
    for (;;) {
      size_t done = 0, parked = 0;
      for (size_t t = 0; t < n; t++) {
        if (fb.state[t] != 0) continue;
        fb.cur = (int)t;
        threadIdx_ = {(unsigned)t, 0, 0};
        blockIdx_ = {bx, 0, 0};
        void* save = nullptr;
        leave(&save, fb.stack[t], kLaneStack);
        mockhip_switch(&fb.sched_sp, fb.sp[t]);
        arrive(save, nullptr, nullptr);
      }
      fb.cur = -1;
      for (size_t t = 0; t < n; t++) {
        done += fb.state[t] == 2;
        parked += fb.state[t] == 1;
      }
      if (done == n) break;
      if (parked + done != n || done != 0) {
        std::fprintf(stderr, "mockhip: a barrier was reached by %zu of %zu lanes of workgroup %u\n", parked, n, bx);
        std::abort();
      }
      for (size_t t = 0; t < n; t++) fb.state[t] = 0;  // everybody has arrived: on to the next phase
    }
  }
#endif
}

}  // namespace mockhip
