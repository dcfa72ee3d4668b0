// A host-only stand-in for the part of the HIP runtime that the swap library uses, for CPU tests.
//
// It lets the REAL host runtime (runtime.hip.inc, kvswap.hip) and the REAL kernel source (kernels.hip.inc)
// be compiled by a host compiler and run on the CPU: streams are in-order queues of operations, events carry
// the generation they were last recorded with, hipStreamWaitEvent captures the generation at the time of the
// call, copies read their source when they EXECUTE (as a copy engine does), and a kernel launch runs the kernel
// body once per (workgroup, lane) with threadIdx / blockIdx set.  Nothing executes when it is enqueued: an
// executor picks, among the streams whose head operation may run, one according to a policy chosen by the test
// (random, or always starving one stream), so the test decides how far the "GPU" lags behind the host and which
// stream runs ahead.  "Device" and "pinned" memory are plain malloc blocks, so AddressSanitizer checks every
// access the kernels make.  Launches that ask for dynamic LDS run the lanes of a workgroup as fibers, so that
// __syncthreads() is a real barrier and data exchanged through LDS is emulated too (see run_grid below).
#pragma once
#include <cstddef>
#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <functional>

typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorOutOfMemory = 2, hipErrorNotReady = 600 };
enum { hipStreamNonBlocking = 1 };
enum { hipHostMallocDefault = 0 };
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2, hipMemcpyDeviceToDevice = 3 };
enum hipMemoryType { hipMemoryTypeHost = 1, hipMemoryTypeDevice = 2 };
typedef void* hipDeviceptr_t;
struct hipPointerAttribute_t { int type; int device; void* devicePointer; void* hostPointer; };
struct hipDeviceProp_t { int multiProcessorCount; };
struct dim3 { unsigned x, y, z; dim3(unsigned a = 1, unsigned b = 1, unsigned c = 1) : x(a), y(b), z(c) {} };

namespace mockhip {
struct Stream;
struct Event;
struct Idx { unsigned x, y, z; };
extern Idx threadIdx_, blockIdx_, gridDim_, blockDim_;
enum Policy { kRandom = 0, kStarve0 = 1, kStarve1 = 2, kLazy = 3 };
// test control
void reset(uint64_t seed);
void set_policy(int policy, Stream* starved);
void enqueue(Stream* s, std::function<void()> fn);
long executed_ops();
long deadlocks();
// Calls so far that take or give back a resource on a real device: hipMalloc, hipHostMalloc, hipFree, hipHostFree,
// event and stream creation and destruction.  An entry point that promises not to allocate leaves it unchanged.
long resource_calls();
// Calls of the CURRENT THREAD so far that block the host until device work has finished (hipStreamSynchronize,
// hipEventSynchronize): an entry point that promises to be asynchronous leaves it unchanged.
long host_waits();
// Failure injection: the n-th call from now, counted over the calls that can fail on a real device (event
// creation, record, wait, query and synchronisation, stream synchronisation, copies, kernel launches), returns
// `code` and does nothing else; n <= 0 disarms.  failure_fired() tells whether it has happened.
void fail_after(long n, int code);
bool failure_fired();
// Runs `lane` once per (workgroup, lane) of the grid with threadIdx / blockIdx set.  A launch without dynamic
// LDS runs its lanes to completion one after the other (its kernels have no barrier on that path).  A launch
// WITH dynamic LDS runs the lanes of a workgroup as fibers: __syncthreads() parks a lane until every lane of
// the workgroup has arrived, as on the device; a barrier that only some lanes reach aborts the program.
void run_grid(dim3 grid, dim3 block, size_t lds_bytes, const std::function<void()>& lane);
void barrier();
bool fibers_available();  // false in a ThreadSanitizer build: launches with LDS must then be avoided
}  // namespace mockhip

typedef mockhip::Stream* hipStream_t;
typedef mockhip::Event* hipEvent_t;

#define threadIdx mockhip::threadIdx_
#define blockIdx mockhip::blockIdx_
#define gridDim mockhip::gridDim_
#define blockDim mockhip::blockDim_
#define __global__
#define __device__
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) x
#define __launch_bounds__(n)
#define __shared__
#define __restrict__
inline void __syncthreads() { mockhip::barrier(); }

hipError_t hipGetLastError();
hipError_t hipGetDevice(int* dev);
hipError_t hipGetDeviceProperties(hipDeviceProp_t* prop, int dev);
hipError_t hipMalloc(void** p, size_t n);
hipError_t hipFree(void* p);
hipError_t hipHostMalloc(void** p, size_t n, unsigned flags);
hipError_t hipHostFree(void* p);
hipError_t hipMemGetAddressRange(hipDeviceptr_t* base, size_t* size, hipDeviceptr_t p);
hipError_t hipPointerGetAttributes(hipPointerAttribute_t* at, const void* p);
hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned flags);
hipError_t hipStreamDestroy(hipStream_t s);
hipError_t hipStreamSynchronize(hipStream_t s);
hipError_t hipStreamWaitEvent(hipStream_t s, hipEvent_t e, unsigned flags);
hipError_t hipEventCreate(hipEvent_t* e);
hipError_t hipEventDestroy(hipEvent_t e);
hipError_t hipEventRecord(hipEvent_t e, hipStream_t s);
hipError_t hipEventQuery(hipEvent_t e);
hipError_t hipEventSynchronize(hipEvent_t e);
hipError_t hipEventElapsedTime(float* ms, hipEvent_t a, hipEvent_t b);
hipError_t hipMemcpyAsync(void* dst, const void* src, size_t n, hipMemcpyKind kind, hipStream_t s);
// A `__device__` variable is an ordinary global here, so its "device address" is its address.
template <class T>
hipError_t hipGetSymbolAddress(void** ptr, const T& symbol) {
  *ptr = (void*)&symbol;
  return hipSuccess;
}

// One kernel launch = one queued operation that runs the body for every lane of every workgroup.
#define hipLaunchKernelGGL(kern, grid, block, lds_bytes, stream, ...)                                   \
  do {                                                                                                  \
    const dim3 g_ = (grid), b_ = (block);                                                               \
    const size_t l_ = (size_t)(lds_bytes);                                                              \
    mockhip::enqueue((stream), [=]() { mockhip::run_grid(g_, b_, l_, [=]() { kern(__VA_ARGS__); }); }); \
  } while (0)
