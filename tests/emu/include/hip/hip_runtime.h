// CPU stand-in for <hip/hip_runtime.h>, for tests only.
//
// Lets the library's kernel sources be compiled with g++ and stepped on the
// host: every GPU lane is a ucontext fiber, a block's fibers run round-robin
// and switch at each cross-lane operation (ds_bpermute, DPP row shifts,
// ballots) and at block barriers, which is enough to reproduce the lock-step
// semantics of a 64-wide wavefront for convergent code. Device memory is host
// memory followed by an inaccessible guard page, so an access past the end of a
// buffer faults at once. Nothing in the shipped library includes this file; it
// shadows the real header only on the include path of the test build.
#pragma once
#include <stddef.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>
#include <cmath>
#include <functional>

#define __global__
#define __device__
#define __host__
#define __forceinline__ inline
#define __launch_bounds__(...)
#define __shared__ static
#define __align__(n) __attribute__((aligned(n)))
#define HIP_SYMBOL(x) x
#define __builtin_nontemporal_store(v, p) (*(p) = (v))
#define __builtin_nontemporal_load(p) (*(p))

struct dim3 {
  unsigned x, y, z;
  dim3(unsigned x_ = 1, unsigned y_ = 1, unsigned z_ = 1) : x(x_), y(y_), z(z_) {}
};
struct uint4 {
  unsigned x, y, z, w;
};
static inline uint4 make_uint4(unsigned x, unsigned y, unsigned z, unsigned w) {
  uint4 r = {x, y, z, w};
  return r;
}

typedef int hipError_t;
enum { hipSuccess = 0, hipErrorInvalidValue = 1, hipErrorOutOfMemory = 2 };
typedef void* hipStream_t;
enum hipMemcpyKind { hipMemcpyHostToDevice = 1, hipMemcpyDeviceToHost = 2, hipMemcpyDeviceToDevice = 3 };
struct hipDeviceProp_t {
  int multiProcessorCount;
  char name[64];
};

namespace hipemu {
struct LaneState {
  dim3 tid;
  dim3 bid;
  dim3 bdim;
  dim3 gdim;
};
LaneState* current();
void launch(dim3 grid, dim3 block, const std::function<void()>& body);
uint32_t bpermute(int byte_addr, uint32_t v);
uint32_t dpp(uint32_t old, uint32_t src, int ctrl, int row_mask, int bank_mask, bool bound_ctrl);
uint64_t ballot(bool p);
uint32_t readlane(uint32_t v, int src_lane);
void barrier();
void* dev_alloc(size_t bytes);
void dev_free(void* p);
}  // namespace hipemu

#define threadIdx (hipemu::current()->tid)
#define blockIdx (hipemu::current()->bid)
#define blockDim (hipemu::current()->bdim)
#define gridDim (hipemu::current()->gdim)

#define hipLaunchKernelGGL(kernel, grid, block, shmem, stream, ...) \
  ((void)(stream), hipemu::launch((grid), (block), [&]() { kernel(__VA_ARGS__); }))

static inline int __builtin_amdgcn_ds_bpermute(int addr, int v) { return (int)hipemu::bpermute(addr, (uint32_t)v); }
static inline int __builtin_amdgcn_update_dpp(int old, int src, int ctrl, int row_mask, int bank_mask,
                                              bool bound_ctrl) {
  return (int)hipemu::dpp((uint32_t)old, (uint32_t)src, ctrl, row_mask, bank_mask, bound_ctrl);
}
// every lane of an emulated wavefront is active, so the first active lane is lane 0
static inline int __builtin_amdgcn_readfirstlane(int v) { return (int)hipemu::readlane((uint32_t)v, 0); }
static inline int __builtin_amdgcn_readlane(int v, int lane) { return (int)hipemu::readlane((uint32_t)v, lane); }
static inline uint64_t __builtin_amdgcn_ballot_w64(bool p) { return hipemu::ballot(p); }
static inline void __builtin_amdgcn_sched_barrier(int) {}
static inline void __builtin_amdgcn_sched_group_barrier(int, int, int) {}
static inline void __syncthreads() { hipemu::barrier(); }
static inline uint32_t atomicOr(uint32_t* p, uint32_t v) {
  uint32_t o = *p;
  *p = o | v;
  return o;
}
static inline uint32_t atomicMax(uint32_t* p, uint32_t v) {
  uint32_t o = *p;
  if (v > o) *p = v;
  return o;
}
static inline uint32_t atomicAdd(uint32_t* p, uint32_t v) {
  uint32_t o = *p;
  *p = o + v;
  return o;
}

static inline hipError_t hipGetDevice(int* d) {
  *d = 0;
  return hipSuccess;
}
static inline hipError_t hipGetDeviceProperties(hipDeviceProp_t* p, int) {
  memset(p, 0, sizeof(*p));
  p->multiProcessorCount = 1;  // tiny "chip": small batches already exercise the grid-stride loops
  strcpy(p->name, "cpu-emulation");
  return hipSuccess;
}
static inline hipError_t hipMalloc(void** p, size_t bytes) {
  *p = hipemu::dev_alloc(bytes);
  return *p ? hipSuccess : hipErrorOutOfMemory;
}
static inline hipError_t hipFree(void* p) {
  hipemu::dev_free(p);
  return hipSuccess;
}
static inline hipError_t hipMemcpy(void* d, const void* s, size_t n, hipMemcpyKind) {
  memcpy(d, s, n);
  return hipSuccess;
}
static inline hipError_t hipMemcpyAsync(void* d, const void* s, size_t n, hipMemcpyKind, hipStream_t) {
  memcpy(d, s, n);
  return hipSuccess;
}
static inline hipError_t hipMemsetAsync(void* d, int v, size_t n, hipStream_t) {
  memset(d, v, n);
  return hipSuccess;
}
static inline hipError_t hipGetSymbolAddress(void** p, const void* symbol) {
  *p = (void*)symbol;  // the emulated "device" array is the host array itself
  return hipSuccess;
}
static inline hipError_t hipDeviceSynchronize() { return hipSuccess; }
// host staging: everything is synchronous in the emulation, events and streams are placeholders
typedef void* hipEvent_t;
enum { hipHostMallocDefault = 0, hipStreamNonBlocking = 1, hipEventDisableTiming = 2 };
static inline hipError_t hipHostMalloc(void** p, size_t bytes, unsigned) {
  *p = malloc(bytes ? bytes : 1);
  return *p ? hipSuccess : hipErrorOutOfMemory;
}
static inline hipError_t hipHostFree(void* p) {
  free(p);
  return hipSuccess;
}
static inline hipError_t hipStreamCreateWithFlags(hipStream_t* s, unsigned) {
  *s = (hipStream_t)1;
  return hipSuccess;
}
static inline hipError_t hipStreamDestroy(hipStream_t) { return hipSuccess; }
static inline hipError_t hipStreamSynchronize(hipStream_t) { return hipSuccess; }
static inline hipError_t hipStreamWaitEvent(hipStream_t, hipEvent_t, unsigned) { return hipSuccess; }
static inline hipError_t hipEventCreateWithFlags(hipEvent_t* e, unsigned) {
  *e = (hipEvent_t)1;
  return hipSuccess;
}
static inline hipError_t hipEventDestroy(hipEvent_t) { return hipSuccess; }
static inline hipError_t hipEventRecord(hipEvent_t, hipStream_t) { return hipSuccess; }
static inline hipError_t hipEventSynchronize(hipEvent_t) { return hipSuccess; }
static inline hipError_t hipGetLastError() { return hipSuccess; }
static inline const char* hipGetErrorString(hipError_t) { return "emulated"; }
