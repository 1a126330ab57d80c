// Roofline denominators measured on the part itself: issue rates of the candidate multiply
// instructions (no memory traffic, independent accumulator streams) and plain HBM fill / copy / read
// rates. Built into libhaflo_peak.so, a library of its own that the operators never load; bench_peak.py
// drives it and times each launch with HIP events.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/haflo_peak.h"

namespace {

typedef uint32_t u32;
typedef uint64_t u64;

constexpr int kStreams = 16;  // independent accumulators per lane: enough to cover the pipeline latency

__device__ __forceinline__ u32 next_operand(u32 b) {
  b ^= b << 13;
  b ^= b >> 17;
  b ^= b << 5;
  return b;
}

// one 32x32+64 -> 64 multiply-add (v_mad_u64_u32) per stream and iteration
__global__ __launch_bounds__(256) void k_mad_u64_u32(u32* out, u32 seed, int iters) {
  u64 acc[kStreams];
  u32 a[kStreams];
  u32 b = seed ^ (u32)threadIdx.x;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) {
    acc[k] = (u64)k;
    a[k] = (seed + (u32)threadIdx.x) * (u32)(2 * k + 1) + (u32)k;
  }
  for (int it = 0; it < iters; ++it) {
    b = next_operand(b);
#pragma unroll
    for (int k = 0; k < kStreams; ++k) acc[k] = (u64)a[k] * (u64)b + acc[k];
  }
  u64 s = 0;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) s ^= acc[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = (u32)s ^ (u32)(s >> 32);
}

// one v_mul_lo_u32 and one v_mul_hi_u32 per stream and iteration (the 32-bit-limb alternative)
__global__ __launch_bounds__(256) void k_mul_lo_hi(u32* out, u32 seed, int iters) {
  u32 lo[kStreams], hi[kStreams];
  const u32 a = seed + (u32)threadIdx.x, b = (seed ^ (u32)threadIdx.x) | 0x80000001u;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) {
    lo[k] = (u32)k + 3u;
    hi[k] = 0xFFFFFF00u + (u32)k;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kStreams; ++k) {
      lo[k] = (a + (u32)k) * lo[k];
      hi[k] = __umulhi(b, hi[k]) | 0x80000000u;
    }
  }
  u32 s = 0;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) s ^= lo[k] ^ hi[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// one v_mul_u32_u24 per stream and iteration (the 24-bit-limb alternative)
__global__ __launch_bounds__(256) void k_mul_u24(u32* out, u32 seed, int iters) {
  u32 v[kStreams];
  const u32 a = (seed + (u32)threadIdx.x) | 1u;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) v[k] = (u32)k + 5u;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kStreams; ++k) v[k] = __umul24(a, v[k]) + 1u;
  }
  u32 s = 0;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) s ^= v[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// one FP64 fused multiply-add per stream and iteration (the 52-bit-limb alternative)
__global__ __launch_bounds__(256) void k_fma_f64(u32* out, u32 seed, int iters) {
  double acc[kStreams];
  const double a = 1.0 + (double)(seed + threadIdx.x) * 1e-12, b = 1e-9;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) acc[k] = (double)k;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kStreams; ++k) acc[k] = __builtin_fma(a, acc[k], b);
  }
  double s = 0;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) s += acc[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = (u32)__double_as_longlong(s);
}

// one 32-bit add per stream and iteration: the plain full-rate VALU instruction, for reference
__global__ __launch_bounds__(256) void k_add_u32(u32* out, u32 seed, int iters) {
  u32 acc[kStreams];
  const u32 a = seed + (u32)threadIdx.x;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) acc[k] = (u32)k;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kStreams; ++k) acc[k] = acc[k] + (a ^ acc[(k + 1) % kStreams]);
  }
  u32 s = 0;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) s ^= acc[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// HBM: 16-byte accesses, grid-stride
__global__ __launch_bounds__(256) void k_fill(uint4* dst, size_t n16) {
  const uint4 v = make_uint4(1u, 2u, 3u, 4u);
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) dst[i] = v;
}
__global__ __launch_bounds__(256) void k_copy(uint4* __restrict__ dst, const uint4* __restrict__ src, size_t n16) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) dst[i] = src[i];
}
__global__ __launch_bounds__(256) void k_read(u32* out, const uint4* __restrict__ src, size_t n16) {
  u32 s = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n16; i += (size_t)gridDim.x * blockDim.x) {
    const uint4 v = src[i];
    s ^= v.x ^ v.y ^ v.z ^ v.w;
  }
  if (s == 0x9E3779B9u) out[0] = s;  // practically never: the loads only have to be used
}

}  // namespace

extern "C" {

int haflo_peak_streams(void) { return kStreams; }

int haflo_peak_alu(int kind, int blocks, int iters, uint32_t* d_out, void* stream) {
  if (blocks <= 0 || iters <= 0 || !d_out) return -1;
  hipStream_t st = (hipStream_t)stream;
  const dim3 grid((unsigned)blocks), block(256);
  switch (kind) {
    case HAFLO_PEAK_MAD_U64_U32: hipLaunchKernelGGL(k_mad_u64_u32, grid, block, 0, st, d_out, 12345u, iters); break;
    case HAFLO_PEAK_MUL_LO_HI: hipLaunchKernelGGL(k_mul_lo_hi, grid, block, 0, st, d_out, 12345u, iters); break;
    case HAFLO_PEAK_MUL_U24: hipLaunchKernelGGL(k_mul_u24, grid, block, 0, st, d_out, 12345u, iters); break;
    case HAFLO_PEAK_FMA_F64: hipLaunchKernelGGL(k_fma_f64, grid, block, 0, st, d_out, 12345u, iters); break;
    case HAFLO_PEAK_ADD_U32: hipLaunchKernelGGL(k_add_u32, grid, block, 0, st, d_out, 12345u, iters); break;
    default: return -1;
  }
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

int haflo_peak_hbm(int kind, int blocks, void* d_dst, const void* d_src, size_t bytes, void* stream) {
  if (blocks <= 0 || !d_dst || (bytes & 15)) return -1;
  hipStream_t st = (hipStream_t)stream;
  const dim3 grid((unsigned)blocks), block(256);
  const size_t n16 = bytes / 16;
  switch (kind) {
    case HAFLO_PEAK_FILL: hipLaunchKernelGGL(k_fill, grid, block, 0, st, (uint4*)d_dst, n16); break;
    case HAFLO_PEAK_COPY:
      if (!d_src) return -1;
      hipLaunchKernelGGL(k_copy, grid, block, 0, st, (uint4*)d_dst, (const uint4*)d_src, n16);
      break;
    case HAFLO_PEAK_READ:
      if (!d_src) return -1;
      hipLaunchKernelGGL(k_read, grid, block, 0, st, (u32*)d_dst, (const uint4*)d_src, n16);
      break;
    default: return -1;
  }
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
