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

// Every chain takes its second operand from the neighbouring chain's accumulator of the previous
// iteration: nothing is loop-invariant (so nothing can be hoisted), no chain waits for another within an
// iteration, and the loop's own bookkeeping is scalar, so the vector unit issues the instruction under test
// and nothing else.

// one 32x32+64 -> 64 multiply-add (v_mad_u64_u32) per chain and iteration
__global__ __launch_bounds__(256) void k_mad_u64_u32(u32* out, u32 seed, int iters) {
  u64 acc[kStreams];
  u32 a[kStreams];
#pragma unroll
  for (int k = 0; k < kStreams; ++k) {
    acc[k] = (u64)(seed * (u32)(k + 1) + (u32)threadIdx.x) | 1ull;
    a[k] = ((seed + (u32)threadIdx.x) * (u32)(2 * k + 1) + (u32)k) | 0x10000001u;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kStreams; ++k) acc[k] = (u64)a[k] * (u64)(u32)acc[(k + 1) % kStreams] + acc[k];
  }
  u64 s = 0;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) s ^= acc[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = (u32)s ^ (u32)(s >> 32);
}

// one v_mul_lo_u32 and one v_mul_hi_u32 per chain and iteration (32-bit limbs: the two halves of a
// product), plus the add that a limb product needs to be accumulated
__global__ __launch_bounds__(256) void k_mul_lo_hi(u32* out, u32 seed, int iters) {
  u32 lo[kStreams], hi[kStreams], a[kStreams];
#pragma unroll
  for (int k = 0; k < kStreams; ++k) {
    lo[k] = (seed * (u32)(k + 3) + (u32)threadIdx.x) | 1u;
    hi[k] = (u32)k;
    a[k] = ((seed + (u32)threadIdx.x) * (u32)(2 * k + 1) + (u32)k) | 0x80000001u;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kStreams; ++k) {
      const u32 other = lo[(k + 1) % kStreams];
      hi[k] += __umulhi(a[k], other);
      lo[k] = a[k] * other;
    }
  }
  u32 s = 0;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) s ^= lo[k] ^ hi[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// one v_mad_u32_u24 per chain and iteration (24-bit limbs: the low 32 bits of a 24x24 product, accumulated)
__global__ __launch_bounds__(256) void k_mad_u24(u32* out, u32 seed, int iters) {
  u32 v[kStreams], a[kStreams];
#pragma unroll
  for (int k = 0; k < kStreams; ++k) {
    v[k] = (seed * (u32)(k + 5) + (u32)threadIdx.x) | 1u;
    a[k] = ((seed + (u32)threadIdx.x) * (u32)(2 * k + 1)) | 0x800001u;
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kStreams; ++k) v[k] = __umul24(a[k], v[(k + 1) % kStreams]) + v[k];
  }
  u32 s = 0;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) s ^= v[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// one FP64 fused multiply-add per chain and iteration (limbs in doubles)
__global__ __launch_bounds__(256) void k_fma_f64(u32* out, u32 seed, int iters) {
  double acc[kStreams], a[kStreams];
#pragma unroll
  for (int k = 0; k < kStreams; ++k) {
    acc[k] = 1.0 + (double)k + (double)threadIdx.x * 1e-3;
    a[k] = 1e-4 * (double)(1 + ((seed + (u32)k) & 7u));
  }
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kStreams; ++k) acc[k] = __builtin_fma(a[k], acc[(k + 1) % kStreams], acc[k]);
  }
  double s = 0;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) s += acc[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = (u32)__double_as_longlong(s);
}

// one 32-bit add per chain and iteration: a plain full-rate VALU instruction, for reference
__global__ __launch_bounds__(256) void k_add_u32(u32* out, u32 seed, int iters) {
  u32 acc[kStreams];
#pragma unroll
  for (int k = 0; k < kStreams; ++k) acc[k] = seed * (u32)(k + 1) + (u32)threadIdx.x;
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int k = 0; k < kStreams; ++k) acc[k] = acc[k] + acc[(k + 1) % kStreams];
  }
  u32 s = 0;
#pragma unroll
  for (int k = 0; k < kStreams; ++k) s ^= acc[k];
  out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// HBM: 16-byte accesses; a block works through contiguous tiles of kTile accesses per lane (so that
// several independent accesses are in flight per lane), tiles handed out grid-stride
constexpr int kTile = 4;
typedef u32 v4u __attribute__((ext_vector_type(4)));  // 16 bytes, a type the non-temporal builtins accept
__global__ __launch_bounds__(256) void k_fill(v4u* dst, size_t n16) {
  const v4u v = {1u, 2u, 3u, 4u};
  const size_t per_block = (size_t)blockDim.x * kTile;
  for (size_t base = (size_t)blockIdx.x * per_block; base < n16; base += (size_t)gridDim.x * per_block) {
#pragma unroll
    for (int u = 0; u < kTile; ++u) {
      const size_t i = base + (size_t)u * blockDim.x + threadIdx.x;
      if (i < n16) __builtin_nontemporal_store(v, dst + i);
    }
  }
}
__global__ __launch_bounds__(256) void k_copy(v4u* __restrict__ dst, const v4u* __restrict__ src, size_t n16) {
  const size_t per_block = (size_t)blockDim.x * kTile;
  for (size_t base = (size_t)blockIdx.x * per_block; base < n16; base += (size_t)gridDim.x * per_block) {
    v4u v[kTile];
#pragma unroll
    for (int u = 0; u < kTile; ++u) {
      const size_t i = base + (size_t)u * blockDim.x + threadIdx.x;
      if (i < n16) v[u] = __builtin_nontemporal_load(src + i);
    }
#pragma unroll
    for (int u = 0; u < kTile; ++u) {
      const size_t i = base + (size_t)u * blockDim.x + threadIdx.x;
      if (i < n16) __builtin_nontemporal_store(v[u], dst + i);
    }
  }
}
__global__ __launch_bounds__(256) void k_read(u32* out, const v4u* __restrict__ src, size_t n16) {
  u32 s = 0;
  const size_t per_block = (size_t)blockDim.x * kTile;
  for (size_t base = (size_t)blockIdx.x * per_block; base < n16; base += (size_t)gridDim.x * per_block) {
#pragma unroll
    for (int u = 0; u < kTile; ++u) {
      const size_t i = base + (size_t)u * blockDim.x + threadIdx.x;
      if (i < n16) {
        const v4u v = __builtin_nontemporal_load(src + i);
        s ^= v.x ^ v.y ^ v.z ^ v.w;
      }
    }
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
    case HAFLO_PEAK_MUL_U24: hipLaunchKernelGGL(k_mad_u24, grid, block, 0, st, d_out, 12345u, iters); break;
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
    case HAFLO_PEAK_FILL: hipLaunchKernelGGL(k_fill, grid, block, 0, st, (v4u*)d_dst, n16); break;
    case HAFLO_PEAK_COPY:
      if (!d_src) return -1;
      hipLaunchKernelGGL(k_copy, grid, block, 0, st, (v4u*)d_dst, (const v4u*)d_src, n16);
      break;
    case HAFLO_PEAK_READ:
      if (!d_src) return -1;
      hipLaunchKernelGGL(k_read, grid, block, 0, st, (u32*)d_dst, (const v4u*)d_src, n16);
      break;
    default: return -1;
  }
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
