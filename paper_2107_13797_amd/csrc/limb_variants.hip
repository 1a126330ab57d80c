// Alternative limb widths for the Montgomery product, measured against the shipped core: one big
// integer per lane (no cross-lane traffic, so only the arithmetic differs), a modulus of about 522 bits,
// `iters` dependent products x <- x * y / R mod n per lane. Part of libhaflo_peak.so (measurement only).
//   29-bit limbs: the shipped montmul<18, 1> (v_mad_u64_u32 into 64-bit columns, no carry instruction);
//   24-bit limbs: v_mul_u32_u24 + v_mul_hi_u32_u24 per limb product, 64-bit columns kept as two words;
//   23-bit limbs in doubles: one FP64 FMA per limb product (46-bit products, a column takes at most 46 of
//     them before it leaves the window: exact in 53 bits), quotient digits and carries by floor().
// Inputs and outputs are in each variant's own radix (the host packs and unpacks); results are lazy
// (below 2n), the caller reduces them.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/haflo_peak.h"
#include "bigdev.hpp"

namespace {

using haflo::dev::u32;
using haflo::dev::u64;

// ---- 29-bit limbs: the shipped core --------------------------------------------------------------------
constexpr int kL29 = 18;
__global__ __launch_bounds__(256) void k_chain29(const u32* __restrict__ x, const u32* __restrict__ y,
                                                 const u32* __restrict__ n, u32 n0inv, int iters,
                                                 u32* __restrict__ out, size_t count) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  haflo::dev::Grp<1> g;
  u32 a[kL29], b[kL29], m[kL29];
#pragma unroll
  for (int j = 0; j < kL29; ++j) {
    a[j] = x[i * kL29 + j];
    b[j] = y[i * kL29 + j];
    m[j] = n[j];
  }
  for (int it = 0; it < iters; ++it) haflo::dev::montmul<kL29, 1>(a, a, b, m, n0inv, g);
#pragma unroll
  for (int j = 0; j < kL29; ++j) out[i * kL29 + j] = a[j];
}
// the same chain of squarings (x <- x^2 / R), with the symmetric half left out
__global__ __launch_bounds__(256) void k_chain29_sqr(const u32* __restrict__ x, const u32* __restrict__ n, u32 n0inv,
                                                     int iters, u32* __restrict__ out, size_t count) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  haflo::dev::Grp<1> g;
  u32 a[kL29], m[kL29];
#pragma unroll
  for (int j = 0; j < kL29; ++j) {
    a[j] = x[i * kL29 + j];
    m[j] = n[j];
  }
  for (int it = 0; it < iters; ++it) haflo::dev::montsqr<kL29, 1>(a, a, m, n0inv, g);
#pragma unroll
  for (int j = 0; j < kL29; ++j) out[i * kL29 + j] = a[j];
}

// ---- 24-bit limbs: the 24-bit multiply instructions -------------------------------------------------------
constexpr int kL24 = 22;
constexpr u32 kMask24 = 0xFFFFFFu;
// col += a * b for 24-bit a, b: the low 32 bits and the high 16 bits of the product come from two
// instructions, then a 64-bit add in two
__device__ __forceinline__ void mac24(u32& lo, u32& hi, u32 a, u32 b) {
  u32 pl, ph;
  asm("v_mul_u32_u24 %0, %1, %2" : "=v"(pl) : "v"(a), "v"(b));
  asm("v_mul_hi_u32_u24 %0, %1, %2" : "=v"(ph) : "v"(a), "v"(b));
  const u64 s = (((u64)hi << 32) | lo) + (((u64)ph << 32) | pl);
  lo = (u32)s;
  hi = (u32)(s >> 32);
}
__global__ __launch_bounds__(256) void k_chain24(const u32* __restrict__ x, const u32* __restrict__ y,
                                                 const u32* __restrict__ n, u32 n0inv, int iters,
                                                 u32* __restrict__ out, size_t count) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  u32 a[kL24], b[kL24], m[kL24];
#pragma unroll
  for (int j = 0; j < kL24; ++j) {
    a[j] = x[i * kL24 + j];
    b[j] = y[i * kL24 + j];
    m[j] = n[j];
  }
  for (int it = 0; it < iters; ++it) {
    u32 lo[kL24], hi[kL24];
#pragma unroll
    for (int j = 0; j < kL24; ++j) lo[j] = hi[j] = 0u;
#pragma unroll
    for (int r = 0; r < kL24; ++r) {
      const u32 bi = b[r];
#pragma unroll
      for (int j = 0; j < kL24; ++j) mac24(lo[j], hi[j], a[j], bi);
      const u32 q = (lo[0] * n0inv) & kMask24;
#pragma unroll
      for (int j = 0; j < kL24; ++j) mac24(lo[j], hi[j], m[j], q);
      // drop the lowest column (zero modulo 2^24): its upper part is the carry into the next one
      u64 c = ((((u64)hi[0]) << 32) | lo[0]) >> 24;
#pragma unroll
      for (int j = 1; j < kL24; ++j) {
        const u64 v = (((u64)hi[j] << 32) | lo[j]) + (j == 1 ? c : 0ull);
        lo[j - 1] = (u32)v;
        hi[j - 1] = (u32)(v >> 32);
      }
      lo[kL24 - 1] = hi[kL24 - 1] = 0u;
    }
    // compress the columns to 24-bit limbs (lazy: the value stays below 2n)
    u64 c = 0;
#pragma unroll
    for (int j = 0; j < kL24; ++j) {
      const u64 v = (((u64)hi[j] << 32) | lo[j]) + c;
      a[j] = (u32)v & kMask24;
      c = v >> 24;
    }
  }
#pragma unroll
  for (int j = 0; j < kL24; ++j) out[i * kL24 + j] = a[j];
}

// ---- 23-bit limbs in doubles: FP64 FMA --------------------------------------------------------------------
constexpr int kL23 = 23;
__global__ __launch_bounds__(256) void k_chain23f(const double* __restrict__ x, const double* __restrict__ y,
                                                  const double* __restrict__ n, double n0inv, int iters,
                                                  double* __restrict__ out, size_t count) {
  const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  if (i >= count) return;
  const double two23 = 8388608.0, inv23 = 1.0 / 8388608.0;
  double a[kL23], b[kL23], m[kL23];
#pragma unroll
  for (int j = 0; j < kL23; ++j) {
    a[j] = x[i * kL23 + j];
    b[j] = y[i * kL23 + j];
    m[j] = n[j];
  }
  for (int it = 0; it < iters; ++it) {
    double t[kL23];
#pragma unroll
    for (int j = 0; j < kL23; ++j) t[j] = 0.0;
#pragma unroll
    for (int r = 0; r < kL23; ++r) {
      const double bi = b[r];
#pragma unroll
      for (int j = 0; j < kL23; ++j) t[j] = __builtin_fma(a[j], bi, t[j]);
      // q = (t0 mod 2^23) * n0inv mod 2^23, all exact in doubles
      const double low = t[0] - __builtin_floor(t[0] * inv23) * two23;
      const double qq = low * n0inv;
      const double q = qq - __builtin_floor(qq * inv23) * two23;
#pragma unroll
      for (int j = 0; j < kL23; ++j) t[j] = __builtin_fma(m[j], q, t[j]);
      const double carry = t[0] * inv23;  // exact: t0 is a multiple of 2^23
#pragma unroll
      for (int j = 1; j < kL23; ++j) t[j - 1] = t[j] + (j == 1 ? carry : 0.0);
      t[kL23 - 1] = 0.0;
    }
    double c = 0.0;
#pragma unroll
    for (int j = 0; j < kL23; ++j) {
      const double v = t[j] + c;
      c = __builtin_floor(v * inv23);
      a[j] = v - c * two23;
    }
  }
#pragma unroll
  for (int j = 0; j < kL23; ++j) out[i * kL23 + j] = a[j];
}

}  // namespace

extern "C" {

int haflo_peak_limbs(int kind, uint32_t* limbs, uint32_t* limb_bits) {
  int l, bts;
  switch (kind) {
    case HAFLO_LIMBS_29_MAD64:
    case HAFLO_LIMBS_29_MAD64_SQUARE: l = kL29, bts = 29; break;
    case HAFLO_LIMBS_24_MUL24: l = kL24, bts = 24; break;
    case HAFLO_LIMBS_23_FMA64: l = kL23, bts = 23; break;
    default: return -1;
  }
  if (limbs) *limbs = (uint32_t)l;
  if (limb_bits) *limb_bits = (uint32_t)bts;
  return 0;
}

int haflo_peak_montmul_chain(int kind, const void* d_x, const void* d_y, const void* d_n, uint64_t n0inv, int iters,
                             void* d_out, size_t count, void* stream) {
  if (!d_x || !d_n || !d_out || iters <= 0 || count == 0) return -1;
  if (kind != HAFLO_LIMBS_29_MAD64_SQUARE && !d_y) return -1;
  hipStream_t st = (hipStream_t)stream;
  const dim3 grid((unsigned)((count + 255) / 256)), block(256);
  switch (kind) {
    case HAFLO_LIMBS_29_MAD64:
      hipLaunchKernelGGL(k_chain29, grid, block, 0, st, (const u32*)d_x, (const u32*)d_y, (const u32*)d_n, (u32)n0inv, iters,
                         (u32*)d_out, count);
      break;
    case HAFLO_LIMBS_29_MAD64_SQUARE:
      hipLaunchKernelGGL(k_chain29_sqr, grid, block, 0, st, (const u32*)d_x, (const u32*)d_n, (u32)n0inv, iters,
                         (u32*)d_out, count);
      break;
    case HAFLO_LIMBS_24_MUL24:
      hipLaunchKernelGGL(k_chain24, grid, block, 0, st, (const u32*)d_x, (const u32*)d_y, (const u32*)d_n, (u32)n0inv, iters,
                         (u32*)d_out, count);
      break;
    case HAFLO_LIMBS_23_FMA64:
      hipLaunchKernelGGL(k_chain23f, grid, block, 0, st, (const double*)d_x, (const double*)d_y, (const double*)d_n,
                         (double)n0inv, iters, (double*)d_out, count);
      break;
    default: return -1;
  }
  return hipGetLastError() == hipSuccess ? 0 : -4;
}

}  // extern "C"
