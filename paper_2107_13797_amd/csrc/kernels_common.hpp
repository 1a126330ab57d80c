// Kernel-side helpers shared by the operator kernels: per-lane copies of the
// modulus, batch iteration, window-table exponentiation.
#pragma once
#include "bigdev.hpp"
#include "haflo_internal.hpp"

namespace haflo {
namespace dev {

template <int LPT>
struct ModRegs {
  u32 n[LPT];
  u32 n0inv;
};

template <int LPT, int T>
__device__ __forceinline__ void load_mod(ModRegs<LPT>& m, const ModRef& ref, const Grp<T>& g) {
  load_limbs<LPT, T>(m.n, ref.n, g);
  m.n0inv = ref.n0inv;
}

// Batch iteration: every block walks the same number of rounds so that
// block-wide barriers inside the loop body are legal; a group whose item index
// is past the end computes on zeros and stores nothing.
template <int T>
struct Batch {
  int gpb;  // groups per block
  int gib;  // this lane's group inside the block
  __device__ __forceinline__ Batch() {
    gpb = (int)blockDim.x / T;
    gib = (int)threadIdx.x / T;
  }
  __device__ __forceinline__ size_t first() const { return (size_t)blockIdx.x * gpb; }
  __device__ __forceinline__ size_t stride() const { return (size_t)gridDim.x * gpb; }
  // index of this group's private slot in a per-launch workspace
  __device__ __forceinline__ size_t slot() const { return (size_t)blockIdx.x * gpb + gib; }
};

// One cheap carry pass for a lazy sum: limbs end below 2^29 + 2^4.
template <int LPT, int T>
__device__ __forceinline__ void partial_norm(u32 (&x)[LPT], const Grp<T>& g) {
  u32 c = 0;
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    u32 v = x[j] + c;
    x[j] = v & LIMB_MASK;
    c = v >> LIMB_BITS;
  }
  if (T > 1) x[0] += g.from_lower(c);
}

struct SchedInline {
  u32 steps[64];
  int nsteps;
  int first;
  int table_len;
  int is_zero;
};
__device__ __forceinline__ u32 sched_step(const SchedRef& s, int i) { return s.steps[i]; }
__device__ __forceinline__ u32 sched_step(const SchedInline& s, int i) { return s.steps[i]; }

// acc = x^e in Montgomery form for the fixed exponent described by `S`
// (sliding windows over a table of odd powers kept in this group's workspace
// slot: table_len entries of NL limbs, each lane reading back only the limbs
// it wrote itself). xbar: Montgomery form of x, lazy. acc: lazy, < 2n.
template <int LPT, int T, class Sched>
__device__ __forceinline__ void modexp_fixed(u32 (&acc)[LPT], const u32 (&xbar)[LPT], const ModRegs<LPT>& M,
                                             const Sched& S, u32* table, const u32* r1, const Grp<T>& g) {
  constexpr int NL = LPT * T;
  if (S.is_zero) {
    load_limbs<LPT, T>(acc, r1, g);
    return;
  }
  store_limbs<LPT, T>(table, xbar, g);
  if (S.table_len > 1) {
    u32 x2[LPT], cur[LPT];
    montmul<LPT, T>(x2, xbar, xbar, M.n, M.n0inv, g);
#pragma unroll
    for (int j = 0; j < LPT; ++j) cur[j] = xbar[j];
#pragma unroll 1
    for (int i = 1; i < S.table_len; ++i) {
      montmul<LPT, T>(cur, cur, x2, M.n, M.n0inv, g);
      store_limbs<LPT, T>(table + (size_t)i * NL, cur, g);
    }
  }
  load_limbs<LPT, T>(acc, table + (size_t)S.first * NL, g);
#pragma unroll 1
  for (int s = 0; s < S.nsteps; ++s) {
    u32 st = sched_step(S, s);
    int nsq = (int)(st >> 16);
    u32 idx = st & 0xFFFFu;
#pragma unroll 1
    for (int i = 0; i < nsq; ++i) montmul<LPT, T>(acc, acc, acc, M.n, M.n0inv, g);
    if (idx != kNoMul) {
      u32 t[LPT];
      load_limbs<LPT, T>(t, table + (size_t)idx * NL, g);
      montmul<LPT, T>(acc, acc, t, M.n, M.n0inv, g);
    }
  }
}

}  // namespace dev
}  // namespace haflo

#define HAFLO_LAUNCH(KERNEL, SHAPE, STREAM, ...) \
  hipLaunchKernelGGL(KERNEL, dim3((SHAPE).blocks), dim3((SHAPE).threads), 0, (STREAM), __VA_ARGS__)

// Dispatch a kernel template on the (limbs per lane, lanes per integer)
// geometry of a modulus. Expands `CALL(LPT, T)`.
#define HAFLO_DISPATCH_GEOMETRY(m, CALL)                          \
  do {                                                            \
    if ((m).lpt == 18 && (m).t == 1) { CALL(18, 1); }             \
    else if ((m).lpt == 18 && (m).t == 2) { CALL(18, 2); }        \
    else if ((m).lpt == 18 && (m).t == 4) { CALL(18, 4); }        \
    else if ((m).lpt == 18 && (m).t == 8) { CALL(18, 8); }        \
    else if ((m).lpt == 18 && (m).t == 16) { CALL(18, 16); }      \
    else if ((m).lpt == 9 && (m).t == 1) { CALL(9, 1); }          \
    else return HAFLO_EINVAL;                                     \
  } while (0)
