// Ciphertext matrix-vector products, ciphertext summation and the modular
// inverse they need for negative exponents. Kernels and C entry points.
//
// X^T [[d]] (orientation 0): the bases c_i are shared by every output column,
//   so each base gets a table of its powers c_i^0..c_i^16; with signed 5-bit
//   digits d_s of |x_ij| output column j is
//   prod_s ( prod_i table_i[|d_s|] )^(32^s), with the terms of either sign
//   collected separately and one inversion per column. Tall matrices take the
//   bucket method of kernels_buckets.hip instead, which ends in the same
//   per-column pair of products.
// X [[w]] (orientation 1): the few bases c_j are shared by every output row,
//   so each base (and its inverse) gets positional tables c_j^(d 2^(w s)); an
//   output row is a plain product of table entries over its non-zero entries,
//   which are compacted per row first; rows are processed in the order of
//   their list lengths.
#include "kernels_common.hpp"

#include <stdlib.h>

#include <algorithm>

using namespace haflo;
using namespace haflo::dev;

namespace {

// Orientation 1: unsigned 8-bit digits of |x|, positional tables.
constexpr int kWin = 8;                    // window width of the exponent digits
constexpr int kWinEntries = 1 << kWin;     // table entries per base and position (entry 0 unused)
constexpr int kMaxPos = (32 + kWin - 1) / kWin;  // digit positions of a 32-bit magnitude

// Orientation 0: signed 5-bit digits. |x| + c, c = 16 (32^S - 1) / 31, is read in base 32 and
// each digit e is taken as d = e - 16 in [-16, 15], so |x| = sum d_s 32^s: the table holds only
// c^0..c^16 and a negative digit sends the term to the accumulator of the opposite sign.
constexpr int kSWin = 5;
constexpr int kSEntries = 17;
constexpr int kSMaxPos = 7;  // 32^7 - c_7 > 2^31
__host__ __device__ inline unsigned long long signed_digit_offset(int npos) {
  unsigned long long c = 0;
  for (int s = 0; s < npos; ++s) c = c * 32ull + 16ull;
  return c;
}
// positions needed so that maxmag + c_S < 32^S (0 for an all-zero matrix)
__host__ __device__ inline int signed_digit_positions(unsigned maxmag) {
  if (maxmag == 0) return 0;
  for (int s = 1; s < kSMaxPos; ++s)
    if ((unsigned long long)maxmag + signed_digit_offset(s) < (1ull << (kSWin * s))) return s;
  return kSMaxPos;
}

// ---------------------------------------------------------------------------
// modular inverse by batched division steps
// ---------------------------------------------------------------------------

// 29 division steps of the Bernstein-Yang 2-adic gcd recurrence on the low
// bits of (f, g), f odd:
//   g odd and delta > 0:  (delta, f, g) <- (1 - delta, g, (g - f) / 2)
//   g odd otherwise:      (delta, f, g) <- (1 + delta, f, (g + f) / 2)
//   g even:               (delta, f, g) <- (1 + delta, f, g / 2)
// Returns the integer matrix with 2^29 (f', g') = (u f + v g, q f + r g); every
// entry has magnitude at most 2^29 and each row sums to at most 2^29 in
// magnitude.
// The steps are taken in runs: all the halvings that g's trailing zeros allow at once (a count of
// trailing zeros), then, g being odd, the combination of one odd step without its halving, which the
// next run takes. The odd step is written with masks instead of selects - swap and negate,
// (f, g) <- (g, -f) and the matrix rows likewise, when delta > 0, then g += f - so that it is straight-line
// code on the scalar unit (a whole-wavefront group, where f0 and g0 are wave-uniform) as well as on the
// vector unit. About half as many loop rounds as steps, none of them with a branch inside.
__device__ __forceinline__ void divsteps29(int& delta, u32 f0, u32 g0, s32& u, s32& v, s32& q, s32& r) {
  s32 eta = -delta;  // the swap condition is eta < 0
  u32 uu = 1, vv = 0, qq = 0, rr = 1;  // the matrix, in wrapping arithmetic
  int left = LIMB_BITS;
  for (;;) {
    const int z = __builtin_ctz(g0 | (1u << left));  // bits [0, left) of g0 are exact, bit `left` ends the run
    g0 >>= z;
    uu <<= z;
    vv <<= z;
    eta -= z;
    left -= z;
    if (left == 0) break;
    const u32 c = (u32)(eta >> 31);  // all ones: swap
    u32 t = (f0 ^ g0) & c;
    f0 ^= t;
    g0 ^= t;
    g0 = ((g0 ^ c) - c) + f0;
    t = (uu ^ qq) & c;
    uu ^= t;
    qq ^= t;
    qq = ((qq ^ c) - c) + uu;
    t = (vv ^ rr) & c;
    vv ^= t;
    rr ^= t;
    rr = ((rr ^ c) - c) + vv;
    eta = (s32)(((u32)eta ^ c) - c);
  }
  delta = -eta;
  u = (s32)uu;
  v = (s32)vv;
  q = (s32)qq;
  r = (s32)rr;
}

// Shared tail of the two linear updates: absorb the carry of the lane below,
// then drop the (vanished) lowest limb; the top lane's carry becomes the new,
// signed, top limb.
template <int LPT, int T>
__device__ __forceinline__ void shift_down(s32 (&x)[LPT], s32 (&nx)[LPT], s64 carry, const Grp<T>& g) {
  if (T > 1) {
    s32 cin = (s32)g.from_lower((u32)(s32)carry);
    s64 v0 = (s64)nx[0] + (s64)cin;
    nx[0] = (s32)(v0 & (s64)LIMB_MASK);
    nx[1] += (s32)(v0 >> LIMB_BITS);
  }
  s32 down = (s32)g.from_upper((u32)nx[0]);
#pragma unroll
  for (int j = 0; j + 1 < LPT; ++j) x[j] = nx[j + 1];
  x[LPT - 1] = (g.k == T - 1) ? (s32)carry : down;
}

// out = in^-1 * R^2 ... precisely: for `a` the Montgomery form x R of a unit x
// modulo the odd modulus m, returns the Montgomery form x^-1 R (canonical).
// Works on signed numbers in radix 2^29 whose top limb carries the sign:
// (f, g) start at (m, a) and are driven to (+-1, 0) by batches of 29 division
// steps, (d, e) start at (0, 1) and follow the same matrices modulo m, so that
// d * a = f (mod m) throughout; |d| grows by at most m per batch, which the
// head-room of the radix above m absorbs. nbatch bounds the number of batches.
template <int LPT, int T>
__device__ __forceinline__ void invert_mont(u32 (&out)[LPT], const u32 (&a)[LPT], const ModRegs<LPT>& M,
                                            const u32* r3, int nbatch, const Grp<T>& g) {
  s32 f[LPT], gg[LPT], d[LPT], e[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    f[j] = (s32)M.n[j];
    gg[j] = (s32)a[j];
    d[j] = 0;
    e[j] = 0;
  }
  if (g.k == 0) e[0] = 1;
  int delta = 1;
#pragma unroll 1
  for (int b = 0; b < nbatch; ++b) {
    s32 any = 0;
#pragma unroll
    for (int j = 0; j < LPT; ++j) any |= gg[j];
    if (!wave_any(any != 0)) break;
    u32 f0 = g.bcast0((u32)f[0]), g0 = g.bcast0((u32)gg[0]);
    s32 u, v, q, r;
    divsteps29(delta, f0, g0, u, v, q, r);
    {
      s64 cf = 0, cg = 0;
      s32 nf[LPT], ng[LPT];
#pragma unroll
      for (int j = 0; j < LPT; ++j) {
        s64 tf = (s64)u * f[j] + (s64)v * gg[j] + cf;
        s64 tg = (s64)q * f[j] + (s64)r * gg[j] + cg;
        nf[j] = (s32)(tf & (s64)LIMB_MASK);
        cf = tf >> LIMB_BITS;
        ng[j] = (s32)(tg & (s64)LIMB_MASK);
        cg = tg >> LIMB_BITS;
      }
      shift_down<LPT, T>(f, nf, cf, g);
      shift_down<LPT, T>(gg, ng, cg, g);
    }
    {
      // multiples of m that clear the lowest limb of each combination
      u32 lowd = (u32)u * (u32)d[0] + (u32)v * (u32)e[0];
      u32 lowe = (u32)q * (u32)d[0] + (u32)r * (u32)e[0];
      u32 kd = g.bcast0((lowd * M.n0inv) & LIMB_MASK);
      u32 ke = g.bcast0((lowe * M.n0inv) & LIMB_MASK);
      s64 cd = 0, ce = 0;
      s32 nd[LPT], ne[LPT];
#pragma unroll
      for (int j = 0; j < LPT; ++j) {
        s64 td = (s64)u * d[j] + (s64)v * e[j] + (s64)((u64)kd * M.n[j]) + cd;
        s64 te = (s64)q * d[j] + (s64)r * e[j] + (s64)((u64)ke * M.n[j]) + ce;
        nd[j] = (s32)(td & (s64)LIMB_MASK);
        cd = td >> LIMB_BITS;
        ne[j] = (s32)(te & (s64)LIMB_MASK);
        ce = te >> LIMB_BITS;
      }
      shift_down<LPT, T>(d, nd, cd, g);
      shift_down<LPT, T>(e, ne, ce, g);
    }
  }
  // f = +-1 now; the inverse is sign(f) * d modulo m
  u32 f0 = g.bcast0((u32)f[0]) & LIMB_MASK;
  bool fneg = (f0 != 1u);
#pragma unroll
  for (int j = 0; j < LPT; ++j) d[j] = fneg ? -d[j] : d[j];
  int top = resolve<LPT, T>(d, g);
  bool neg = top < 0;
  // from here on every group of the wave runs the same cross-lane code and
  // only selects differ
#pragma unroll
  for (int j = 0; j < LPT; ++j) d[j] = neg ? -d[j] : d[j];
  resolve<LPT, T>(d, g);
  u32 x[LPT], t[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) x[j] = (u32)d[j];
  load_limbs<LPT, T>(t, r3, g);
  montmul<LPT, T>(x, x, t, M.n, M.n0inv, g);  // |d| R^-1 * R^3 / R = |d| R
  canonicalise<LPT, T>(x, M.n, g);
  s32 y[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) y[j] = neg ? (s32)M.n[j] - (s32)x[j] : (s32)x[j];
  resolve<LPT, T>(y, g);
#pragma unroll
  for (int j = 0; j < LPT; ++j) x[j] = (u32)y[j];
  canonicalise<LPT, T>(x, M.n, g);  // m - 0 = m folds back to 0
#pragma unroll
  for (int j = 0; j < LPT; ++j) out[j] = x[j];
}

// The same inverse modulo n^2, through n: y = x^-1 mod n costs half the division steps (the modulus
// has half the bits), and one Newton step lifts it, x^-1 = y (2 - x y) mod n^2.
//   a: Montgomery form x R mod n^2 (lazy), M2/mod2: n^2, Mn: the modulus n with the same R and limb
//   count, nbatch_n: batches for the bit length of n. Returns x^-1 R mod n^2, canonical.
template <int LPT, int T>
__device__ __forceinline__ void invert_lifted(u32 (&out)[LPT], const u32 (&a)[LPT], const ModRegs<LPT>& mod2,
                                              const ModRef& M2, const ModRef& Mn, int nbatch_n, const Grp<T>& g) {
  ModRegs<LPT> mn;
  load_mod<LPT, T>(mn, Mn, g);
  u32 y[LPT], t[LPT];
  load_limbs<LPT, T>(t, Mn.r1, g);
  montmul<LPT, T>(y, a, t, mn.n, mn.n0inv, g);  // a (R mod n) / R = a mod n, which is x R mod n
  canonicalise<LPT, T>(y, mn.n, g);
  invert_mont<LPT, T>(y, y, mn, Mn.r3, nbatch_n, g);  // (x^-1 mod n) R mod n
  load_limbs<LPT, T>(t, Mn.one, g);
  montmul<LPT, T>(y, y, t, mn.n, mn.n0inv, g);  // x^-1 mod n, as a plain integer
  canonicalise<LPT, T>(y, mn.n, g);
  load_limbs<LPT, T>(t, M2.r2, g);
  montmul<LPT, T>(y, y, t, mod2.n, mod2.n0inv, g);  // Y = y R mod n^2
  montmul<LPT, T>(t, a, y, mod2.n, mod2.n0inv, g);  // x y R mod n^2
  canonicalise<LPT, T>(t, mod2.n, g);
  // u = (2 - x y) R + n^2 > 0, below 3 n^2
  u32 r1[LPT];
  load_limbs<LPT, T>(r1, M2.r1, g);
  s32 u[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) u[j] = (s32)(2u * r1[j] + mod2.n[j]) - (s32)t[j];
  resolve<LPT, T>(u, g);
#pragma unroll
  for (int j = 0; j < LPT; ++j) t[j] = (u32)u[j];
  montmul<LPT, T>(y, y, t, mod2.n, mod2.n0inv, g);
  canonicalise<LPT, T>(y, mod2.n, g);
#pragma unroll
  for (int j = 0; j < LPT; ++j) out[j] = y[j];
}

template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_invert(ModRef M, ModRef Mn, const u32* in, u32* out, size_t count,
                                                          int nbatch_n) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 x[LPT];
    if (active) load_limbs<LPT, T>(x, in + item * (size_t)NL, g);
    else zero_limbs<LPT>(x);
    invert_lifted<LPT, T>(x, x, mod, M, Mn, nbatch_n, g);
    if (active) store_limbs<LPT, T>(out + item * (size_t)NL, x, g);
  }
}

// ---------------------------------------------------------------------------
// shared pieces
// ---------------------------------------------------------------------------

// largest |x| in the matrix (atomicMax into a zeroed word)
__global__ __launch_bounds__(kBlockThreads) void k_zero_word(u32* p, int n) {
  // the largest |x|, a work counter and, for orientation 1, the histogram of list lengths
  if (blockIdx.x == 0)
    for (int i = (int)threadIdx.x; i < n; i += (int)blockDim.x) p[i] = 0u;
}
__global__ __launch_bounds__(kBlockThreads) void k_maxmag(const int* __restrict__ X, size_t total, u32* maxmag) {
  u32 m = 0;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += (size_t)gridDim.x * blockDim.x) {
    int x = X[i];
    u32 mag = x < 0 ? 0u - (u32)x : (u32)x;
    m = mag > m ? mag : m;
  }
  // the word only grows: a wavefront whose maximum is already there leaves it alone, so the atomics on the one
  // address stay few
  const u32 best = wave_max(m);
  if ((threadIdx.x & (WAVE - 1)) == 0 && best > *(volatile u32*)maxmag) atomicMax(maxmag, best);
}
__device__ __forceinline__ int bit_length(u32 v) { return v ? 32 - __builtin_clz(v) : 0; }

// product of the per-group accumulators of a block, left in group 0.
// lds: (groups per block / 2) * NL limbs.
template <int LPT, int T>
__device__ __forceinline__ void block_product(u32 (&acc)[LPT], u32* lds, const ModRegs<LPT>& mod, const Batch<T>& bt,
                                              const Grp<T>& g) {
  constexpr int NL = LPT * T;
  for (int stride = bt.gpb >> 1; stride >= 1; stride >>= 1) {
    if (bt.gib >= stride && bt.gib < 2 * stride) {
      u32* dst = lds + (bt.gib - stride) * NL + g.k * LPT;
#pragma unroll
      for (int j = 0; j < LPT; ++j) dst[j] = acc[j];
    }
    __syncthreads();
    u32 t[LPT], r[LPT];
    bool take = bt.gib < stride;
    const u32* src = lds + (take ? bt.gib : 0) * NL + g.k * LPT;
#pragma unroll
    for (int j = 0; j < LPT; ++j) t[j] = src[j];
    montmul<LPT, T>(r, acc, t, mod.n, mod.n0inv, g);
    if (take) {
#pragma unroll
      for (int j = 0; j < LPT; ++j) acc[j] = r[j];
    }
    __syncthreads();
  }
}

// ---------------------------------------------------------------------------
// orientation 0: out[j] = prod_i c_i^X[i][j]
// ---------------------------------------------------------------------------

// block (j, s, rs): product over the rows of slice rs of table_i[digit s of
// |X[i][j]|], positive and negative entries apart -> partials[j][s][sign][rs]
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads, 3) void k_xtd_main(ModRef M, const int* __restrict__ X, size_t rows,
                                                            size_t cols, const u32* __restrict__ tables, int rsplit,
                                                            u32* __restrict__ partials,
                                                            const u32* __restrict__ maxmag) {
  constexpr int NL = LPT * T;
  __shared__ u32 lds[(kBlockThreads / 2) * LPT];
  Grp<T> g;
  Batch<T> bt;
  // Blocks are handed to the 8 XCDs round-robin. The `cols` blocks of one (s, rs) slice read
  // the same table entries, so a slice is kept on one XCD (whose L2 then serves the re-reads)
  // and consecutive slices go to consecutive XCDs. The grid holds a multiple of 8 slices.
  const size_t xcd = blockIdx.x % 8u, local = blockIdx.x / 8u;
  const size_t slice = xcd + 8u * (local / cols);
  const size_t j = local % cols;
  const int rs = (int)(slice % (size_t)rsplit);
  const int s = (int)(slice / (size_t)rsplit);
  if (s >= kSMaxPos) return;  // padding slices
  const int npos = signed_digit_positions(*maxmag);
  if (s >= npos) return;  // no digit at this position anywhere
  const u64 offset = signed_digit_offset(npos);
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const size_t r0 = rows * (size_t)rs / (size_t)rsplit, r1 = rows * (size_t)(rs + 1) / (size_t)rsplit;
  u32 accp[LPT], accn[LPT];
  load_limbs<LPT, T>(accp, M.r1, g);
#pragma unroll
  for (int jj = 0; jj < LPT; ++jj) accn[jj] = accp[jj];
  for (size_t base = r0; base < r1; base += (size_t)bt.gpb) {
    size_t i = base + bt.gib;
    bool active = i < r1;
    int x = active ? X[i * cols + j] : 0;
    u32 mag = x < 0 ? 0u - (u32)x : (u32)x;
    int d = (int)((((u64)mag + offset) >> (s * kSWin)) & 31ull) - 16;
    u32 dgt = (u32)(d < 0 ? -d : d);
    const u32* entry = active ? tables + (i * (size_t)kSEntries + dgt) * NL : M.r1;
    u32 cur[LPT];
    bool neg = (x < 0) != (d < 0);
#pragma unroll
    for (int jj = 0; jj < LPT; ++jj) cur[jj] = neg ? accn[jj] : accp[jj];
    montmul_mem<LPT, T>(cur, cur, entry, mod.n, mod.n0inv, g);
#pragma unroll
    for (int jj = 0; jj < LPT; ++jj) {
      if (neg) accn[jj] = cur[jj];
      else accp[jj] = cur[jj];
    }
  }
  block_product<LPT, T>(accp, lds, mod, bt, g);
  block_product<LPT, T>(accn, lds, mod, bt, g);
  if (bt.gib == 0) {
    size_t slot = ((j * (size_t)kSMaxPos + (size_t)s) * 2) * (size_t)rsplit + (size_t)rs;
    store_limbs<LPT, T>(partials + slot * NL, accp, g);
    store_limbs<LPT, T>(partials + (slot + (size_t)rsplit) * NL, accn, g);
  }
}

// one group per (j, sign): P = prod_s (prod_rs partial[j][s][sign][rs])^(2^(w s)), top position first
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_xtd_horner(ModRef M, size_t cols, int rsplit,
                                                              const u32* __restrict__ partials, u32* __restrict__ P,
                                                              const u32* __restrict__ maxmag) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const int npos = signed_digit_positions(*maxmag);
  const size_t count = cols * 2;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    size_t j = active ? item >> 1 : 0;
    size_t sign = item & 1;
    u32 acc[LPT], t[LPT];
    load_limbs<LPT, T>(acc, M.r1, g);
#pragma unroll 1
    for (int s = npos - 1; s >= 0; --s) {
      if (s != npos - 1) {
#pragma unroll 1
        for (int i = 0; i < kSWin; ++i) montsqr<LPT, T>(acc, acc, mod.n, mod.n0inv, g);
      }
#pragma unroll 1
      for (int rs = 0; rs < rsplit; ++rs) {
        size_t slot = ((j * (size_t)kSMaxPos + (size_t)s) * 2 + sign) * (size_t)rsplit + (size_t)rs;
        load_limbs<LPT, T>(t, partials + slot * NL, g);
        montmul<LPT, T>(acc, acc, t, mod.n, mod.n0inv, g);
      }
    }
    if (active) store_limbs<LPT, T>(P + item * (size_t)NL, acc, g);
  }
}

// out[j] = P[j][+] * (P[j][-])^-1
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_xtd_finish(ModRef M, ModRef Mn, size_t cols,
                                                              const u32* __restrict__ P, u32* __restrict__ out,
                                                              int nbatch_n) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  for (size_t base = bt.first(); base < cols; base += bt.stride()) {
    size_t j = base + bt.gib;
    bool active = j < cols;
    u32 pos[LPT], neg[LPT];
    if (active) {
      load_limbs<LPT, T>(pos, P + (2 * j) * (size_t)NL, g);
      load_limbs<LPT, T>(neg, P + (2 * j + 1) * (size_t)NL, g);
    } else {
      load_limbs<LPT, T>(pos, M.r1, g);
      load_limbs<LPT, T>(neg, M.r1, g);
    }
    invert_lifted<LPT, T>(neg, neg, mod, M, Mn, nbatch_n, g);
    montmul<LPT, T>(pos, pos, neg, mod.n, mod.n0inv, g);
    canonicalise<LPT, T>(pos, mod.n, g);
    if (active) store_limbs<LPT, T>(out + j * (size_t)NL, pos, g);
  }
}

// ---------------------------------------------------------------------------
// orientation 1: out[i] = prod_j c_j^X[i][j]
// ---------------------------------------------------------------------------

// Positional tables T[j][sign][s][d] = b^(d 256^s), b = c_j or its inverse, d = 1..255.
// k_xw_positions, one group per (j, sign, s): T[1] = b^(256^s) by 8 s squarings. Then eight launches of
// k_xw_level with B = 1, 2, 4, .., 128, one group per entry d in (B, 2 B]: T[d] = T[d - B] * T[B]. Every entry
// costs one product and the chain is 8 s + 8 products long.
// PAIR: the tables are in the pair form modulo M (see Elem); the bases, stored ciphertexts, are taken into it
// as they are loaded (k_lo, k_hi: see to_pair).
template <int LPT, int T, bool PAIR>
__global__ __launch_bounds__(kBlockThreads) void k_xw_positions(ModRef M, const u32* __restrict__ k_lo,
                                                                const u32* __restrict__ k_hi,
                                                                const u32* __restrict__ bases,
                                                                const u32* __restrict__ invbases, size_t cols,
                                                                u32* __restrict__ tables,
                                                                const u32* __restrict__ maxmag) {
  using Ops = ElemOps<LPT, T, PAIR>;
  constexpr int EL = Ops::kLimbs;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const int npos = (bit_length(*maxmag) + kWin - 1) / kWin;
  const size_t count = cols * 2 * (size_t)npos;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    const size_t it = base + bt.gib;
    const bool active = it < count;
    const size_t item = active ? it / (size_t)npos : 0;  // j * 2 + sign
    const int s = active ? (int)(it - item * (size_t)npos) : 0;
    const u32* src = (item & 1) ? invbases : bases;
    typename Ops::E x, t;
    if constexpr (PAIR) to_pair<LPT, T>(x.x0, x.x1, src + (item >> 1) * (size_t)EL, k_lo, k_hi, mod, g);
    else Ops::load(x, src + (item >> 1) * (size_t)EL, g);
    // every group of a wavefront runs the same squarings; the ones that are done discard theirs
#pragma unroll 1
    for (int i = 0; wave_any(i < kWin * s); ++i) {
      Ops::copy(t, x);
      Ops::sqr(t, mod, g);
      if (i < kWin * s) Ops::copy(x, t);
    }
    u32* tb = tables + ((item * (size_t)kMaxPos + (size_t)s) * (size_t)kWinEntries) * EL;
    if (active) Ops::store(tb + EL, x, g);
  }
}

template <int LPT, int T, bool PAIR>
__global__ __launch_bounds__(kBlockThreads) void k_xw_level(ModRef M, const u32* __restrict__ one, size_t cols, int B,
                                                            u32* __restrict__ tables,
                                                            const u32* __restrict__ maxmag) {
  using Ops = ElemOps<LPT, T, PAIR>;
  constexpr int EL = Ops::kLimbs;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const int npos = (bit_length(*maxmag) + kWin - 1) / kWin;
  const int per = B < kWinEntries - 1 - B ? B : kWinEntries - 1 - B;  // entries B + 1 .. min(2 B, 255)
  const size_t count = cols * 2 * (size_t)npos * (size_t)per;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    const size_t it = base + bt.gib;
    const bool active = it < count;
    const size_t tab = active ? it / (size_t)per : 0;  // (j * 2 + sign) * npos + s
    const int d = B + 1 + (active ? (int)(it - tab * (size_t)per) : 0);
    const size_t item = tab / (size_t)(npos ? npos : 1);
    const int s = (int)(tab - item * (size_t)(npos ? npos : 1));
    u32* tb = tables + ((item * (size_t)kMaxPos + (size_t)s) * (size_t)kWinEntries) * EL;
    typename Ops::E a;
    Ops::load(a, active ? tb + (size_t)(d - B) * EL : one, g);
    Ops::mul_mem(a, active ? tb + (size_t)B * EL : one, mod, g);
    if (active) Ops::store(tb + (size_t)d * EL, a, g);
  }
}

// Rows are handed to the wavefronts of k_xw_main in the order of their list lengths, longest
// first, so that the rows a wavefront multiplies side by side finish together. The lengths are
// sorted by counting in kLenBins classes.
constexpr int kLenBins = 1024;
__device__ __forceinline__ u32 length_bin(u32 len, size_t longest) {
  return (u32)(((u64)len * (u64)(kLenBins - 1)) / (u64)(longest ? longest : 1));
}

// Per row: the list of table entries its product consists of, one per non-zero 8-bit digit
// of every non-zero |X[row][c]|: entry index ((c*2 + sign)*kMaxPos + s)*256 + digit, in units of
// one table entry. One wave per row; lists: rows * cols * kMaxPos words, counts: rows.
__global__ __launch_bounds__(kBlockThreads) void k_xw_lists(const int* __restrict__ X, size_t rows, size_t cols,
                                                            u32* __restrict__ lists, u32* __restrict__ counts,
                                                            const u32* __restrict__ maxmag) {
  const int lane = (int)(threadIdx.x & (WAVE - 1));
  const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
  const size_t nwaves = ((size_t)gridDim.x * blockDim.x) / WAVE;
  const int npos = (bit_length(*maxmag) + kWin - 1) / kWin;
  for (size_t row = wave; row < rows; row += nwaves) {
    u32* mine = lists + row * cols * (size_t)kMaxPos;
    u32 written = 0;
    for (size_t c0 = 0; c0 < cols; c0 += WAVE) {
      size_t c = c0 + (size_t)lane;
      int x = (c < cols) ? X[row * cols + c] : 0;
      u32 mag = x < 0 ? 0u - (u32)x : (u32)x;
      u32 tsel = (u32)c * 2u + (x < 0 ? 1u : 0u);
      for (int s = 0; s < npos; ++s) {
        u32 dgt = (mag >> (s * kWin)) & (u32)(kWinEntries - 1);
        u64 mask = __builtin_amdgcn_ballot_w64(dgt != 0u);
        if (dgt != 0u) {
          u32 before = (u32)__builtin_popcountll(mask & ((1ull << lane) - 1ull));
          mine[written + before] = (tsel * (u32)kMaxPos + (u32)s) * (u32)kWinEntries + dgt;
        }
        written += (u32)__builtin_popcountll(mask);
      }
    }
    if (lane == 0) counts[row] = written;
  }
}

// Counting sort of the rows by length class, in two passes around k_xw_order_scan. A block takes 256
// rows at a time and counts them in LDS first, so that global memory sees one atomic per class and
// block. SCATTER = false: bins[b] += rows of class b. SCATTER = true: bins[] are the cursors left by the
// scan; the block reserves its share of every class and writes order[cursor + rank in the block] = row.
template <bool SCATTER>
__global__ __launch_bounds__(kBlockThreads) void k_xw_order(const u32* __restrict__ counts, size_t rows, size_t cols,
                                                            u32* __restrict__ bins, u32* __restrict__ order,
                                                            const u32* __restrict__ maxmag) {
  __shared__ u32 hist[kLenBins];
  __shared__ u32 start[SCATTER ? kLenBins : 1];
  const int npos = (bit_length(*maxmag) + kWin - 1) / kWin;
  const size_t longest = cols * (size_t)npos;
  for (size_t r0 = (size_t)blockIdx.x * kBlockThreads; r0 < rows; r0 += (size_t)gridDim.x * kBlockThreads) {
    for (int l = (int)threadIdx.x; l < kLenBins; l += kBlockThreads) hist[l] = 0u;
    __syncthreads();
    const size_t row = r0 + threadIdx.x;
    const bool active = row < rows;
    const u32 bin = active ? length_bin(counts[row], longest) : 0u;
    const u32 rank = active ? atomicAdd(&hist[bin], 1u) : 0u;
    __syncthreads();
    for (int l = (int)threadIdx.x; l < kLenBins; l += kBlockThreads) {
      const u32 c = hist[l];
      if (c == 0u) continue;
      const u32 before = atomicAdd(&bins[l], c);
      if (SCATTER) start[l] = before;
    }
    if (SCATTER) {
      __syncthreads();
      if (active) order[start[bin] + rank] = (u32)row;
    }
    __syncthreads();
  }
}

// bins[b] = number of rows in longer classes than b: where class b starts in the sorted order.
// One block.
__global__ __launch_bounds__(kBlockThreads) void k_xw_order_scan(u32* __restrict__ bins) {
  constexpr int PER = kLenBins / kBlockThreads;
  __shared__ u32 part[kBlockThreads];
  const int t = (int)threadIdx.x;
  // thread t owns the classes kLenBins-1 - (t*PER + i), i = 0..PER-1, i.e. the order longest first
  u32 own[PER], sum = 0;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    own[i] = bins[kLenBins - 1 - (t * PER + i)];
    sum += own[i];
  }
  part[t] = sum;
  __syncthreads();
  for (int d = 1; d < kBlockThreads; d <<= 1) {
    u32 add = t >= d ? part[t - d] : 0u;
    __syncthreads();
    part[t] += add;
    __syncthreads();
  }
  u32 run = part[t] - sum;
#pragma unroll
  for (int i = 0; i < PER; ++i) {
    bins[kLenBins - 1 - (t * PER + i)] = run;
    run += own[i];
  }
}

// The product of the listed table entries of every row. A row's list is cut into 2^seg_shift segments of
// near-equal length and one lane group multiplies one segment (few rows with long lists would otherwise
// leave most of the chip idle); with one segment the group writes the canonical result to out[row], else
// its lazy partial product to partial[row][segment] for k_xw_combine. Work items are taken in the order
// `order` (rows with the longest lists first): a wavefront takes the run of its own index first, then
// runs drawn from a counter (zero at launch), so that long lists do not leave the rest of the chip waiting.
// PAIR: the table entries are pairs modulo M (see Elem); a finished product leaves the pair form (`leave` = the
// pair constant R_N) and is stored as the canonical integer, the form of a stored ciphertext.
template <int LPT, int T, bool PAIR>
__device__ __forceinline__ void xw_store_result(u32* dst, Elem<LPT, PAIR>& acc, bool active, const u32* leave,
                                                const ModRegs<LPT>& mod, const Grp<T>& g) {
  if constexpr (PAIR) {
    pairmul_mem<LPT, T>(acc.x0, acc.x1, acc.x0, acc.x1, leave, mod.n, mod.n0inv, g);
    pair_canonical<LPT, T>(acc.x0, acc.x1, mod.n, g);
    u32 lo[LPT], hi[LPT];
    pair_to_integer<LPT, T>(lo, hi, acc.x0, acc.x1, mod.n, g);
    if (active) {
      store_limbs<LPT, T>(dst, lo, g);
      store_limbs<LPT, T>(dst + LPT * T, hi, g);
    }
  } else {
    canonicalise<LPT, T>(acc.x0, mod.n, g);
    if (active) store_limbs<LPT, T>(dst, acc.x0, g);
  }
}

template <int LPT, int T, bool PAIR>
__global__ __launch_bounds__(kBlockThreads, 3) void k_xw_main(ModRef M, const u32* __restrict__ one,
                                                           const u32* __restrict__ leave, size_t rows,
                                                           size_t list_stride, const u32* __restrict__ lists,
                                                           const u32* __restrict__ counts,
                                                           const u32* __restrict__ order,
                                                           const u32* __restrict__ tables, u32* __restrict__ next_item,
                                                           int seg_shift, u32* __restrict__ partial,
                                                           u32* __restrict__ out) {
  using Ops = ElemOps<LPT, T, PAIR>;
  constexpr int EL = Ops::kLimbs;
  constexpr int GW = WAVE / T;
  Grp<T> g;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const int lane = (int)(threadIdx.x & (WAVE - 1));
  const size_t nwaves = ((size_t)gridDim.x * blockDim.x) / WAVE;
  const size_t items = rows << seg_shift;
  const u32 nseg = 1u << seg_shift;
  size_t w0 = (((size_t)blockIdx.x * blockDim.x + threadIdx.x) / WAVE) * GW;
  while (w0 < items) {
    const size_t item = w0 + (size_t)(lane / T);
    const bool active = item < items;
    const size_t row = active ? (size_t)order[item >> seg_shift] : 0;
    const u32 seg = (u32)item & (nseg - 1u);
    const u32 cnt = active ? counts[row] : 0u;
    const u32 e0 = (u32)(((u64)cnt * seg) >> seg_shift), e1 = (u32)(((u64)cnt * (seg + 1u)) >> seg_shift);
    const u32* mine = lists + row * list_stride;
    auto entry = [&](u32 e) -> const u32* { return (e < e1) ? tables + (size_t)mine[e] * EL : one; };
    typename Ops::E acc;
    Ops::load(acc, entry(e0), g);
#pragma unroll 1
    for (u32 e = e0 + 1; wave_any(e < e1); ++e) {
      // the next entry is looked up and touched while this one is multiplied; a group that has run out
      // of entries multiplies by one and stays in step with its wave
      const u32 touch = Ops::touch(entry(e + 1), g);
      Ops::mul_mem(acc, entry(e), mod, g);
      keep_live(touch);
    }
    if (seg_shift == 0) {
      xw_store_result<LPT, T, PAIR>(out + row * (size_t)EL, acc, active, leave, mod, g);
    } else if (active) {
      Ops::store(partial + ((row << seg_shift) + seg) * (size_t)EL, acc, g);
    }
    u32 drawn = 0;
    if (lane == 0) drawn = atomicAdd(next_item, (u32)GW);
    w0 = nwaves * GW + (size_t)(u32)__builtin_amdgcn_ds_bpermute(0, (int)drawn);
  }
}

// out[row] = product of the row's 2^seg_shift partial products, canonical
template <int LPT, int T, bool PAIR>
__global__ __launch_bounds__(kBlockThreads) void k_xw_combine(ModRef M, const u32* __restrict__ leave, size_t rows,
                                                              int seg_shift, const u32* __restrict__ partial,
                                                              u32* __restrict__ out) {
  using Ops = ElemOps<LPT, T, PAIR>;
  constexpr int EL = Ops::kLimbs;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  for (size_t base = bt.first(); base < rows; base += bt.stride()) {
    const size_t row = base + bt.gib;
    const bool active = row < rows;
    const u32* mine = partial + ((active ? row : 0) << seg_shift) * (size_t)EL;
    typename Ops::E acc;
    Ops::load(acc, mine, g);
#pragma unroll 1
    for (int sgm = 1; sgm < (1 << seg_shift); ++sgm) Ops::mul_mem(acc, mine + (size_t)sgm * EL, mod, g);
    xw_store_result<LPT, T, PAIR>(out + (active ? row : 0) * (size_t)EL, acc, active, leave, mod, g);
  }
}

// ---------------------------------------------------------------------------
// summation
// ---------------------------------------------------------------------------
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_sum(ModRef M, const u32* __restrict__ in, size_t count,
                                                       u32* __restrict__ out, int canonical) {
  constexpr int NL = LPT * T;
  __shared__ u32 lds[(kBlockThreads / 2) * LPT];
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  u32 acc[LPT], t[LPT];
  load_limbs<LPT, T>(acc, M.r1, g);
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    const u32* src = item < count ? in + item * (size_t)NL : M.r1;
    load_limbs<LPT, T>(t, src, g);
    montmul<LPT, T>(acc, acc, t, mod.n, mod.n0inv, g);
  }
  block_product<LPT, T>(acc, lds, mod, bt, g);
  if (canonical) canonicalise<LPT, T>(acc, mod.n, g);
  if (bt.gib == 0) store_limbs<LPT, T>(out + (size_t)blockIdx.x * NL, acc, g);
}

// batches of 29 division steps that always suffice for the modulus n
int inverse_batches(const haflo_ctx* ctx) {
  size_t bits = ctx->Nw.mod.bits();
  size_t steps = (49 * bits + 57) / 17;
  return (int)((steps + LIMB_BITS - 1) / LIMB_BITS);
}

struct XtdPlan {
  int rsplit;
  size_t off_tables, off_partials, off_P, total;  // in u32 words; word 0 holds the largest |x|
};
XtdPlan xtd_plan(const haflo_ctx* ctx, size_t rows, size_t cols) {
  XtdPlan p;
  const int gpb = kBlockThreads / ctx->N.t;
  // aim at ~4 blocks per compute unit assuming 4 live digit positions, keep >= 2 rows per group
  size_t want = ((size_t)ctx->num_cu * 4 + cols * 4 - 1) / (cols ? cols * 4 : 1);
  size_t maxsplit = rows / ((size_t)gpb * 2);
  if (want > maxsplit) want = maxsplit;
  if (want < 1) want = 1;
  if (want > 64) want = 64;
  p.rsplit = (int)want;
  const size_t nl = (size_t)ctx->N.nl;
  p.off_tables = 64;
  p.off_partials = p.off_tables + rows * kSEntries * nl;
  p.off_P = p.off_partials + cols * kSMaxPos * 2 * (size_t)p.rsplit * nl;
  p.total = p.off_P + cols * 2 * nl;
  return p;
}

// Tall matrices go through the bucket method (one product per exponent digit instead of four or
// five, no tables); below the row threshold its fixed cost per column (1024 buckets per digit
// position) outweighs that. The threshold is a setting of the context (haflo_ctx_set_xtd_bucket_min_rows).
bool use_buckets(const haflo_ctx* ctx, size_t rows, size_t cols) {
  return rows >= ctx->xtd_bucket_min_rows && rows > 0 && xtd_buckets_fit(rows, cols);
}
struct XtdBucketLayout {
  size_t off_P, off_ws, total;  // in u32 words; word 0 holds the largest |x|
};
XtdBucketLayout xtd_bucket_layout(const haflo_ctx* ctx, size_t rows, size_t cols) {
  XtdBucketLayout l;
  l.off_P = 64;
  l.off_ws = (l.off_P + cols * 2 * (size_t)ctx->N.nl + 63) & ~(size_t)63;
  l.total = l.off_ws + xtd_bucket_plan(ctx, rows, cols).total;
  return l;
}

struct XwPlan {
  // in u32 words; word 0 holds the largest |x|, word 1 the row counter of k_xw_main, words
  // [kXwBinsAt, kXwBinsAt + kLenBins) the length classes
  size_t off_inv, off_tables, off_nz, off_cnt, off_order, off_partial, total;
  int seg_shift;  // every row's list is multiplied in 2^seg_shift segments
};
constexpr size_t kXwBinsAt = 64;
// Segments per row: doubled while the chip would hold fewer than four wavefronts per SIMD, up to 8
// and while a full row still gives every segment a few entries.
int xw_seg_shift(const haflo_ctx* ctx, size_t rows, size_t cols) {
  const size_t per_wave = (size_t)(64 / ctx->N.t), want_waves = (size_t)ctx->num_cu * 32;
  int sh = 0;
  while (sh < 3 && (rows << sh) < want_waves * per_wave && cols >= ((size_t)4 << sh)) ++sh;
  return sh;
}
XwPlan xw_plan(const haflo_ctx* ctx, size_t rows, size_t cols) {
  XwPlan p;
  const size_t nl = (size_t)ctx->N.nl;
  p.off_inv = kXwBinsAt + kLenBins;
  p.off_tables = p.off_inv + cols * nl;
  p.off_nz = p.off_tables + cols * 2 * kMaxPos * kWinEntries * nl;
  p.off_cnt = p.off_nz + rows * cols * kMaxPos;
  p.off_order = p.off_cnt + rows;
  p.off_partial = p.off_order + rows;
  p.seg_shift = xw_seg_shift(ctx, rows, cols);
  p.total = p.off_partial + (p.seg_shift ? (rows << p.seg_shift) * nl : 0);
  return p;
}

int sum_blocks(const haflo_ctx* ctx, size_t count) {
  const int gpb = kBlockThreads / ctx->N.t;
  size_t need = (count + (size_t)gpb * 4 - 1) / ((size_t)gpb * 4);
  size_t cap = (size_t)ctx->num_cu * 4;
  if (need < 1) need = 1;
  return (int)(need < cap ? need : cap);
}

int launch_maxmag(const haflo_ctx* ctx, const int32_t* X, size_t total, u32* word, int zero_words, hipStream_t st) {
  LaunchShape one;
  one.blocks = 1;
  one.threads = kBlockThreads;
  one.gpb = kBlockThreads;
  HAFLO_LAUNCH(k_zero_word, one, st, word, zero_words);
  if (total) {
    LaunchShape sh = launch_shape(ctx, (total + 15) / 16, 1, 8);  // sixteen entries per lane: few wavefronts, few atomics
    HAFLO_LAUNCH(k_maxmag, sh, st, X, total, word);
  }
  return hip_status(hipGetLastError());
}

// Launch shape and geometry of a short, latency-bound kernel over `count` big integers modulo `m`: one
// wavefront per integer while every integer can have a SIMD to itself, else twice the lanes per integer
// while the chip is mostly idle, else the modulus's own geometry.
LaunchShape latency_shape(const haflo_ctx* ctx, size_t count, const ModHost& m) {
  LaunchShape sh;
  if (haflo_has_wave_geometry(m) && count <= (size_t)ctx->num_cu * 4) {
    sh.blocks = (int)(count ? count : 1);
    sh.threads = 64;
    sh.gpb = 1;
    sh.geo = kGeoWave;
    return sh;
  }
  const bool wide = haflo::few_groups(ctx, count);
  sh = launch_shape(ctx, count, wide ? haflo_wide_lanes(m) : m.t, 8);
  sh.geo = wide ? kGeoWide : kGeoPlain;
  return sh;
}
#define HAFLO_DISPATCH_SHAPE(sh, m, CALL)                                    \
  do {                                                                       \
    if ((sh).geo == kGeoWave) { HAFLO_DISPATCH_GEOMETRY_WAVE(m, CALL); }     \
    else if ((sh).geo == kGeoWide) { HAFLO_DISPATCH_GEOMETRY_WIDE(m, CALL); } \
    else { HAFLO_DISPATCH_GEOMETRY(m, CALL); }                               \
  } while (0)

}  // namespace

namespace haflo {

int invert_batch(const haflo_ctx* ctx, const uint32_t* in, uint32_t* out, size_t count, hipStream_t st) {
  const ModHost& m = ctx->N;
  const LaunchShape sh = latency_shape(ctx, count, m);
  const int nbatch = inverse_batches(ctx);
#define CALL(LPT, T) HAFLO_LAUNCH((k_invert<LPT, T>), sh, st, m.ref(), ctx->Nw.ref(), in, out, count, nbatch)
  HAFLO_DISPATCH_SHAPE(sh, m, CALL);
#undef CALL
  return hip_status(hipGetLastError());
}

}  // namespace haflo

extern "C" {

size_t haflo_workspace_bytes(const haflo_ctx* ctx, int op, size_t rows, size_t cols) {
  if (!ctx) return (size_t)-1;
  switch (op) {
    case HAFLO_OP_ENCRYPT: return ws_encrypt(ctx, rows);
    case HAFLO_OP_DECRYPT: return ctx->has_priv ? ws_decrypt(ctx, rows) : (size_t)-1;
    case HAFLO_OP_SCALAR_MUL: return ws_scalar_mul(ctx, rows);
    case HAFLO_OP_TAYLOR_LOSS: return ws_taylor_loss(ctx, rows);
    case HAFLO_OP_ENCRYPT_OBFUSCATOR: return ws_encrypt_obf(ctx, rows);
    case HAFLO_OP_FORE_GRADIENT:
      return ((rows * (size_t)ctx->lp * 4 + 255) & ~(size_t)255) + ((rows * (size_t)ctx->N.nl * 4 + 255) & ~(size_t)255) +
             ws_encrypt(ctx, rows);
    case HAFLO_OP_MATVEC_XT_D:
      if (!cols) return 0;
      return (use_buckets(ctx, rows, cols) ? xtd_bucket_layout(ctx, rows, cols).total : xtd_plan(ctx, rows, cols).total) * 4;
    case HAFLO_OP_MATVEC_X_W: return xw_plan(ctx, rows, cols).total * 4;
    case HAFLO_OP_SUM_SEGMENTS:
      if (rows >= (1ull << 32) || cols >= (1ull << 24)) return (size_t)-1;
      return cols ? seg_sum_plan(ctx, rows, cols).total * 4 : 0;
    default: return (size_t)-1;
  }
}

int haflo_cipher_matvec(const haflo_ctx* ctx, int orientation, const void* d_c, const int32_t* d_X, size_t rows,
                        size_t cols, void* d_out, void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx || (orientation != 0 && orientation != 1)) return HAFLO_EINVAL;
  const size_t nin = orientation == 0 ? rows : cols;
  const size_t nout = orientation == 0 ? cols : rows;
  if (nout == 0) return HAFLO_OK;
  if (!d_out || (nin && (!d_c || !d_X))) return HAFLO_EINVAL;
  const ModHost& m = ctx->N;
  hipStream_t st = (hipStream_t)stream;
  const size_t need = haflo_workspace_bytes(ctx, orientation == 0 ? HAFLO_OP_MATVEC_XT_D : HAFLO_OP_MATVEC_X_W, rows, cols);
  if (!d_workspace || workspace_bytes < need) return HAFLO_EINVAL;
  u32* ws = (u32*)d_workspace;
  const bool buckets = orientation == 0 && use_buckets(ctx, rows, cols);
  int rc = buckets ? HAFLO_OK
                   : launch_maxmag(ctx, d_X, rows * cols, ws, orientation == 0 ? 2 : (int)(kXwBinsAt + kLenBins), st);
  if (rc != HAFLO_OK) return rc;
  const int nbatch = inverse_batches(ctx);
  if (buckets) {
    const XtdBucketLayout l = xtd_bucket_layout(ctx, rows, cols);
    u32* P = ws + l.off_P;
    rc = xtd_buckets(ctx, (const u32*)d_c, d_X, rows, cols, ws + l.off_ws, P, st);
    if (rc != HAFLO_OK) return rc;
    const LaunchShape sh = latency_shape(ctx, cols, m);
#define CALL(LPT, T) HAFLO_LAUNCH((k_xtd_finish<LPT, T>), sh, st, m.ref(), ctx->Nw.ref(), cols, (const u32*)P, (u32*)d_out, nbatch)
    HAFLO_DISPATCH_SHAPE(sh, m, CALL);
#undef CALL
  } else if (orientation == 0) {
    const XtdPlan p = xtd_plan(ctx, rows, cols);
    u32* tables = ws + p.off_tables;
    u32* partials = ws + p.off_partials;
    u32* P = ws + p.off_P;
    if (rows) {
      rc = power_tables(ctx, (const u32*)d_c, tables, kSEntries, rows, st);
      if (rc != HAFLO_OK) return rc;
      LaunchShape mainsh;
      mainsh.threads = kBlockThreads;
      mainsh.gpb = kBlockThreads / m.t;
      mainsh.blocks = (int)(cols * ((((size_t)p.rsplit * kSMaxPos) + 7) / 8 * 8));
#define CALL(LPT, T) \
  HAFLO_LAUNCH((k_xtd_main<LPT, T>), mainsh, st, m.ref(), d_X, rows, cols, (const u32*)tables, p.rsplit, partials, (const u32*)ws)
      HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
    }
    {
      const bool wide = haflo::few_groups(ctx, cols * 2);
      const LaunchShape sh = launch_shape(ctx, cols * 2, wide ? haflo_wide_lanes(m) : m.t, 8);
#define CALL(LPT, T) \
  HAFLO_LAUNCH((k_xtd_horner<LPT, T>), sh, st, m.ref(), cols, p.rsplit, (const u32*)partials, P, (const u32*)ws)
      if (wide) { HAFLO_DISPATCH_GEOMETRY_WIDE(m, CALL); } else { HAFLO_DISPATCH_GEOMETRY(m, CALL); }
#undef CALL
    }
    {
      const LaunchShape sh = latency_shape(ctx, cols, m);
#define CALL(LPT, T) HAFLO_LAUNCH((k_xtd_finish<LPT, T>), sh, st, m.ref(), ctx->Nw.ref(), cols, (const u32*)P, (u32*)d_out, nbatch)
      HAFLO_DISPATCH_SHAPE(sh, m, CALL);
#undef CALL
    }
  } else {
    const XwPlan p = xw_plan(ctx, rows, cols);
    u32* inv = ws + p.off_inv;
    u32* tables = ws + p.off_tables;
    u32* lists = ws + p.off_nz;
    u32* cnt = ws + p.off_cnt;
    // The tables and the row products are in the pair form modulo n (5/8 of the limb products of a full-length
    // product; every supported key size has that geometry); a row's result leaves it as it is stored.
    const ModHost& mh = ctx->Nh;
    if (!haflo_has_pair_geometry(mh)) return HAFLO_EINVAL;
    const ModRef M = mh.ref();
    const int lanes = 2 * mh.t;
    const u32* one = mh.d_pairs + (size_t)kConstR1 * 2 * mh.nl;
    const u32* leave = mh.d_pairs + (size_t)kConstR3 * 2 * mh.nl;
    if (cols) {
      rc = invert_batch(ctx, (const u32*)d_c, inv, cols, st);
      if (rc != HAFLO_OK) return rc;
      {
        const LaunchShape sh = launch_shape(ctx, cols * 2 * kMaxPos, lanes, 8);
#define CALL(LPT, T)                                                                                                \
  HAFLO_LAUNCH((k_xw_positions<LPT, T, true>), sh, st, M, (const u32*)(mh.d_pairs + (size_t)kConstR4 * 2 * mh.nl), \
               (const u32*)(mh.d_pairs + (size_t)kConstR5 * 2 * mh.nl), (const u32*)d_c, (const u32*)inv, cols,     \
               tables, (const u32*)ws)
        HAFLO_DISPATCH_PAIRS(mh, CALL);
#undef CALL
      }
      for (int B = 1; B < kWinEntries; B *= 2) {
        const size_t groups = cols * 2 * kMaxPos * (size_t)std::min(B, kWinEntries - 1 - B);
        const LaunchShape sh = launch_shape(ctx, groups, lanes, 8);
#define CALL(LPT, T) HAFLO_LAUNCH((k_xw_level<LPT, T, true>), sh, st, M, one, cols, B, tables, (const u32*)ws)
        HAFLO_DISPATCH_PAIRS(mh, CALL);
#undef CALL
      }
    }
    u32* bins = ws + kXwBinsAt;
    u32* order = ws + p.off_order;
    {
      const LaunchShape sh = launch_shape(ctx, rows, 64, 8);
      HAFLO_LAUNCH(k_xw_lists, sh, st, d_X, rows, cols, lists, cnt, (const u32*)ws);
      LaunchShape per_row, single;
      per_row.threads = single.threads = kBlockThreads;
      per_row.gpb = single.gpb = kBlockThreads;
      per_row.blocks = (int)std::min((rows + kBlockThreads - 1) / kBlockThreads, (size_t)ctx->num_cu * 8);
      single.blocks = 1;
      HAFLO_LAUNCH(k_xw_order<false>, per_row, st, (const u32*)cnt, rows, cols, bins, order, (const u32*)ws);
      HAFLO_LAUNCH(k_xw_order_scan, single, st, bins);
      HAFLO_LAUNCH(k_xw_order<true>, per_row, st, (const u32*)cnt, rows, cols, bins, order, (const u32*)ws);
    }
    u32* partial = ws + p.off_partial;
    {
      const LaunchShape sh = launch_shape(ctx, rows << p.seg_shift, lanes, 3);
#define CALL(LPT, T)                                                                                            \
  HAFLO_LAUNCH((k_xw_main<LPT, T, true>), sh, st, M, one, leave, rows, cols * (size_t)kMaxPos, (const u32*)lists, \
               (const u32*)cnt, (const u32*)order, (const u32*)tables, ws + 1, p.seg_shift, partial, (u32*)d_out)
      HAFLO_DISPATCH_PAIRS(mh, CALL);
#undef CALL
    }
    if (p.seg_shift) {
      const LaunchShape sh = launch_shape(ctx, rows, lanes, 8);
#define CALL(LPT, T) \
  HAFLO_LAUNCH((k_xw_combine<LPT, T, true>), sh, st, M, leave, rows, p.seg_shift, (const u32*)partial, (u32*)d_out)
      HAFLO_DISPATCH_PAIRS(mh, CALL);
#undef CALL
    }
  }
  return hip_status(hipGetLastError());
}

int haflo_cipher_sum(const haflo_ctx* ctx, const void* d_c, size_t count, void* d_out, void* d_workspace,
                     size_t workspace_bytes, void* stream) {
  if (!ctx || !d_out || (count && !d_c)) return HAFLO_EINVAL;
  const ModHost& m = ctx->N;
  hipStream_t st = (hipStream_t)stream;
  const int nb = sum_blocks(ctx, count);
  // partial products of the first level, then of every further level, ping-pong in the workspace
  const int gpw = kBlockThreads / haflo_wide_lanes(m);  // groups per block of the later levels
  const size_t second = (size_t)(nb + gpw - 1) / gpw;
  if (!d_workspace || workspace_bytes < ((size_t)nb + second) * m.nl * 4) return HAFLO_EINVAL;
  u32* buf[2] = {(u32*)d_workspace, (u32*)d_workspace + (size_t)nb * m.nl};
  LaunchShape sh;
  sh.threads = kBlockThreads;
  sh.gpb = kBlockThreads / m.t;
  sh.blocks = nb;
  if (nb == 1) {
#define CALL(LPT, T) HAFLO_LAUNCH((k_sum<LPT, T>), sh, st, m.ref(), (const u32*)d_c, count, (u32*)d_out, 1)
    HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
    return hip_status(hipGetLastError());
  }
#define CALL(LPT, T) HAFLO_LAUNCH((k_sum<LPT, T>), sh, st, m.ref(), (const u32*)d_c, count, buf[0], 0)
  HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  // Further levels: one partial per lane group and a tree inside the block, in the wide geometry
  // (few integers are left and every level is a chain of only log2(groups) + 1 products).
  size_t n = (size_t)nb;
  int from = 0;
  while (n > 1) {
    LaunchShape lv;
    lv.threads = kBlockThreads;
    lv.gpb = gpw;
    lv.blocks = (int)((n + gpw - 1) / gpw);
    const bool last = lv.blocks == 1;
    u32* dst = last ? (u32*)d_out : buf[from ^ 1];
    const u32* src = buf[from];
#define CALL(LPT, T) HAFLO_LAUNCH((k_sum<LPT, T>), lv, st, m.ref(), src, n, dst, last ? 1 : 0)
    HAFLO_DISPATCH_GEOMETRY_WIDE(m, CALL);
#undef CALL
    n = (size_t)lv.blocks;
    from ^= 1;
  }
  return hip_status(hipGetLastError());
}

int haflo_cipher_sum_segments(const haflo_ctx* ctx, const void* d_c, size_t count, const uint32_t* d_offsets,
                              size_t nseg, void* d_out, uint32_t* d_status, void* d_workspace, size_t workspace_bytes,
                              void* stream) {
  if (!ctx || count >= (1ull << 32) || nseg >= (1ull << 24)) return HAFLO_EINVAL;
  if (nseg == 0) return HAFLO_OK;
  if (!d_offsets || !d_out || (count && !d_c)) return HAFLO_EINVAL;
  if (!d_workspace || workspace_bytes < seg_sum_plan(ctx, count, nseg).total * 4) return HAFLO_EINVAL;
  return seg_sum(ctx, (const u32*)d_c, d_offsets, count, nseg, (u32*)d_out, d_status, (u32*)d_workspace,
                 (hipStream_t)stream);
}

}  // extern "C"
