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
  unsigned block, nblocks;  // this block's index among the blocks that share the batch
  __device__ __forceinline__ Batch() : Batch(blockIdx.x, gridDim.x) {}
  __device__ __forceinline__ Batch(unsigned block_, unsigned nblocks_) : block(block_), nblocks(nblocks_) {
    gpb = (int)blockDim.x / Grp<T>::kPitch;
    gib = (int)threadIdx.x / Grp<T>::kPitch;
  }
  __device__ __forceinline__ size_t first() const { return (size_t)block * gpb; }
  __device__ __forceinline__ size_t stride() const { return (size_t)nblocks * gpb; }
  // index of this group's private slot in a per-launch workspace
  __device__ __forceinline__ size_t slot() const { return (size_t)block * gpb + gib; }
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

// largest value of `m` over the wavefront, bit by bit from the top: keep the lanes that still can hold it
__device__ __forceinline__ u32 wave_max(u32 m) {
  u32 best = 0;
  bool cand = true;
#pragma unroll 1
  for (int b = 31; b >= 0; --b) {
    bool has = cand && ((m >> b) & 1u);
    if (__builtin_amdgcn_ballot_w64(has) != 0ull) {
      best |= 1u << b;
      cand = has;
    }
  }
  return best;
}

// Program storage for the exponentiation engine: a device array for long
// programs (key-length exponents), an array inside the kernel arguments for
// short ones (64-bit exponents), so that no device memory has to be allocated
// or written for a per-call exponent.
struct ProgPtr {
  const u32* ins;
  int len;
  __device__ __forceinline__ u32 at(int pc) const { return ins[pc]; }
};
constexpr int kInlineProgMax = 192;
struct ProgInline {
  u32 ins[kInlineProgMax];
  int len;
  __device__ __forceinline__ u32 at(int pc) const { return ins[pc]; }
};

// Operands of one engine launch (all device pointers; unused ones may be null).
struct EngineIO {
  const u32* constant[kNumConst];  // per-modulus limb arrays, see kConst*
  const u32* in_words[2];          // per-element arrays of in_nwords 32-bit words
  int in_nwords;
  const u32* in_limbs;             // per-element limb arrays, in_limbs_stride limbs apart
  int in_limbs_stride;
  int in_limbs_valid;              // limbs an element's array holds (read as zero above); 0 = as many as asked for
  const unsigned long long* k64;   // per-element exponent for the *_TD instructions
  u32* out;                        // NL limbs per element (canonical) or null
  u32* tables;                     // table_entries * NL limbs per slot
  int table_entries;
  int table_per_item;              // 1: slot = element index (tables are an output), 0: slot = lane group
  size_t first;                    // index of the launch's first element in the per-element arrays
  int out_mode;                    // pair engine: what is stored, see kOut*
};

// The exponentiation engine: every lane group runs the batch-uniform program
// `P` on its element. All Montgomery products of all operators built on it go
// through the one unrolled loop instantiated here, which keeps the register
// footprint at what a single product needs.
template <int LPT, int T, class Prog>
__device__ __forceinline__ void engine_run(const ModRef& M, const Prog& P, const EngineIO& io, size_t count,
                                           unsigned block, unsigned nblocks) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt(block, nblocks);
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    const bool active = base + bt.gib < count;
    const size_t item = io.first + base + bt.gib;
    const bool tab_ok = active || !io.table_per_item;
    u32* table = io.tables + (io.table_per_item ? (active ? item : 0) : bt.slot()) * (size_t)io.table_entries * NL;
    const u64 k = (io.k64 && active) ? io.k64[item] : 0ull;
    u32 acc[LPT];
    zero_limbs<LPT>(acc);
#pragma unroll 1
    for (int pc = 0; pc < P.len; ++pc) {
      const u32 ins = P.at(pc);
      const u32 op = ins & 0xFFu, a = (ins >> 8) & 0xFFFu, b = ins >> 20;
      if (op >= ENG_LOAD_T) {
        if (op == ENG_STORE_T) {
          if (tab_ok) store_limbs<LPT, T>(table + (size_t)a * NL, acc, g);
        } else if (op == ENG_LOAD_W || op == ENG_LOAD_WH) {
          if (active)
            load_words_as_limbs<LPT, T>(acc, io.in_words[a] + item * (size_t)io.in_nwords, io.in_nwords, g,
                                        op == ENG_LOAD_WH ? NL : 0);
          else zero_limbs<LPT>(acc);
        } else if (op == ENG_LOAD_L) {
          const u32* src = io.in_limbs + item * (size_t)io.in_limbs_stride + (size_t)a * NL;
          if (!active) zero_limbs<LPT>(acc);
          else if (io.in_limbs_valid) load_limbs_below<LPT, T>(acc, src, io.in_limbs_valid - (int)a * NL, g);
          else load_limbs<LPT, T>(acc, src, g);
        } else {
          const u32* src;
          if (op == ENG_LOAD_C || op == ENG_ADD_C) src = io.constant[a];
          else src = table + (size_t)(op == ENG_LOAD_TD ? (u32)(k >> a) & 15u : a) * NL;
          u32 t[LPT];
          if (tab_ok || op == ENG_LOAD_C || op == ENG_ADD_C) load_limbs<LPT, T>(t, src, g);
          else zero_limbs<LPT>(t);
          if (op == ENG_ADD_C || op == ENG_ADD_T) {
#pragma unroll
            for (int j = 0; j < LPT; ++j) acc[j] += t[j];
            partial_norm<LPT, T>(acc, g);
          } else {
#pragma unroll
            for (int j = 0; j < LPT; ++j) acc[j] = t[j];
          }
        }
        continue;
      }
      if (op == ENG_SQ) {
        montsqr<LPT, T>(acc, acc, mod.n, mod.n0inv, g);
      } else {
        // the multiplier is read limb by limb straight from its table slot or constant array
        const u32* src;
        if (op == ENG_MUL_C) src = io.constant[a];
        else src = table + (size_t)(op == ENG_MUL_TD ? (u32)(k >> a) & 15u : a) * NL;
        if (!(tab_ok || op == ENG_MUL_C)) src = io.constant[kConstR1];
        if (Grp<T>::kWhole) {
          // a lone wavefront cannot hide a load every few steps: the lanes fetch their limbs of the
          // multiplier once (one latency per product) and the steps take them from registers
          u32 t[LPT];
          load_limbs<LPT, T>(t, src, g);
          montmul<LPT, T>(acc, acc, t, mod.n, mod.n0inv, g);
        } else {
          montmul_mem<LPT, T>(acc, acc, src, mod.n, mod.n0inv, g);
        }
      }
      if (op == ENG_MUL_T_ST && tab_ok) store_limbs<LPT, T>(table + (size_t)b * NL, acc, g);
    }
    if (io.out) {
      canonicalise<LPT, T>(acc, mod.n, g);
      if (active) store_limbs<LPT, T>(io.out + item * (size_t)NL, acc, g);
    }
  }
}

template <int LPT, int T, class Prog>
__global__ __launch_bounds__(kBlockThreads, 4) void k_engine(ModRef M, Prog P, EngineIO io, size_t count) {
  engine_run<LPT, T, Prog>(M, P, io, count, blockIdx.x, gridDim.x);
}

// Canonical pair: x0 below s with what it exceeded s by carried into x1 (the value is x0 + s x1), then x1
// below s (it may exceed 2s by a hair after a product, or by more after the carry: two subtractions).
// Input: a lazy pair as a product leaves it.
template <int LPT, int T>
__device__ __forceinline__ void pair_canonical(u32 (&x0)[LPT], u32 (&x1)[LPT], const u32 (&n)[LPT], const Grp<T>& g) {
  resolve<LPT, T>(x0, g);
  s32 d[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) d[j] = (s32)x0[j] - (s32)n[j];
  const int top = resolve<LPT, T>(d, g);
  if (top >= 0) {
#pragma unroll
    for (int j = 0; j < LPT; ++j) x0[j] = (u32)d[j];
    if (g.k == 0) x1[0] += 1u;
  }
  canonicalise<LPT, T>(x1, n, g);
  canonicalise<LPT, T>(x1, n, g);
}
// The integer x0 + s x1 of a canonical pair, as its low and high NL limbs (canonical)
template <int LPT, int T>
__device__ __forceinline__ void pair_to_integer(u32 (&lo)[LPT], u32 (&hi)[LPT], const u32 (&x0)[LPT],
                                                const u32 (&x1)[LPT], const u32 (&n)[LPT], const Grp<T>& g) {
  mulwide<LPT, T>(lo, hi, n, x1, g);
#pragma unroll
  for (int j = 0; j < LPT; ++j) lo[j] += x0[j];
  const int carry = resolve<LPT, T>(lo, g);
  if (g.k == 0) hi[0] += (u32)carry;
  resolve<LPT, T>(hi, g);
}

// The same engine on residues modulo s^2 held as pairs of residues modulo s (pairmul_core): `M` is the
// modulus s with half the limbs of s^2; an element of the tables and of the constant arrays is
// [x0: NL limbs][x1: NL limbs]. Instructions as above, with these readings: ENG_LOAD_W is the pair (w, 0),
// ENG_LOAD_W1 the pair (1, w), i.e. 1 + s w; ENG_LOAD_L a takes limbs [a NL, (a + 1) NL) of the element's
// limb input as (l, 0). When the program ends, acc holds the result X as a pair; io.out_mode says what is
// stored: kOutInteger, the canonical integer x0 + s x1 on 2 NL limbs (low half, high half); kOutSecond, the
// canonical x1 on NL limbs, for results that are 1 modulo s (x0 = 1), whose (X - 1) / s it is.
enum { kOutInteger = 0, kOutSecond = 1 };
template <int LPT, int T, class Prog>
__device__ __forceinline__ void engine_run_pairs(const ModRef& M, const Prog& P, const EngineIO& io, size_t count,
                                                 unsigned block, unsigned nblocks) {
  constexpr int NL = LPT * T;  // limbs of s; an element has 2 NL
  Grp<T> g;
  Batch<T> bt(block, nblocks);
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    const bool active = base + bt.gib < count;
    const size_t item = io.first + base + bt.gib;
    u32* table = io.tables + bt.slot() * (size_t)io.table_entries * (2 * NL);
    const u64 k = (io.k64 && active) ? io.k64[item] : 0ull;
    u32 x0[LPT], x1[LPT];
    zero_limbs<LPT>(x0);
    zero_limbs<LPT>(x1);
#pragma unroll 1
    for (int pc = 0; pc < P.len; ++pc) {
      const u32 ins = P.at(pc);
      const u32 op = ins & 0xFFu, a = (ins >> 8) & 0xFFFu, b = ins >> 20;
      if (op == ENG_SQ) {
        pairsqr<LPT, T>(x0, x1, x0, x1, mod.n, mod.n0inv, g);
      } else if (op == ENG_MUL_T || op == ENG_MUL_T_ST || op == ENG_MUL_C || op == ENG_MUL_TD) {
        const u32* src;
        if (op == ENG_MUL_C) src = io.constant[a];
        else src = table + (size_t)(op == ENG_MUL_TD ? (u32)(k >> a) & 15u : a) * (2 * NL);
        if (Grp<T>::kWhole) {
          // a lone wavefront cannot hide a load every few steps: the lanes fetch their limbs of the
          // multiplier once and the steps take them from registers
          u32 t0[LPT], t1[LPT];
          load_limbs<LPT, T>(t0, src, g);
          load_limbs<LPT, T>(t1, src + NL, g);
          pairmul<LPT, T>(x0, x1, x0, x1, t0, t1, mod.n, mod.n0inv, g);
        } else {
          pairmul_mem<LPT, T>(x0, x1, x0, x1, src, mod.n, mod.n0inv, g);
        }
        if (op == ENG_MUL_T_ST) {
          store_limbs<LPT, T>(table + (size_t)b * (2 * NL), x0, g);
          store_limbs<LPT, T>(table + (size_t)b * (2 * NL) + NL, x1, g);
        }
      } else if (op == ENG_STORE_T) {
        store_limbs<LPT, T>(table + (size_t)a * (2 * NL), x0, g);
        store_limbs<LPT, T>(table + (size_t)a * (2 * NL) + NL, x1, g);
      } else if (op == ENG_LOAD_T || op == ENG_LOAD_C || op == ENG_LOAD_TD || op == ENG_ADD_T || op == ENG_ADD_C) {
        const u32* src;
        if (op == ENG_LOAD_C || op == ENG_ADD_C) src = io.constant[a];
        else src = table + (size_t)(op == ENG_LOAD_TD ? (u32)(k >> a) & 15u : a) * (2 * NL);
        u32 t0[LPT], t1[LPT];
        load_limbs<LPT, T>(t0, src, g);
        load_limbs<LPT, T>(t1, src + NL, g);
        if (op == ENG_ADD_T || op == ENG_ADD_C) {
#pragma unroll
          for (int j = 0; j < LPT; ++j) {
            x0[j] += t0[j];
            x1[j] += t1[j];
          }
          partial_norm<LPT, T>(x0, g);
          partial_norm<LPT, T>(x1, g);
        } else {
#pragma unroll
          for (int j = 0; j < LPT; ++j) {
            x0[j] = t0[j];
            x1[j] = t1[j];
          }
        }
      } else if (op == ENG_LOAD_W || op == ENG_LOAD_W1) {
        u32 w[LPT];
        if (active) load_words_as_limbs<LPT, T>(w, io.in_words[a] + item * (size_t)io.in_nwords, io.in_nwords, g, 0);
        else zero_limbs<LPT>(w);
#pragma unroll
        for (int j = 0; j < LPT; ++j) {
          x0[j] = op == ENG_LOAD_W ? w[j] : ((g.k == 0 && j == 0) ? 1u : 0u);
          x1[j] = op == ENG_LOAD_W ? 0u : w[j];
        }
      } else if (op == ENG_LOAD_L) {
        const u32* src = io.in_limbs + item * (size_t)io.in_limbs_stride + (size_t)a * NL;
        if (!active) zero_limbs<LPT>(x0);
        else if (io.in_limbs_valid) load_limbs_below<LPT, T>(x0, src, io.in_limbs_valid - (int)a * NL, g);
        else load_limbs<LPT, T>(x0, src, g);
        zero_limbs<LPT>(x1);
      }
    }
    pair_canonical<LPT, T>(x0, x1, mod.n, g);
    if (io.out_mode == kOutSecond) {
      if (active) store_limbs<LPT, T>(io.out + item * (size_t)NL, x1, g);
    } else {
      u32 lo[LPT], hi[LPT];
      pair_to_integer<LPT, T>(lo, hi, x0, x1, mod.n, g);
      if (active) {
        store_limbs<LPT, T>(io.out + item * (size_t)(2 * NL), lo, g);
        store_limbs<LPT, T>(io.out + item * (size_t)(2 * NL) + NL, hi, g);
      }
    }
  }
}

template <int LPT, int T, class Prog>
__global__ __launch_bounds__(kBlockThreads, 4) void k_engine_pairs(ModRef M, Prog P, EngineIO io, size_t count) {
  engine_run_pairs<LPT, T, Prog>(M, P, io, count, blockIdx.x, gridDim.x);
}

// Two independent jobs of the same geometry in one launch (the two prime-power
// branches of decryption): the first `split` blocks run job 0, the rest job 1.
struct EngineJob {
  ModRef M;
  ProgPtr P;
  EngineIO io;
};
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads, 4) void k_engine_pair(EngineJob j0, EngineJob j1, unsigned split,
                                                                  size_t count) {
  if (blockIdx.x < split) engine_run<LPT, T, ProgPtr>(j0.M, j0.P, j0.io, count, blockIdx.x, split);
  else engine_run<LPT, T, ProgPtr>(j1.M, j1.P, j1.io, count, blockIdx.x - split, gridDim.x - split);
}

// the same for the pair engine
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads, 4) void k_engine_pairs2(EngineJob j0, EngineJob j1, unsigned split,
                                                                    size_t count) {
  if (blockIdx.x < split) engine_run_pairs<LPT, T, ProgPtr>(j0.M, j0.P, j0.io, count, blockIdx.x, split);
  else engine_run_pairs<LPT, T, ProgPtr>(j1.M, j1.P, j1.io, count, blockIdx.x - split, gridDim.x - split);
}


// What the reduction kernels multiply: a Montgomery residue of LPT T limbs, or (PAIR) a residue modulo the
// square of the LPT T-limb modulus held as a pair, 2 LPT T limbs in memory ([x0][x1]), with pairmul_core's
// products. The kernels are written once against this.
template <int LPT, bool PAIR>
struct Elem {
  u32 x0[LPT];
  u32 x1[PAIR ? LPT : 1];
};
template <int LPT, int T, bool PAIR>
struct ElemOps {
  static constexpr int kLimbs = (PAIR ? 2 : 1) * LPT * T;  // limbs of an element in memory
  using E = Elem<LPT, PAIR>;
  static __device__ __forceinline__ void load(E& e, const u32* p, const Grp<T>& g) {
    load_limbs<LPT, T>(e.x0, p, g);
    if constexpr (PAIR) load_limbs<LPT, T>(e.x1, p + LPT * T, g);
  }
  static __device__ __forceinline__ void store(u32* p, const E& e, const Grp<T>& g) {
    store_limbs<LPT, T>(p, e.x0, g);
    if constexpr (PAIR) store_limbs<LPT, T>(p + LPT * T, e.x1, g);
  }
  static __device__ __forceinline__ void copy(E& d, const E& s) {
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
      d.x0[j] = s.x0[j];
      if constexpr (PAIR) d.x1[j] = s.x1[j];
    }
  }
  // one word of every cache line of the element at p, so that it is on its way while something else runs
  static __device__ __forceinline__ u32 touch(const u32* p, const Grp<T>& g) {
    u32 v = p[g.k * LPT];
    if constexpr (PAIR) v ^= p[LPT * T + g.k * LPT];
    return v;
  }
  static __device__ __forceinline__ void mul_mem(E& acc, const u32* p, const ModRegs<LPT>& mod, const Grp<T>& g) {
    if constexpr (PAIR) pairmul_mem<LPT, T>(acc.x0, acc.x1, acc.x0, acc.x1, p, mod.n, mod.n0inv, g);
    else montmul_mem<LPT, T>(acc.x0, acc.x0, p, mod.n, mod.n0inv, g);
  }
  static __device__ __forceinline__ void mul(E& acc, const E& b, const ModRegs<LPT>& mod, const Grp<T>& g) {
    if constexpr (PAIR) pairmul<LPT, T>(acc.x0, acc.x1, acc.x0, acc.x1, b.x0, b.x1, mod.n, mod.n0inv, g);
    else montmul<LPT, T>(acc.x0, acc.x0, b.x0, mod.n, mod.n0inv, g);
  }
  static __device__ __forceinline__ void sqr(E& acc, const ModRegs<LPT>& mod, const Grp<T>& g) {
    if constexpr (PAIR) pairsqr<LPT, T>(acc.x0, acc.x1, acc.x0, acc.x1, mod.n, mod.n0inv, g);
    else montsqr<LPT, T>(acc.x0, acc.x0, mod.n, mod.n0inv, g);
  }
};


// A stored ciphertext (Montgomery form modulo n^2 at the full radix R_N, 2 LPT T limbs at `w`) into the pair
// form modulo n (Montgomery form at the half radix R): W = w_lo + R w_hi goes to
// (w_lo, 0) k_lo + (w_hi, 0) k_hi with the pair constants k_lo = R^2 / R_N and k_hi = R^3 / R_N. The result is
// lazy (each half below 4n, limbs partially normalised), which is what a product takes.
template <int LPT, int T>
__device__ __forceinline__ void to_pair(u32 (&x0)[LPT], u32 (&x1)[LPT], const u32* w, const u32* k_lo, const u32* k_hi,
                                        const ModRegs<LPT>& mod, const Grp<T>& g) {
  constexpr int NLH = LPT * T;
  u32 b0[LPT], b1[LPT];
  load_limbs<LPT, T>(x0, w, g);
  load_limbs<LPT, T>(b0, w + NLH, g);
  zero_limbs<LPT>(x1);
  zero_limbs<LPT>(b1);
  pairmul_mem<LPT, T>(x0, x1, x0, x1, k_lo, mod.n, mod.n0inv, g);
  pairmul_mem<LPT, T>(b0, b1, b0, b1, k_hi, mod.n, mod.n0inv, g);
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    x0[j] += b0[j];
    x1[j] += b1[j];
  }
  partial_norm<LPT, T>(x0, g);
  partial_norm<LPT, T>(x1, g);
}
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads, 4) void k_to_pairs(ModRef M, const u32* __restrict__ k_lo,
                                                               const u32* __restrict__ k_hi,
                                                               const u32* __restrict__ in, size_t count,
                                                               u32* __restrict__ out) {
  constexpr int NLH = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    const size_t it = base + bt.gib;
    const bool active = it < count;
    u32 a0[LPT], a1[LPT];
    to_pair<LPT, T>(a0, a1, in + (active ? it : 0) * (size_t)(2 * NLH), k_lo, k_hi, mod, g);
    if (active) {
      store_limbs<LPT, T>(out + it * (size_t)(2 * NLH), a0, g);
      store_limbs<LPT, T>(out + it * (size_t)(2 * NLH) + NLH, a1, g);
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

// The same dispatch for the short, latency-bound kernels at the end of a reduction, where only a
// few big integers are left: spread each over twice the lanes (9 limbs per lane) so that a single
// product finishes sooner. The limb arrays in memory are the same for both geometries.
#define HAFLO_DISPATCH_GEOMETRY_WIDE(m, CALL)                     \
  do {                                                            \
    if ((m).lpt == 18 && (m).t == 1) { CALL(9, 2); }              \
    else if ((m).lpt == 18 && (m).t == 2) { CALL(9, 4); }         \
    else if ((m).lpt == 18 && (m).t == 4) { CALL(9, 8); }         \
    else if ((m).lpt == 18 && (m).t == 8) { CALL(9, 16); }        \
    else if ((m).lpt == 18 && (m).t == 16) { CALL(18, 16); }      \
    else if ((m).lpt == 9 && (m).t == 1) { CALL(9, 1); }          \
    else return HAFLO_EINVAL;                                     \
  } while (0)
// The pair arithmetic modulo the square of `mh` (18 limbs per lane as a plain modulus): 9 limbs of each half
// per lane on twice the lanes. Expands `CALL(9, T)`.
#define HAFLO_DISPATCH_PAIRS(mh, CALL)                            \
  do {                                                            \
    if ((mh).lpt == 18 && (mh).t == 1) { CALL(9, 2); }            \
    else if ((mh).lpt == 18 && (mh).t == 2) { CALL(9, 4); }       \
    else if ((mh).lpt == 18 && (mh).t == 4) { CALL(9, 8); }       \
    else if ((mh).lpt == 18 && (mh).t == 8) { CALL(9, 16); }      \
    else return HAFLO_EINVAL;                                     \
  } while (0)
inline bool haflo_has_pair_geometry(const haflo::ModHost& mh) { return mh.d_pairs && mh.lpt == 18 && mh.t <= 8; }
// The same dispatch for batches of at most one big integer per SIMD, where the latency of one product is all
// that counts: one integer per wavefront on 18 to 48 lanes with 2 to 6 limbs each (steps of a dozen
// instructions instead of two to four dozen). Moduli without such a geometry take the wide one.
#define HAFLO_DISPATCH_GEOMETRY_WAVE(m, CALL)                     \
  do {                                                            \
    if ((m).nl == 36) { CALL(2, 18); }                            \
    else if ((m).nl == 72) { CALL(2, 36); }                       \
    else if ((m).nl == 144) { CALL(3, 48); }                      \
    else if ((m).nl == 288) { CALL(6, 48); }                      \
    else HAFLO_DISPATCH_GEOMETRY_WIDE(m, CALL);                   \
  } while (0)
inline bool haflo_has_wave_geometry(const haflo::ModHost& m) { return m.nl == 36 || m.nl == 72 || m.nl == 144 || m.nl == 288; }
// true when so few big integers are in flight that the chip is mostly idle anyway
namespace haflo {
inline bool few_groups(const haflo_ctx* ctx, size_t groups, int per_cu = 8) {
  return groups <= (size_t)ctx->num_cu * (size_t)per_cu;
}
}
// lanes per big integer under HAFLO_DISPATCH_GEOMETRY_WIDE
inline int haflo_wide_lanes(const haflo::ModHost& m) { return (m.lpt == 18 && m.t < 16) ? 2 * m.t : m.t; }
