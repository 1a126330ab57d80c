// X^T [[d]] for tall matrices by the bucket method: no per-base tables, one
// Montgomery product per non-zero exponent digit.
//
// Every |x_ij| is read in signed base-1024 digits (|x| = sum_s d_s 1024^s,
// d_s in [-512, 511]). For output column j, digit position s and effective sign
// (sign of x_ij times sign of d_s), the rows whose digit has magnitude m form
// the bucket (j, s, sign, m); with B = product of c_i over a bucket,
//   out_j = P_j[+] / P_j[-],  P_j[sg] = prod_s ( prod_m B(j,s,sg,m)^m )^(1024^s).
// Steps:
//   1. count the bucket sizes, prefix-sum them, scatter the row indices into
//      one array sorted by bucket (atomics; the order inside a bucket is
//      arbitrary and does not change the canonical result);
//   2. reduce every bucket to its product in rounds: a round cuts each bucket's
//      items into chunks of at most 16 or 32, one lane group multiplies one chunk,
//      the chunk products are the next round's items. A bucket of any size (a
//      column of equal entries puts all its rows into one) is spread over the
//      whole chip, and the number of rounds is fixed by the row count;
//   3. prod_m B_m^m with m = 32 h + (l + 1): 16 + 32 sub-products over h and l,
//      two running products, five squarings;
//   4. Horner over the digit positions, and P[+] * P[-]^-1 by the caller.
#include "kernels_common.hpp"

#include <algorithm>

using namespace haflo;
using namespace haflo::dev;

namespace {

constexpr int kDigitBits = 10;
constexpr int kMags = 512;     // digit magnitudes 1..512
constexpr int kMaxPos = 4;     // 1024^4 - offset(4) > 2^31
// Items per lane group and round: 2^cb with cb chosen per call (chunk_bits): long chunks for matrices that fill
// the chip many times over (fewer items for the later rounds), short ones where the longest chain of products is
// what the call waits for.
constexpr int kChunkBitsMin = 4, kChunkBitsMax = 5, kChunkMax = 1 << kChunkBitsMax;
constexpr int kLoCount = 32, kHiCount = 16, kSubProducts = kLoCount + kHiCount;  // m = 32 h + l + 1

__host__ __device__ inline unsigned long long digit_offset(int npos) {
  unsigned long long c = 0;
  for (int s = 0; s < npos; ++s) c = c * 1024ull + 512ull;
  return c;
}
// positions needed so that maxmag + offset(S) < 1024^S (0 for an all-zero matrix)
__host__ __device__ inline int digit_positions(unsigned maxmag) {
  if (maxmag == 0) return 0;
  for (int s = 1; s < kMaxPos; ++s)
    if ((unsigned long long)maxmag + digit_offset(s) < (1ull << (kDigitBits * s))) return s;
  return kMaxPos;
}
__global__ __launch_bounds__(kBlockThreads) void k_bk_zero(u32* p, size_t n) {
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += (size_t)gridDim.x * blockDim.x) p[i] = 0u;
}

// Words of the statistics block at the start of the workspace (zeroed with the counters): the largest
// magnitude and bucket, the chunk counter of every round, and for the rounds that hand their chunks out in
// the order of their lengths (k_bk_order) the length classes: kOrdClasses counts, then as many cursors.
constexpr int kOrdRounds = 2, kOrdClasses = 64;
enum { kStatMaxMag = 0, kStatMaxCount = 1, kStatNextChunk = 2, kStatOrder = 16,
       kStatWords = kStatOrder + kOrdRounds * 2 * kOrdClasses };

// Every non-zero digit of every entry, always over kMaxPos positions (positions above the largest
// magnitude only hold zero digits). A block takes kTermRows rows of one column and counts its digits in
// LDS first, so that global memory sees one atomic per bucket and block instead of one per digit.
// SCATTER = false: cnt[key] += bucket sizes, stats[kStatMaxMag] = largest |x|.
// SCATTER = true: cnt[] are running cursors (zero at launch); the block reserves its share of every
// bucket with one atomic, then writes sorted[off[key] + reserved + rank inside the block] = row.
constexpr int kTermRows = 8192;
constexpr int kLocalKeys = kMaxPos * 2 * kMags;  // buckets of one column
template <bool SCATTER>
__global__ __launch_bounds__(kBlockThreads) void k_bk_terms(const int* __restrict__ X, size_t rows, size_t cols,
                                                            u32* __restrict__ cnt, const u32* __restrict__ off,
                                                            u32* __restrict__ sorted, u32* __restrict__ stats) {
  __shared__ u32 hist[kLocalKeys];
  __shared__ u32 reserved[SCATTER ? kLocalKeys : 1];
  const unsigned long long offset = digit_offset(kMaxPos);
  const size_t j = (size_t)blockIdx.x % cols;
  const size_t r0 = ((size_t)blockIdx.x / cols) * kTermRows;
  const size_t r1 = r0 + kTermRows < rows ? r0 + kTermRows : rows;
  for (int l = (int)threadIdx.x; l < kLocalKeys; l += kBlockThreads) hist[l] = 0u;
  __syncthreads();
  // local bucket index (position * 2 + sign) * 512 + magnitude - 1 of digit s of entry x, or -1
  auto local_key = [&](int x, int s) -> int {
    const u32 mag = x < 0 ? 0u - (u32)x : (u32)x;
    const int d = (int)((((unsigned long long)mag + offset) >> (s * kDigitBits)) & 1023ull) - 512;
    if (d == 0) return -1;
    const int negative = ((x < 0) != (d < 0)) ? 1 : 0;
    return (s * 2 + negative) * kMags + (d < 0 ? -d : d) - 1;
  };
  auto global_key = [&](int l) -> size_t {
    const int s = l / (2 * kMags), rest = l - s * 2 * kMags;
    return (((size_t)s * cols + j) * 2) * (size_t)kMags + (size_t)rest;
  };
  u32 largest = 0;
  for (size_t i = r0 + threadIdx.x; i < r1; i += kBlockThreads) {
    const int x = X[i * cols + j];
    if (x == 0) continue;
    const u32 mag = x < 0 ? 0u - (u32)x : (u32)x;
    largest = mag > largest ? mag : largest;
    for (int s = 0; s < kMaxPos; ++s) {
      const int l = local_key(x, s);
      if (l >= 0) atomicAdd(&hist[l], 1u);
    }
  }
  __syncthreads();
  for (int l = (int)threadIdx.x; l < kLocalKeys; l += kBlockThreads) {
    const u32 c = hist[l];
    if (c == 0u) continue;
    const u32 before = atomicAdd(&cnt[global_key(l)], c);
    if (SCATTER) {
      reserved[l] = before;
      hist[l] = 0u;  // from here on the rank inside the block
    }
  }
  if (!SCATTER) {
    largest = wave_max(largest);
    if ((threadIdx.x & (WAVE - 1)) == 0 && largest) atomicMax(&stats[kStatMaxMag], largest);
    return;
  }
  __syncthreads();
  for (size_t i = r0 + threadIdx.x; i < r1; i += kBlockThreads) {
    const int x = X[i * cols + j];
    if (x == 0) continue;
    for (int s = 0; s < kMaxPos; ++s) {
      const int l = local_key(x, s);
      if (l < 0) continue;
      const u32 rank = atomicAdd(&hist[l], 1u);
      sorted[(size_t)off[global_key(l)] + reserved[l] + rank] = (u32)i;
    }
  }
}

// Items of a key with `c` rows at the start of round r: ceil(c / 2^(cb r)).
__host__ __device__ inline u32 items_at(u32 c, int r, int cb) {
  const int sh = cb * r;
  return sh >= 32 ? (c != 0u) : (u32)(((u64)c + ((1ull << sh) - 1ull)) >> sh);
}

// Rounds that have work when the largest bucket holds `largest` rows: round 0, then every round that
// still finds a key with more than one item.
__host__ __device__ inline int rounds_run(u32 largest, int cb) {
  int r = 1;
  while (items_at(largest, r, cb) > 1u) ++r;
  return r;
}

// Exclusive prefix sums over the keys, for all rounds at once: component 0 of key k is its row count
// (offsets into the sorted row array), component r + 1 its number of chunks in round r
// (= its items at round r + 1). Two kernels: per-block totals, then every block adds up the totals
// before it and scans its own kScanKeys keys. offs: (rounds + 1) arrays of K + 1 words.
constexpr int kScanThreads = 256, kScanPer = 8, kScanKeys = kScanThreads * kScanPer;
constexpr int kMaxComp = 9;  // 16^8 = 2^32 bounds the rounds

// sum over the block of v, returned to every thread (red: kScanThreads words)
__device__ __forceinline__ u32 block_sum(u32 v, u32* red) {
  __syncthreads();
  red[threadIdx.x] = v;
  __syncthreads();
  for (int step = kScanThreads >> 1; step >= 1; step >>= 1) {
    if ((int)threadIdx.x < step) red[threadIdx.x] += red[threadIdx.x + step];
    __syncthreads();
  }
  return red[0];
}

__global__ __launch_bounds__(kScanThreads) void k_bk_scan_totals(const u32* __restrict__ cnt, size_t K, int ncomp,
                                                                int cb, u32* __restrict__ totals,
                                                                u32* __restrict__ stats) {
  __shared__ u32 red[kScanThreads];
  u32 mine[kMaxComp];
  for (int c = 0; c < kMaxComp; ++c) mine[c] = 0u;
  const size_t k0 = ((size_t)blockIdx.x * kScanThreads + threadIdx.x) * kScanPer;
  u32 largest = 0;
  for (int i = 0; i < kScanPer; ++i) {
    const u32 n = (k0 + i < K) ? cnt[k0 + i] : 0u;
    largest = n > largest ? n : largest;
    for (int c = 0; c < ncomp; ++c) mine[c] += items_at(n, c, cb);
  }
  largest = wave_max(largest);
  if ((threadIdx.x & (WAVE - 1)) == 0 && largest) atomicMax(&stats[kStatMaxCount], largest);
  for (int c = 0; c < ncomp; ++c) {
    u32 t = block_sum(mine[c], red);
    if (threadIdx.x == 0) totals[(size_t)c * gridDim.x + blockIdx.x] = t;
  }
}

__global__ __launch_bounds__(kScanThreads) void k_bk_scan_final(const u32* __restrict__ cnt, size_t K, int ncomp,
                                                               int cb, const u32* __restrict__ totals,
                                                               u32* __restrict__ offs) {
  __shared__ u32 red[kScanThreads];
  __shared__ u32 scan[kScanThreads];
  const size_t k0 = ((size_t)blockIdx.x * kScanThreads + threadIdx.x) * kScanPer;
  u32 n[kScanPer];
  for (int i = 0; i < kScanPer; ++i) n[i] = (k0 + i < K) ? cnt[k0 + i] : 0u;
  for (int c = 0; c < ncomp; ++c) {
    u32 before = 0;
    for (unsigned b = threadIdx.x; b < blockIdx.x; b += kScanThreads) before += totals[(size_t)c * gridDim.x + b];
    before = block_sum(before, red);
    u32 mine = 0;
    for (int i = 0; i < kScanPer; ++i) mine += items_at(n[i], c, cb);
    // Hillis-Steele inclusive scan of the per-thread sums
    scan[threadIdx.x] = mine;
    __syncthreads();
    for (int step = 1; step < kScanThreads; step <<= 1) {
      u32 add = ((int)threadIdx.x >= step) ? scan[threadIdx.x - step] : 0u;
      __syncthreads();
      scan[threadIdx.x] += add;
      __syncthreads();
    }
    u32 run = before + scan[threadIdx.x] - mine;
    u32* dst = offs + (size_t)c * (K + 1);
    for (int i = 0; i < kScanPer; ++i) {
      if (k0 + i < K) dst[k0 + i] = run;
      run += items_at(n[i], c, cb);
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == kScanThreads - 1) dst[K] = run;
    __syncthreads();
  }
}

// Chunk q of a round: its key (the one with choff[key] <= q < choff[key + 1]), and which part of the key's
// items it takes: near-equal shares of at most 2^cb.
struct ChunkAt {
  size_t key;
  u32 begin, len;
};
__device__ __forceinline__ ChunkAt chunk_at(u32 q, bool active, const u32* __restrict__ cnt,
                                            const u32* __restrict__ choff, size_t K, int round, int cb) {
  const u32 qq = active ? q : 0u;
  size_t lo = 0, hi = K;
  while (hi - lo > 1) {
    size_t mid = (lo + hi) >> 1;
    if (choff[mid] <= qq) lo = mid;
    else hi = mid;
  }
  const u32 first_chunk = choff[lo], nc = choff[lo + 1] - first_chunk, n = items_at(cnt[lo], round, cb);
  const u32 cc = qq - first_chunk;
  ChunkAt c = {lo, 0u, 0u};
  if (active && nc != 0u) {
    c.begin = (u32)(((u64)n * cc) / nc);
    c.len = (u32)(((u64)n * (cc + 1u)) / nc) - c.begin;  // at most 2^cb
  }
  return c;
}

// The chunks of a round in the order of their lengths, longest first: the lane groups of a wavefront multiply
// their chunks in lock-step up to the longest of them, so chunks of one length side by side leave no product
// slot empty (in consecutive order about 15 % of the first round's slots and a third of the second's are
// padding at 64 rows per bucket).
// A counting sort over the 2^cb lengths in two passes: SCATTER = false counts the classes into bins[0 ..
// kOrdClasses); SCATTER = true reserves places through the cursors bins[kOrdClasses ..) and writes
// order[place] = chunk. A block takes 256 chunks at a time and counts in LDS first.
template <bool SCATTER>
__global__ __launch_bounds__(kBlockThreads) void k_bk_order(const u32* __restrict__ cnt,
                                                            const u32* __restrict__ choff, size_t K, int round,
                                                            int cb, u32* __restrict__ stats,
                                                            u32* __restrict__ order) {
  static_assert(kChunkMax < kOrdClasses, "one class per chunk length");
  __shared__ u32 hist[kOrdClasses];
  __shared__ u32 start[kOrdClasses];
  if (round >= rounds_run(stats[kStatMaxCount], cb)) return;
  u32* bins = stats + kStatOrder + round * 2 * kOrdClasses;
  const u32 total = choff[K];
  for (u32 q0 = blockIdx.x * kBlockThreads; q0 < total; q0 += gridDim.x * kBlockThreads) {
    if (threadIdx.x < kOrdClasses) hist[threadIdx.x] = 0u;
    __syncthreads();
    const u32 q = q0 + threadIdx.x;
    const bool active = q < total;
    const u32 cls = (1u << cb) - chunk_at(q, active, cnt, choff, K, round, cb).len;  // 0: the longest
    const u32 rank = active ? atomicAdd(&hist[cls], 1u) : 0u;
    __syncthreads();
    if (threadIdx.x < kOrdClasses && hist[threadIdx.x] != 0u) {
      const u32 l = threadIdx.x;
      const u32 before = atomicAdd(&bins[(SCATTER ? kOrdClasses : 0) + l], hist[l]);
      if (SCATTER) {
        u32 first = 0;
        for (u32 i = 0; i < l; ++i) first += bins[i];
        start[l] = first + before;
      }
    }
    if (SCATTER) {
      __syncthreads();
      if (active) order[start[cls] + rank] = q;
    }
    __syncthreads();
  }
}

// Reduction round `round`. Key k owns items [off[k], off[k] + items_at(cnt[k], round, cb)) and is cut into
// choff[k+1] - choff[k] chunks of near-equal size; chunk q's product goes to out[q]. FIRST: item t is the
// ciphertext of row sorted[t]; otherwise item t is in[t]. PAIR: the items are pairs modulo M (see Elem);
// `one` is the Montgomery one in the items' form. `order`: the chunks in the order in which they are handed
// out (k_bk_order), or null for 0, 1, 2, ...
template <int LPT, int T, bool FIRST, bool PAIR>
__global__ __launch_bounds__(kBlockThreads, 3) void k_bk_round(ModRef M, const u32* __restrict__ one,
                                                            const u32* __restrict__ in,
                                                            const u32* __restrict__ sorted,
                                                            const u32* __restrict__ cnt,
                                                            const u32* __restrict__ off,
                                                            const u32* __restrict__ choff, size_t K,
                                                            int round, int cb, u32* __restrict__ stats,
                                                            const u32* __restrict__ order,
                                                            u32* __restrict__ out) {
  using Ops = ElemOps<LPT, T, PAIR>;
  constexpr int EL = Ops::kLimbs;
  constexpr int GW = WAVE / T;                 // lane groups per wavefront
  constexpr int IDX = (kChunkMax + T - 1) / T;  // row indices each lane keeps for its group's chunk
  Grp<T> g;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const int lane = (int)(threadIdx.x & (WAVE - 1));
  if (round >= rounds_run(stats[kStatMaxCount], cb)) return;  // every bucket already is a single item
  u32* next_chunk = stats + kStatNextChunk + round;
  const u32 total = choff[K];
  // A wavefront takes GW consecutive chunks (of `order`) at a time: first the run of its own index, then runs
  // drawn from a counter (zero at launch) behind those, until the end is passed.
  const u32 nwaves = (u32)((gridDim.x * blockDim.x) / WAVE);
  u32 q0 = (u32)((blockIdx.x * blockDim.x + threadIdx.x) / WAVE) * (u32)GW;
  for (;; ) {
    if (q0 >= total) break;
    const u32 at = q0 + (u32)(lane / T);
    const bool active = at < total;
    const u32 q = (active && order) ? order[at] : at;
    const ChunkAt ch = chunk_at(q, active, cnt, choff, K, round, cb);
    const u32 len = ch.len;
    const size_t start = (size_t)off[ch.key] + ch.begin;
    // first round: the chunk's row indices, spread over the lanes of the group
    u32 idx[IDX];
    if (FIRST) {
#pragma unroll
      for (int r = 0; r < IDX; ++r) {
        const u32 e = (u32)(r * T + g.k);
        idx[r] = e < len ? sorted[start + e] : 0u;
      }
    }
    auto item = [&](u32 e) -> const u32* {
      size_t at = start + e;
      if (FIRST) {
        u32 v = idx[0];
#pragma unroll
        for (int r = 1; r < IDX; ++r) v = ((int)(e / T) == r) ? idx[r] : v;
        at = g.bcast(v, (int)(e % T));
      }
      return e < len ? in + at * (size_t)EL : one;
    };
    typename Ops::E acc;
    Ops::load(acc, item(0), g);
#pragma unroll 1
    for (u32 e = 1; wave_any(e < len); ++e) {
      // Touch the next item while this one is multiplied: the lanes of the group read words one lane's
      // share apart, which covers every cache line of the item; the value only has to stay live.
      const u32 touch = Ops::touch(item(e + 1), g);
      // a group that has run out of items multiplies by one and stays in step with its wave
      Ops::mul_mem(acc, item(e), mod, g);
      keep_live(touch);
    }
    if (active) Ops::store(out + (size_t)q * EL, acc, g);
    u32 drawn = 0;
    if (lane == 0) drawn = atomicAdd(next_chunk, (u32)GW);
    q0 = nwaves * (u32)GW + (u32)__builtin_amdgcn_ds_bpermute(0, (int)drawn);
  }
}

// Sub-products of one (position, column, sign): item g < 16: prod_l B[32 g + l]; item 16 + l: prod_h B[32 h + l].
// B[k] is the single item left of key k after the last round that ran (one when the bucket is empty,
// cnt[k] = 0): item offs_r[k] of that round's output arena, offs_r the offsets of the round after it.
// SPLIT = 4: an item's factors are split over four neighbouring lane groups of a block, which multiply their
// shares side by side and then combine them pairwise through LDS: a chain of 8 + 2 products instead of 32, for
// calls with so few items that the chain is what they wait for. SPLIT = 1: one group per item, no product slot
// spent on combining, for calls whose items fill the chip.
template <int LPT, int T, bool PAIR, int SPLIT>
__global__ __launch_bounds__(kBlockThreads) void k_bk_sub(ModRef M, const u32* __restrict__ one,
                                                          const u32* __restrict__ arena0,
                                                          const u32* __restrict__ arena1,
                                                          const u32* __restrict__ cnt, const u32* __restrict__ offs,
                                                          size_t K, int cb, const u32* __restrict__ stats,
                                                          size_t combos, u32* __restrict__ G) {
  using Ops = ElemOps<LPT, T, PAIR>;
  constexpr int EL = Ops::kLimbs;
  constexpr int GPB = kBlockThreads / Grp<T>::kPitch;
  constexpr int kSubSplit = SPLIT;
  static_assert(SPLIT == 1 || SPLIT == 4, "the pairwise combination below is written for four shares");
  static_assert(GPB % kSubSplit == 0 && kSubSplit * Grp<T>::kPitch <= WAVE, "the groups of an item share a wavefront");
  __shared__ u32 lds[SPLIT > 1 ? (GPB / 2) * EL : 1];
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const int ran = rounds_run(stats[kStatMaxCount], cb);
  const u32* B = ((ran - 1) & 1) ? arena1 : arena0;
  const u32* off = offs + (size_t)ran * (K + 1);
  const size_t count = combos * kSubProducts * kSubSplit;
  const int part = bt.gib % kSubSplit;
  u32* slot = lds + (size_t)(bt.gib / kSubSplit * 2 + (part & 1)) * EL;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    const size_t grp = base + bt.gib;
    const bool active = grp < count;
    const size_t it = grp / kSubSplit;
    const size_t combo = active ? it / kSubProducts : 0;
    const int sub = active ? (int)(it - combo * kSubProducts) : 0;
    const bool is_hi = sub < kHiCount;
    const size_t key0 = combo * kMags + (is_hi ? (size_t)sub * kLoCount : (size_t)(sub - kHiCount));
    const size_t stride = is_hi ? 1 : kLoCount;
    const int per = active ? (is_hi ? kLoCount : kHiCount) / kSubSplit : 0;  // factors of this group's share
    const int e0 = part * per;
    // factor e of this share, or null when its bucket is empty or the share is shorter
    auto locate = [&](int e) -> const u32* {
      const size_t key = key0 + (size_t)(e0 + e) * stride;
      return (e < per && cnt[key] != 0u) ? B + (size_t)off[key] * EL : nullptr;
    };
    typename Ops::E acc;
    Ops::load(acc, one, g);
    const u32* next = locate(0);
    bool any = false;
#pragma unroll 1
    for (int e = 0; e < kLoCount / kSubSplit; ++e) {
      // the next factor is located and touched while this one is multiplied
      const u32* cur = next;
      next = (e + 1 < kLoCount / kSubSplit) ? locate(e + 1) : nullptr;
      const u32 touch = Ops::touch(next ? next : one, g);
      if (wave_any(cur != nullptr)) Ops::mul_mem(acc, cur ? cur : one, mod, g);
      if (SPLIT > 1) any = any || cur != nullptr;
      keep_live(touch);
    }
    // shares 2, 3 hand theirs to shares 0, 1; then share 1 to share 0. Every group of a wavefront runs the
    // products (the ones with nothing to take multiply by one), so that all lanes stay on the same path; the
    // groups of an item sit in one wavefront, and a wavefront whose items are all empty (an unused digit
    // position) skips them.
    if constexpr (SPLIT > 1) {
      const bool work = wave_any(any);
#pragma unroll 1
      for (int half = kSubSplit / 2; half >= 1; half >>= 1) {
        if (part >= half && part < 2 * half) Ops::store(slot, acc, g);
        __syncthreads();
        if (work) Ops::mul_mem(acc, part < half ? (const u32*)(slot + (size_t)(half == 1 ? 1 : 0) * EL) : one, mod, g);
        __syncthreads();
      }
    }
    if (active && part == 0) Ops::store(G + it * (size_t)EL, acc, g);
  }
}

// Weighted products prod_e G[e]^(e+1) in two stages. The low part has the 32 entries Glo[0..31]; the high part
// prod_h Ghi[h]^h is the same form over the 15 entries Ghi[1..15]. Stage 1, per segment of 8 entries
// (4 low segments, 2 high ones): A = prod_u G[8q+u]^(u+1) and T = prod_u G[8q+u] by a running product from
// the top (run *= G; acc *= run). Stage 2: prod_q A_q * (prod_q T_q^q)^8.
constexpr int kSegLen = 8, kLoSegs = kLoCount / kSegLen, kHiSegs = kHiCount / kSegLen, kSegs = kLoSegs + kHiSegs;

template <int LPT, int T, bool PAIR>
__global__ __launch_bounds__(kBlockThreads) void k_bk_fold1(ModRef M, const u32* __restrict__ one,
                                                            const u32* __restrict__ G, size_t combos,
                                                            u32* __restrict__ AT) {
  using Ops = ElemOps<LPT, T, PAIR>;
  constexpr int EL = Ops::kLimbs;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const size_t count = combos * kSegs;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    const size_t it = base + bt.gib;
    const bool active = it < count;
    const size_t combo = active ? it / kSegs : 0;
    const int seg = active ? (int)(it - combo * kSegs) : 0;
    const bool is_hi = seg >= kLoSegs;
    // entry e of the segment's sequence: Glo[e], or Ghi[e + 1] (absent for e = 15)
    const int e0 = (is_hi ? seg - kLoSegs : seg) * kSegLen;
    const u32* seq = G + (combo * kSubProducts + (is_hi ? 1 : kHiCount)) * (size_t)EL;
    const int limit = active ? (is_hi ? kHiCount - 1 : kLoCount) : 0;
    auto entry = [&](int u) -> const u32* { return (e0 + u < limit) ? seq + (size_t)(e0 + u) * EL : one; };
    typename Ops::E run, acc;
    Ops::load(run, entry(kSegLen - 1), g);
    Ops::copy(acc, run);
#pragma unroll 1
    for (int u = kSegLen - 2; u >= 0; --u) {
      Ops::mul_mem(run, entry(u), mod, g);
      Ops::mul(acc, run, mod, g);
    }
    if (active) {
      Ops::store(AT + (it * 2) * (size_t)EL, acc, g);
      Ops::store(AT + (it * 2 + 1) * (size_t)EL, run, g);
    }
  }
}

// R[combo][0] = low part, R[combo][1] = high part
template <int LPT, int T, bool PAIR>
__global__ __launch_bounds__(kBlockThreads) void k_bk_fold2(ModRef M, const u32* __restrict__ one,
                                                            const u32* __restrict__ AT, size_t combos,
                                                            u32* __restrict__ R) {
  using Ops = ElemOps<LPT, T, PAIR>;
  constexpr int EL = Ops::kLimbs;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const size_t count = combos * 2;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    const size_t it = base + bt.gib;
    const bool active = it < count;
    const size_t combo = active ? it >> 1 : 0;
    const bool is_hi = (it & 1) != 0;
    const int nseg = active ? (is_hi ? kHiSegs : kLoSegs) : 0;
    const u32* mine = AT + ((combo * kSegs + (is_hi ? kLoSegs : 0)) * 2) * (size_t)EL;
    auto a_of = [&](int q) -> const u32* { return q < nseg ? mine + (size_t)(2 * q) * EL : one; };
    auto t_of = [&](int q) -> const u32* { return q < nseg ? mine + (size_t)(2 * q + 1) * EL : one; };
    typename Ops::E run, acc;
    Ops::load(run, t_of(kLoSegs - 1), g);
    Ops::copy(acc, run);
#pragma unroll 1
    for (int q = kLoSegs - 2; q >= 1; --q) {
      Ops::mul_mem(run, t_of(q), mod, g);
      Ops::mul(acc, run, mod, g);
    }
#pragma unroll 1
    for (int i = 0; i < 3; ++i) Ops::sqr(acc, mod, g);  // ^8 = ^kSegLen
#pragma unroll 1
    for (int q = 0; q < kLoSegs; ++q) Ops::mul_mem(acc, a_of(q), mod, g);
    if (active) Ops::store(R + it * (size_t)EL, acc, g);
  }
}

// P[j][sign] = prod_s (R_hi[s]^32 R_lo[s])^(1024^s), top position first. PAIR: the result leaves the pair form
// (`leave` = the pair constant R_N) and is stored as the canonical integer, the form of a stored ciphertext.
template <int LPT, int T, bool PAIR>
__global__ __launch_bounds__(kBlockThreads) void k_bk_horner(ModRef M, const u32* __restrict__ one,
                                                             const u32* __restrict__ leave,
                                                             const u32* __restrict__ R, size_t cols,
                                                             u32* __restrict__ P, const u32* __restrict__ stats) {
  using Ops = ElemOps<LPT, T, PAIR>;
  constexpr int EL = Ops::kLimbs;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const int npos = digit_positions(stats[kStatMaxMag]);
  const size_t count = cols * 2;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    const size_t it = base + bt.gib;
    const bool active = it < count;
    const size_t js = active ? it : 0;  // j * 2 + sign
    typename Ops::E acc;
    Ops::load(acc, one, g);
#pragma unroll 1
    for (int s = npos - 1; s >= 0; --s) {
      const u32* r = R + (((size_t)s * cols * 2 + js) * 2) * (size_t)EL;  // [0] low part, [1] high part
#pragma unroll 1
      for (int half = 1; half >= 0; --half) {
        if (s != npos - 1 || half != 1) {
#pragma unroll 1
          for (int i = 0; i < 5; ++i) Ops::sqr(acc, mod, g);
        }
        Ops::mul_mem(acc, r + (size_t)half * EL, mod, g);
      }
    }
    if constexpr (PAIR) {
      Ops::mul_mem(acc, leave, mod, g);
      pair_canonical<LPT, T>(acc.x0, acc.x1, mod.n, g);
      u32 lo[LPT], hi[LPT];
      pair_to_integer<LPT, T>(lo, hi, acc.x0, acc.x1, mod.n, g);
      if (active) {
        store_limbs<LPT, T>(P + it * (size_t)EL, lo, g);
        store_limbs<LPT, T>(P + it * (size_t)EL + LPT * T, hi, g);
      }
    } else {
      if (active) Ops::store(P + it * (size_t)EL, acc, g);
    }
  }
}

// Segmented summation: segment k = elements [o[k], o[k+1]) of one array is a "bucket" whose rows are
// already in place. cnt[k] = its length; offsets that run backwards or past the end of the array are
// the caller's error and give an empty or clipped segment (and a status bit), never an access outside.
__global__ __launch_bounds__(kBlockThreads) void k_seg_counts(const u32* __restrict__ offsets, size_t nseg, u32 count,
                                                              u32* __restrict__ cnt, u32* __restrict__ first,
                                                              u32* __restrict__ status) {
  for (size_t k = (size_t)blockIdx.x * blockDim.x + threadIdx.x; k < nseg; k += (size_t)gridDim.x * blockDim.x) {
    const u32 a = offsets[k], b = offsets[k + 1];
    const u32 a1 = a < count ? a : count, b1 = b < count ? b : count;
    const bool bad = b < a || b > count;
    cnt[k] = b1 > a1 ? b1 - a1 : 0u;
    first[k] = a1;
    if (bad && status) atomicOr(status, (u32)HAFLO_ST_RANGE);
  }
}

// out[k] = the single item left of segment k after the last round that ran, canonical (1 for an empty one)
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_seg_finish(ModRef M, const u32* __restrict__ arena0,
                                                              const u32* __restrict__ arena1,
                                                              const u32* __restrict__ cnt, const u32* __restrict__ offs,
                                                              size_t K, int cb, const u32* __restrict__ stats,
                                                              u32* __restrict__ out) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  const int ran = rounds_run(stats[kStatMaxCount], cb);
  const u32* B = ((ran - 1) & 1) ? arena1 : arena0;
  const u32* off = offs + (size_t)ran * (K + 1);
  for (size_t base = bt.first(); base < K; base += bt.stride()) {
    const size_t k = base + bt.gib;
    const bool active = k < K;
    u32 acc[LPT];
    load_limbs<LPT, T>(acc, (active && cnt[k] != 0u) ? B + (size_t)off[k] * NL : M.r1, g);
    canonicalise<LPT, T>(acc, mod.n, g);
    if (active) store_limbs<LPT, T>(out + k * (size_t)NL, acc, g);
  }
}

int rounds_for(size_t rows, int cb) {
  int r = 0;
  for (size_t reach = 1; reach < rows; reach <<= cb) ++r;
  return r < 1 ? 1 : r;
}

// Chunk size of a call with `items` factors in all: the long chunks once the first round has several full passes
// of chunks over the lane groups the chip holds (then the later rounds' items are what is worth saving), the
// short ones below that, where the call waits for its longest chain of products.
int chunk_bits(const haflo_ctx* ctx, size_t items, int lanes) {
  const size_t resident = (size_t)ctx->num_cu * 3 * (size_t)(kBlockThreads / lanes);
  return (items >> kChunkBitsMax) >= 4 * resident ? kChunkBitsMax : kChunkBitsMin;
}

}  // namespace

namespace haflo {

SegSumPlan seg_sum_plan(const haflo_ctx* ctx, size_t count, size_t nseg) {
  SegSumPlan p;
  const size_t nl = (size_t)ctx->N.nl;
  p.chunk_bits = chunk_bits(ctx, count, ctx->N.t);
  p.rounds = rounds_for(count, p.chunk_bits);
  p.scan_blocks = (nseg + kScanKeys - 1) / kScanKeys;
  size_t p1 = (count >> p.chunk_bits) + nseg;
  if (p1 > count) p1 = count;
  size_t p2 = (p1 >> p.chunk_bits) + nseg;
  if (p2 > p1) p2 = p1;
  size_t w = 0;
  p.off_cnt = w;     w += kStatWords + 2 * nseg;  // statistics and chunk counters, lengths, first elements
  p.off_totals = w;  w += (size_t)(p.rounds + 1) * p.scan_blocks;
  p.off_offs = w;    w += (size_t)(p.rounds + 1) * (nseg + 1);
  w = (w + 63) & ~(size_t)63;
  p.off_arena[0] = w; w += p1 * nl;
  p.off_arena[1] = w; w += p2 * nl;
  p.total = w;
  return p;
}

int seg_sum(const haflo_ctx* ctx, const uint32_t* d_c, const uint32_t* d_offsets, size_t count, size_t nseg,
            uint32_t* d_out, uint32_t* d_status, uint32_t* ws, hipStream_t st) {
  const ModHost& m = ctx->N;
  const SegSumPlan p = seg_sum_plan(ctx, count, nseg);
  const int cb = p.chunk_bits;
  if (p.rounds + 1 > kMaxComp || kStatNextChunk + p.rounds > kStatWords) return HAFLO_EINVAL;
  const size_t K = nseg;
  u32* stats = ws + p.off_cnt;
  u32* cnt = stats + kStatWords;
  u32* first = cnt + K;
  u32* totals = ws + p.off_totals;
  auto offs = [&](int idx) { return ws + p.off_offs + (size_t)idx * (K + 1); };
  LaunchShape one;
  one.blocks = 1;
  one.threads = kBlockThreads;
  one.gpb = kBlockThreads;
  LaunchShape scan;
  scan.blocks = (int)p.scan_blocks;
  scan.threads = kScanThreads;
  scan.gpb = kScanThreads;
  HAFLO_LAUNCH(k_bk_zero, one, st, stats, (size_t)kStatWords);
  HAFLO_LAUNCH(k_seg_counts, launch_shape(ctx, K, 1, 8), st, d_offsets, K, (u32)count, cnt, first, d_status);
  HAFLO_LAUNCH(k_bk_scan_totals, scan, st, (const u32*)cnt, K, p.rounds + 1, cb, totals, stats);
  HAFLO_LAUNCH(k_bk_scan_final, scan, st, (const u32*)cnt, K, p.rounds + 1, cb, (const u32*)totals, offs(0));
  const u32* items = d_c;
  for (int r = 0; r < p.rounds; ++r) {
    size_t bound = count;
    for (int i = 0; i <= r; ++i) bound = (bound >> cb) + K;
    const LaunchShape sh = launch_shape(ctx, bound, m.t, 3);
    u32* out = ws + p.off_arena[r & 1];
    // round 0 reads the elements where they are: a segment's items start at its first element
    const u32* off = r == 0 ? (const u32*)first : (const u32*)offs(r);
#define CALL(LPT, T)                                                                                        \
  HAFLO_LAUNCH((k_bk_round<LPT, T, false, false>), sh, st, m.ref(), (const u32*)m.ref().r1, items,       \
               (const u32*)nullptr, (const u32*)cnt, off, (const u32*)offs(r + 1), K, r, cb, stats, (const u32*)nullptr, out)
    HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
    items = out;
  }
  {
    const LaunchShape sh = launch_shape(ctx, K, m.t, 8);
#define CALL(LPT, T)                                                                          \
  HAFLO_LAUNCH((k_seg_finish<LPT, T>), sh, st, m.ref(), (const u32*)(ws + p.off_arena[0]),  \
               (const u32*)(ws + p.off_arena[1]), (const u32*)cnt, (const u32*)offs(0), K, cb, (const u32*)stats, d_out)
    HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  }
  return hip_status(hipGetLastError());
}

bool xtd_buckets_fit(size_t rows, size_t cols) {
  // row indices, chunk counts and item offsets are 32-bit; the prefix sum over the 4096 keys per column
  // adds up the totals of all earlier blocks in every block, which is meant for at most a few thousand blocks
  return rows < (1ull << 32) && cols != 0 && cols <= 1024 && rows * kMaxPos <= 0xFFFFFFFFull / cols;
}

XtdBucketPlan xtd_bucket_plan(const haflo_ctx* ctx, size_t rows, size_t cols) {
  XtdBucketPlan p;
  const size_t nl = (size_t)ctx->N.nl;
  p.pairs = haflo_has_pair_geometry(ctx->Nh);
  p.chunk_bits = chunk_bits(ctx, rows * cols * 2, p.pairs ? 2 * ctx->Nh.t : ctx->N.t);  // two digits per entry as a rule
  p.rounds = rounds_for(rows, p.chunk_bits);
  p.keys = cols * kMaxPos * 2 * kMags;
  p.scan_blocks = (p.keys + kScanKeys - 1) / kScanKeys;
  const size_t terms = rows * cols * kMaxPos;
  size_t p1 = (terms >> p.chunk_bits) + p.keys;
  if (p1 > terms) p1 = terms;
  size_t p2 = (p1 >> p.chunk_bits) + p.keys;
  if (p2 > p1) p2 = p1;
  const size_t combos = cols * kMaxPos * 2;
  size_t w = 0;
  p.off_cnt = w;     w += kStatWords + 2 * p.keys;  // statistics and chunk counters, row counts, scatter cursors
  p.off_totals = w;  w += (size_t)(p.rounds + 1) * p.scan_blocks;
  p.off_offs = w;    w += (size_t)(p.rounds + 1) * (p.keys + 1);
  p.off_sorted = w;  w += terms;
  w = (w + 63) & ~(size_t)63;
  p.off_arena[0] = w; w += p1 * nl;
  p.off_arena[1] = w; w += p2 * nl;
  p.off_G = w;       w += combos * kSubProducts * nl;
  p.off_AT = w;      w += combos * kSegs * 2 * nl;
  p.off_R = w;       w += combos * 2 * nl;
  p.off_pairs = w;   w += p.pairs ? rows * nl : 0;  // the ciphertexts in the pair form
  p.off_order = w;   w += p1;                       // the chunks of a round in the order of their lengths
  p.total = w;
  return p;
}

int xtd_buckets(const haflo_ctx* ctx, const uint32_t* d_c, const int32_t* d_X, size_t rows, size_t cols,
                uint32_t* ws, uint32_t* d_P, hipStream_t st) {
  const XtdBucketPlan p = xtd_bucket_plan(ctx, rows, cols);
  const int cb = p.chunk_bits;
  if (p.rounds + 1 > kMaxComp || kStatNextChunk + p.rounds > kStatWords) return HAFLO_EINVAL;
  const size_t K = p.keys;
  u32* stats = ws + p.off_cnt;
  u32* cnt = stats + kStatWords;
  u32* cursor = cnt + K;
  u32* totals = ws + p.off_totals;
  // offs(0) = positions in the sorted row array; offs(r + 1) = chunk offsets of round r = item offsets of round r + 1
  auto offs = [&](int idx) { return ws + p.off_offs + (size_t)idx * (K + 1); };
  u32* sorted = ws + p.off_sorted;
  LaunchShape flat;  // one block per column and kTermRows rows
  flat.threads = kBlockThreads;
  flat.gpb = kBlockThreads;
  flat.blocks = (int)(cols * ((rows + kTermRows - 1) / kTermRows));
  const LaunchShape fill = launch_shape(ctx, kStatWords + 2 * K, 1, 8);
  LaunchShape scan;
  scan.blocks = (int)p.scan_blocks;
  scan.threads = kScanThreads;
  scan.gpb = kScanThreads;
  HAFLO_LAUNCH(k_bk_zero, fill, st, stats, kStatWords + 2 * K);
  HAFLO_LAUNCH((k_bk_terms<false>), flat, st, d_X, rows, cols, cnt, (const u32*)nullptr, (u32*)nullptr, stats);
  HAFLO_LAUNCH(k_bk_scan_totals, scan, st, (const u32*)cnt, K, p.rounds + 1, cb, totals, stats);
  HAFLO_LAUNCH(k_bk_scan_final, scan, st, (const u32*)cnt, K, p.rounds + 1, cb, (const u32*)totals, offs(0));
  HAFLO_LAUNCH((k_bk_terms<true>), flat, st, d_X, rows, cols, cursor, (const u32*)offs(0), sorted, stats);
  // The products run on pairs of residues modulo n (5/8 of the limb products of a full-length product; every
  // supported key size has that geometry): the ciphertexts are taken into the pair form once (two products each,
  // against two products per matrix entry below), and the column results leave it in k_bk_horner. The pair form
  // sits on twice the lanes of n, which also suits the short kernels at the end, where few integers are left.
  const ModHost& mh = ctx->Nh;
  if (!p.pairs) return HAFLO_EINVAL;
  const ModRef M = mh.ref();
  const int lanes = 2 * mh.t;
  const u32* one = mh.d_pairs + (size_t)kConstR1 * 2 * mh.nl;
  const u32* leave = mh.d_pairs + (size_t)kConstR3 * 2 * mh.nl;
  u32* cp = ws + p.off_pairs;
  {
    const LaunchShape sh = launch_shape(ctx, rows, lanes, 8);
#define CALL(LPT, T)                                                                                         \
  HAFLO_LAUNCH((k_to_pairs<LPT, T>), sh, st, M, (const u32*)(mh.d_pairs + (size_t)kConstR4 * 2 * mh.nl),    \
               (const u32*)(mh.d_pairs + (size_t)kConstR5 * 2 * mh.nl), d_c, rows, cp)
    HAFLO_DISPATCH_PAIRS(mh, CALL);
#undef CALL
  }
  const u32* items = cp;
  for (int r = 0; r < p.rounds; ++r) {
    // upper bound of the chunks of this round: one lane group each, capped by the grid-stride loop
    size_t bound = rows * cols * kMaxPos;
    for (int i = 0; i <= r; ++i) bound = (bound >> cb) + K;
    const LaunchShape sh = launch_shape(ctx, bound, lanes, 3);
    u32* out = ws + p.off_arena[r & 1];
    const u32* srt = r == 0 ? (const u32*)sorted : (const u32*)nullptr;
    // the rounds with many chunks hand them out in the order of their lengths
    const u32* ord = nullptr;
    if (r < kOrdRounds) {
      LaunchShape osh;
      osh.threads = osh.gpb = kBlockThreads;
      osh.blocks = (int)std::min((bound + kBlockThreads - 1) / kBlockThreads, (size_t)ctx->num_cu * 8);
      u32* order = ws + p.off_order;
      HAFLO_LAUNCH((k_bk_order<false>), osh, st, (const u32*)cnt, (const u32*)offs(r + 1), K, r, cb, stats, order);
      HAFLO_LAUNCH((k_bk_order<true>), osh, st, (const u32*)cnt, (const u32*)offs(r + 1), K, r, cb, stats, order);
      ord = order;
    }
#define CALL_ROUND(LPT, T, FIRST)                                                                        \
  HAFLO_LAUNCH((k_bk_round<LPT, T, FIRST, true>), sh, st, M, one, items, srt, (const u32*)cnt,          \
               (const u32*)offs(r), (const u32*)offs(r + 1), K, r, cb, stats, ord, out)
#define CALL(LPT, T) do { if (r == 0) CALL_ROUND(LPT, T, true); else CALL_ROUND(LPT, T, false); } while (0)
    HAFLO_DISPATCH_PAIRS(mh, CALL);
#undef CALL
#undef CALL_ROUND
    items = out;
  }
  const size_t combos = cols * kMaxPos * 2;
  u32* G = ws + p.off_G;
  u32* AT = ws + p.off_AT;
  u32* R = ws + p.off_R;
  {
    // half of the items belong to unused digit positions and leave at once
    // one lane group per sub-product once those alone give every SIMD four wavefronts, else four
    const bool split = combos * kSubProducts * (size_t)lanes < (size_t)ctx->num_cu * 16 * WAVE;
    const LaunchShape sh = launch_shape(ctx, combos * kSubProducts * (split ? 4 : 1), lanes, 8);
#define CALL_SUB(LPT, T, SPLIT)                                                                         \
  HAFLO_LAUNCH((k_bk_sub<LPT, T, true, SPLIT>), sh, st, M, one, (const u32*)(ws + p.off_arena[0]),     \
               (const u32*)(ws + p.off_arena[1]), (const u32*)cnt, (const u32*)offs(0), K, cb, (const u32*)stats, combos, G)
#define CALL(LPT, T) do { if (split) CALL_SUB(LPT, T, 4); else CALL_SUB(LPT, T, 1); } while (0)
    HAFLO_DISPATCH_PAIRS(mh, CALL);
#undef CALL
#undef CALL_SUB
  }
  {
    const LaunchShape sh = launch_shape(ctx, combos * kSegs, lanes, 8);
#define CALL(LPT, T) HAFLO_LAUNCH((k_bk_fold1<LPT, T, true>), sh, st, M, one, (const u32*)G, combos, AT)
    HAFLO_DISPATCH_PAIRS(mh, CALL);
#undef CALL
  }
  {
    const LaunchShape sh = launch_shape(ctx, combos * 2, lanes, 8);
#define CALL(LPT, T) HAFLO_LAUNCH((k_bk_fold2<LPT, T, true>), sh, st, M, one, (const u32*)AT, combos, R)
    HAFLO_DISPATCH_PAIRS(mh, CALL);
#undef CALL
  }
  {
    const LaunchShape sh = launch_shape(ctx, cols * 2, lanes, 8);
#define CALL(LPT, T) \
  HAFLO_LAUNCH((k_bk_horner<LPT, T, true>), sh, st, M, one, leave, (const u32*)R, cols, d_P, (const u32*)stats)
    HAFLO_DISPATCH_PAIRS(mh, CALL);
#undef CALL
  }
  return hip_status(hipGetLastError());
}

}  // namespace haflo
