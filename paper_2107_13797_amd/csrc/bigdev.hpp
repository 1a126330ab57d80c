// Device-side big-integer core for gfx950: cooperative multi-limb arithmetic
// with one big integer spread over T consecutive lanes of a 64-wide wavefront.
//
// Representation. A big integer of NL = T*LPT limbs is held in radix 2^29:
// lane k of the group (k = 0 least significant) keeps limbs [k*LPT, (k+1)*LPT)
// in registers. 29-bit limbs leave 6 spare bits in a 64-bit accumulator, so a
// column sum of up to 62 limb products needs no carry handling: the inner loops
// are pure v_mad_u64_u32 streams (32x32+64 multiply-add issues at full VALU
// rate on this chip, so every carry instruction saved is a multiply gained).
//
// "Lazy" operands: limbs may exceed 2^29 by a few units (< 2^29 + 2^8) and the
// value may reach a small multiple of the modulus; the radix 2^(29*NL) exceeds
// every modulus by at least 2^10, which keeps Montgomery products below twice
// the modulus without a final subtraction. Only values that are stored or
// compared are brought to canonical form (limbs < 2^29, value < modulus).
//
// Cross-lane traffic: ds_bpermute for broadcasts from a lane chosen at run time,
// DPP moves for broadcasts from lane 0 of a group and for the exchange with the
// neighbouring lane (groups of up to 16 lanes never straddle a 16-lane DPP row;
// a group of more lanes has the wavefront to itself).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace haflo {
namespace dev {

typedef uint32_t u32;
typedef uint64_t u64;
typedef int32_t s32;
typedef int64_t s64;

constexpr int LIMB_BITS = 29;
constexpr u32 LIMB_MASK = (1u << LIMB_BITS) - 1u;
constexpr int WAVE = 64;

__device__ __forceinline__ u64 mad64(u32 a, u32 b, u64 c) { return (u64)a * (u64)b + c; }

// f(integral_constant<int, I>) for I = BEGIN .. END - 1: a loop whose index is a compile-time constant in the body
template <int BEGIN, int END, class F>
__device__ __forceinline__ void static_for(F&& f) {
  if constexpr (BEGIN < END) {
    f(std::integral_constant<int, BEGIN>{});
    static_for<BEGIN + 1, END>(f);
  }
}

// Geometry of the lane group that owns one big integer. Up to 16 lanes, a power of two: groups tile a
// 16-lane DPP row and every lane of the wavefront belongs to one. More than 16 lanes: one group per
// wavefront on lanes 0 .. T-1 (any T up to 64), for batches so small that the latency of a single product
// is what counts; the lanes above hold zeros (zero limbs of the operands and of the modulus keep every
// column of theirs zero, so the top lane of the group receives zeros from above, as it does from the
// first lane of a neighbouring group) and neither load nor store. Neighbour exchange then uses the DPP
// shifts over the whole wavefront, and the quotient digit of lane 0 is read into a scalar register.
template <int T>
struct Grp {
  static_assert(T >= 1 && T <= 64 && (T > 16 || (T & (T - 1)) == 0), "1, 2, 4, 8, 16 lanes, or one group per wavefront");
  static constexpr bool kWhole = T > 16;           // one group per wavefront
  static constexpr int kPitch = kWhole ? WAVE : T;  // lanes from one group to the next
  int k;          // this lane's chunk index inside the group
  int base_addr;  // ds_bpermute byte address of the group's lane 0
  __device__ __forceinline__ Grp() {
    int lane = (int)(threadIdx.x & (WAVE - 1));
    k = lane & (kPitch - 1);
    base_addr = (lane - k) << 2;
  }
  // false on the lanes of a whole-wavefront group that hold no limbs
  __device__ __forceinline__ bool live() const { return !kWhole || k < T; }
  // value of `v` held by lane `src_k` of this group
  __device__ __forceinline__ u32 bcast(u32 v, int src_k) const {
    if (T == 1) return v;
    return (u32)__builtin_amdgcn_ds_bpermute(base_addr + (src_k << 2), (int)v);
  }
  // value of `v` held by lane 0 of this group, through DPP moves: a few VALU cycles instead of a round
  // trip through the LDS crossbar, which matters where the result is needed at once. A group that fills
  // a 16-lane row takes the row broadcast; smaller groups a quad broadcast, then a row shift by 4 lanes
  // into the odd banks; a whole-wavefront group reads lane 0 into a scalar register.
  __device__ __forceinline__ u32 bcast0(u32 v) const {
    if (T == 1) return v;
    int x = (int)v;
    if (kWhole) return (u32)__builtin_amdgcn_readfirstlane(x);
    if (T == 16) return (u32)__builtin_amdgcn_update_dpp(x, x, 0x150 /* row_newbcast:0 */, 0xf, 0xf, false);
    x = __builtin_amdgcn_update_dpp(x, x, T == 2 ? 0xA0 /* quad_perm:[0,0,2,2] */ : 0x00 /* [0,0,0,0] */, 0xf, 0xf, false);
    if (T == 8) x = __builtin_amdgcn_update_dpp(x, x, 0x114 /* row_shr:4 */, 0xf, 0xA, false);
    return (u32)x;
  }
  // bcast0(v & m) with the mask `m` (in a vector register) riding on the first DPP move of the broadcast
  __device__ __forceinline__ u32 bcast0_masked(u32 v, u32 m) const {
    if (T == 1 || kWhole) return bcast0(v & m);
    int x = (int)v;
    if (T == 16) return (u32)__builtin_amdgcn_update_dpp(0, x, 0x150 /* row_newbcast:0 */, 0xf, 0xf, true) & m;
    x = (int)((u32)__builtin_amdgcn_update_dpp(0, x, T == 2 ? 0xA0 /* quad_perm:[0,0,2,2] */ : 0x00 /* [0,0,0,0] */, 0xf, 0xf, true) & m);
    if (T == 8) x = __builtin_amdgcn_update_dpp(x, x, 0x114 /* row_shr:4 */, 0xf, 0xA, false);
    return (u32)x;
  }
  // v of the next-higher lane; 0 past the end of the 16-lane row (of the wavefront for a whole-wavefront
  // group). The top lane of a group that is not at a row end sees lane 0 of the next group.
  __device__ __forceinline__ u32 from_upper_raw(u32 v) const {
    if (T == 1) return 0u;
    if (kWhole) return (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x130 /* wave_shl:1 */, 0xf, 0xf, true);
    return (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x101 /* row_shl:1 */, 0xf, 0xf, true);
  }
  __device__ __forceinline__ u32 from_upper(u32 v) const {
    if (T == 1) return 0u;
    u32 r = from_upper_raw(v);
    return (k >= T - 1) ? 0u : r;
  }
  // v of the next-lower lane; 0 for the group's lane 0 (and for the lanes without limbs)
  __device__ __forceinline__ u32 from_lower(u32 v) const {
    if (T == 1) return 0u;
    if (kWhole) {
      u32 r = (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x138 /* wave_shr:1 */, 0xf, 0xf, true);
      return (k == 0 || k >= T) ? 0u : r;
    }
    u32 r = (u32)__builtin_amdgcn_update_dpp(0, (int)v, 0x111 /* row_shr:1 */, 0xf, 0xf, true);
    return (k == 0) ? 0u : r;
  }
};

__device__ __forceinline__ bool wave_any(bool p) { return __builtin_amdgcn_ballot_w64(p) != 0ull; }

// The constant 8 = 2^32 / 2^29 behind an optimisation barrier: hi * 8 + acc then
// stays a single v_mad_u64_u32 instead of being strength-reduced into a 64-bit
// shift, two masks and an add.
__device__ __forceinline__ u32 opaque_eight() {
  u32 e = 8u;
  asm volatile("" : "+r"(e));
  return e;
}

// The limb mask in a vector register: an AND with it can carry a DPP lane shift on its other operand, which
// a literal operand rules out.
__device__ __forceinline__ u32 opaque_mask() {
  u32 m = 0x1fffffffu;
  asm volatile("" : "+v"(m));
  return m;
}

// Keeps a loaded value (and so the load) alive up to this point without using it.
__device__ __forceinline__ void keep_live(u32 v) { asm volatile("" ::"r"(v)); }

// Push the upper 32 bits of every column accumulator one column up
// (A[j+1] += 8 * hi(A[j]), radix 2^29 vs word 2^32), leaving each column below
// 2^32 (column 0 below 2^36). The top lane's top column is bounded by the value
// bound of the caller and is left alone. `eight` comes from opaque_eight().
template <int LPT, int T>
__device__ __forceinline__ void hi_normalise(u64 (&A)[LPT], const Grp<T>& g, u32 eight) {
#pragma unroll
  for (int j = 0; j + 1 < LPT; ++j) {
    A[j + 1] = mad64((u32)(A[j] >> 32), eight, A[j + 1]);
    A[j] = (u64)(u32)A[j];
  }
  if (T > 1) {
    u32 hi = (u32)(A[LPT - 1] >> 32);
    u32 send = (g.k == T - 1) ? 0u : hi;
    u32 recv = g.from_lower(send);
    if (g.k != T - 1) A[LPT - 1] = (u64)(u32)A[LPT - 1];
    A[0] = mad64(recv, eight, A[0]);
  }
}

// Where the word-serial operand b of a product comes from: the lanes' own
// registers (limb i sits on lane i / LPT and is broadcast with ds_bpermute), or
// an NL-limb array in memory that every lane of the group reads directly.
// limb (o, rr): limb rr of lane o. kAhead = how many steps before its use a limb is requested, so that
// the exchange is complete by then (rr then runs on into lane o + 1); 0 = fetched in its own step.
template <int LPT, int T>
struct BRegs {
  const u32 (&b)[LPT];
  // a step of few limbs is short: ask earlier, so that the crossbar's latency stays covered. A whole-wavefront
  // group reads the limb into a scalar register instead (the lane index is wave-uniform): one instruction, no
  // address register, nothing to wait for.
  static constexpr int kAhead = Grp<T>::kWhole ? 0 : (LPT <= 3 ? LPT : (LPT <= 8 && LPT % 2 == 0 ? 2 : 1));
  __device__ __forceinline__ u32 limb(int o, int rr, const Grp<T>& g) const {
    if (T == 1) return b[rr % LPT];
    if (Grp<T>::kWhole) return (u32)__builtin_amdgcn_readlane((int)b[rr % LPT], o + rr / LPT);
    // past the last limb this reads a lane of the next group (or wraps); that value is never used
    return (u32)__builtin_amdgcn_ds_bpermute(g.base_addr + ((o + rr / LPT) << 2), (int)b[rr % LPT]);
  }
};
template <int LPT, int T>
struct BMem {
  const u32* p;
  static constexpr int kAhead = 0;  // plain loads, which the compiler batches per lane by itself
  __device__ __forceinline__ u32 limb(int o, int rr, const Grp<T>& g) const {
    (void)g;
    return p[o * LPT + rr];
  }
};

// Which products of a squaring a lane computes in the step that broadcasts limb r of some lane: its own
// limb j takes part iff sq_weight(j, r) != 0, with that factor. Seen over all steps this is a round-robin
// tournament on the limb indices of a lane: of the two steps in which the unordered pair
// {(lane k, limb j), (lane o, limb r)} could be formed - step (o, r) on lane k, step (k, j) on lane o -
// exactly one forms it, doubled, when the cyclic distance (j - r) mod LPT is in [1, (LPT-1)/2] or the
// mirror of that range; for j = r, and for the distance LPT/2 that is its own mirror when LPT is even,
// both steps form it, undoubled. Within one lane (k = o) the same rule yields every pair once and the
// square of each limb once. Either step is at or before column j + r + LPT (k + o) becomes the lowest
// column of lane 0, so the quotient digits see complete columns, as in a general product. All lanes use
// the same limb indices in a step, so nothing diverges and nobody idles: 10 of 18 (5 of 9)
// multiply-adds per step instead of 18 (9).
__host__ __device__ constexpr int sq_weight(int lpt, int j, int r) {
  const int d = ((j - r) % lpt + lpt) % lpt;
  if (d == 0) return 1;
  if (lpt % 2 == 0 && d == lpt / 2) return 1;
  return (d <= (lpt - 1) / 2) ? 2 : 0;
}

// Montgomery product out = a * b / 2^(29*NL) mod n, lazy in and out.
//   a, b: limbs < 2^29 + 2^8, values < 4n.  n: canonical limbs of the odd
//   modulus.  n0inv = -n^-1 mod 2^29.  out: limbs < 2^29 + 2^5, value < 2n.
// Word-serial with a sliding accumulator window: step i adds a*b_i, then q*n
// with q chosen so the lowest column vanishes mod 2^29, then drops that column;
// every lane hands the low 29 bits of its lowest column to the lane below and
// keeps the rest as a carry, so no lane is special-cased.
// SQ: b is a itself (bsrc hands out a's limbs) and the symmetric half of the limb products is left out,
// see sq_weight; doubled limbs stay below 2^30 + 2^9, and a column then takes at most 8 doubled and 2
// plain products next to the 18 of the reduction: 36 * 2^58 as before.
template <int LPT, int T, class BSrc, bool SQ = false>
__device__ __forceinline__ void montmul_core(u32 (&out)[LPT], const u32 (&a)[LPT], const BSrc& bsrc,
                                             const u32 (&n)[LPT], u32 n0inv, const Grp<T>& g) {
  static_assert(LPT <= 18, "a column must not collect more than 36 products");
  const u32 eight = opaque_eight();
  [[maybe_unused]] const u32 maskv = opaque_mask();
  u64 A[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) A[j] = 0;
  // A squaring on at most 9 limbs per lane doubles the multiplicand once (9 registers) instead of the
  // broadcast limb in every step: one vector instruction less per step.
  constexpr bool kDoubledA = SQ && T > 1 && LPT <= 9;
  [[maybe_unused]] u32 ad[LPT];
  if constexpr (kDoubledA) {
#pragma unroll
    for (int j = 0; j < LPT; ++j) ad[j] = a[j] + a[j];
  }
  // Nothing a step waits long for: the limbs b_i were asked for kAhead steps earlier, and the quotient
  // digit q is broadcast with DPP moves.
  constexpr int D = BSrc::kAhead;
  constexpr int RING = D > 0 ? D : 1;
  static_assert(LPT % RING == 0, "ring size");
  u32 ring[RING];
#pragma unroll
  for (int d = 0; d < D; ++d) ring[d] = bsrc.limb(0, d, g);
  // a whole-wavefront group has only 2 to 6 steps per lane: four lanes' worth per loop round, so that the sliding
  // window and the ring of requested limbs need no register moves (11 % off a lone wavefront's chain)
  constexpr int kLanesPerRound = Grp<T>::kWhole ? 4 : 1;
#pragma unroll kLanesPerRound
  for (int o = 0; o < T; ++o) {
    static_for<0, LPT>([&](auto rc) {
      constexpr int r = decltype(rc)::value;
      u32 bi;
      if (D > 0) {
        bi = ring[r % RING];
        ring[r % RING] = bsrc.limb(o, r + D, g);
      } else {
        bi = bsrc.limb(o, r, g);
      }
      // the limb products of this step: all of them, or for a squaring those sq_weight selects
      [[maybe_unused]] const u32 bi2 = (SQ && !kDoubledA) ? bi + bi : bi;
      auto product = [&](auto jc) {
        constexpr int j = decltype(jc)::value;
        constexpr int w = SQ ? sq_weight(LPT, j, r) : 1;
        if constexpr (w == 1) A[j] = mad64(a[j], bi, A[j]);
        else if constexpr (w == 2) A[j] = kDoubledA ? mad64(ad[j], bi, A[j]) : mad64(a[j], bi2, A[j]);
      };
      product(std::integral_constant<int, 0>{});
      // the quotient digit: a whole-wavefront group takes the column into a scalar register first, so that the
      // product and the mask are scalar instructions (the pair products measured slower that way and keep the
      // vector form)
      u32 q;
      if constexpr (Grp<T>::kWhole) q = g.bcast0(((u32)A[0] * n0inv) & maskv);
      else q = g.bcast0_masked((u32)A[0] * n0inv, maskv);
      static_for<1, LPT>(product);
      u64 t0 = mad64(q, n[0], A[0]);
      // the low 29 bits go to the lane below (0 on lane 0 of every group, by the choice of q); masked after
      // the move, so that the mask rides on the DPP instruction
      u32 recv = g.from_upper_raw((u32)t0) & maskv;
      u64 carry = t0 >> LIMB_BITS;
      if (LPT > 1) {
        A[0] = mad64(q, n[1], A[1]) + carry;
#pragma unroll
        for (int j = 2; j < LPT; ++j) A[j - 1] = mad64(q, n[j], A[j]);
        A[LPT - 1] = (u64)recv;
      } else {
        A[0] = (u64)recv + carry;
      }
    });
  }
  // A column register lives LPT steps in a lane (it enters at the top as the 29 bits handed over by
  // the lane above and leaves at the bottom) and takes two products per step: at most 2 * 18 products
  // below 2^58.01 plus one carry below 2^36, which fits 64 bits without intermediate carry handling.
  // One pass before the compression keeps the limbs and the carry to the next lane small.
  hi_normalise<LPT, T>(A, g, eight);
  // Compress the columns to 32-bit limbs: ripple inside the lane, then hand the
  // lane's carry to the lane above (which absorbs it lazily in its limb 0).
  u64 c = 0;
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    u64 v = A[j] + c;
    out[j] = (u32)v & LIMB_MASK;
    c = v >> LIMB_BITS;
  }
  if (T > 1) out[0] += g.from_lower((u32)c);
}

// The same product for a whole-wavefront group of at most 3 limbs per lane, with the column accumulators held
// at 8 times their value, which puts the limb boundary of the lowest column on the 32-bit word boundary:
// the quotient digit needs no mask ((8 x) * n0inv mod 2^32 = 8 q exactly), the 29 bits for the lane below are
// the low word as it is, and the carry is the high word (times 8 again, folded into a multiply-add). A lone
// wavefront is bound by its instruction count, and this step has 5 multiply-adds and 4 other instructions
// where the plain one has 4 and 7. The operands enter shifted (a by 1 bit, b by 2; a by 2 for the doubled
// products of a squaring): lazy limbs below 2^29 + 2^8 leave room for that, and a column of at most 6 products
// stays below 2^64 / 8. Same result as montmul_core, bit for bit.
template <int LPT, int T, bool SQ>
__device__ __forceinline__ void montmul_whole_x8(u32 (&out)[LPT], const u32 (&a)[LPT], const u32 (&b)[LPT],
                                                 const u32 (&n)[LPT], u32 n0inv, const Grp<T>& g) {
  static_assert(Grp<T>::kWhole && LPT >= 2 && LPT <= 3, "6 products per column at most");
  const u32 eight = opaque_eight();
  u32 a2[LPT], b4[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    a2[j] = a[j] << 1;
    b4[j] = b[j] << 2;  // for a squaring also a times 4: the multiplicand of the doubled products
  }
  u64 A[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) A[j] = 0;
#pragma unroll 4
  for (int o = 0; o < T; ++o) {
    static_for<0, LPT>([&](auto rc) {
      constexpr int r = decltype(rc)::value;
      const u32 bi = (u32)__builtin_amdgcn_readlane((int)b4[r], o);
      auto product = [&](auto jc) {
        constexpr int j = decltype(jc)::value;
        constexpr int w = SQ ? sq_weight(LPT, j, r) : 1;
        if constexpr (w == 1) A[j] = mad64(a2[j], bi, A[j]);
        else if constexpr (w == 2) A[j] = mad64(b4[j], bi, A[j]);
      };
      product(std::integral_constant<int, 0>{});
      const u32 q8 = g.bcast0((u32)A[0] * n0inv);
      static_for<1, LPT>(product);
      const u64 t0 = mad64(q8, n[0], A[0]);
      const u32 recv = g.from_upper_raw((u32)t0);
      A[0] = mad64((u32)(t0 >> 32), eight, mad64(q8, n[1], A[1]));
#pragma unroll
      for (int j = 2; j < LPT; ++j) A[j - 1] = mad64(q8, n[j], A[j]);
      A[LPT - 1] = (u64)recv;
    });
  }
#pragma unroll
  for (int j = 0; j < LPT; ++j) A[j] >>= 3;
  hi_normalise<LPT, T>(A, g, eight);
  u64 c = 0;
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    u64 v = A[j] + c;
    out[j] = (u32)v & LIMB_MASK;
    c = v >> LIMB_BITS;
  }
  out[0] += g.from_lower((u32)c);
}


// b in registers (out may alias a and b)
template <int LPT, int T>
__device__ __forceinline__ void montmul(u32 (&out)[LPT], const u32 (&a)[LPT], const u32 (&b)[LPT],
                                        const u32 (&n)[LPT], u32 n0inv, const Grp<T>& g) {
  if constexpr (Grp<T>::kWhole && LPT <= 3) {
    montmul_whole_x8<LPT, T, false>(out, a, b, n, n0inv, g);
  } else {
    BRegs<LPT, T> src = {b};
    montmul_core<LPT, T>(out, a, src, n, n0inv, g);
  }
}

// out = a * a / 2^(29*NL) mod n with the symmetric half of the limb products left out (out may alias a)
template <int LPT, int T>
__device__ __forceinline__ void montsqr(u32 (&out)[LPT], const u32 (&a)[LPT], const u32 (&n)[LPT], u32 n0inv,
                                        const Grp<T>& g) {
  if constexpr (Grp<T>::kWhole && LPT <= 3) {
    montmul_whole_x8<LPT, T, true>(out, a, a, n, n0inv, g);
  } else {
    BRegs<LPT, T> src = {a};
    montmul_core<LPT, T, BRegs<LPT, T>, true>(out, a, src, n, n0inv, g);
  }
}

// b = NL limbs at `bmem`, the same array for every lane of the group
template <int LPT, int T>
__device__ __forceinline__ void montmul_mem(u32 (&out)[LPT], const u32 (&a)[LPT], const u32* bmem,
                                            const u32 (&n)[LPT], u32 n0inv, const Grp<T>& g) {
  BMem<LPT, T> src = {bmem};
  montmul_core<LPT, T>(out, a, src, n, n0inv, g);
}

// ---------------------------------------------------------------------------
// Arithmetic modulo n^2 on pairs of residues modulo n
// ---------------------------------------------------------------------------
// A residue X modulo n^2 is held as two half-length integers, X = x0 + n x1 (x0, x1 lazy residues modulo
// n, NL limbs each, R = 2^(29 NL) the Montgomery radix of n). For X Y = x0 y0 + n (x0 y1 + x1 y0) (mod n^2),
// let m = x0 y0 (-1/n) mod R be the quotient of the Montgomery reduction of x0 y0 and t = (x0 y0 + m n) / R
// its result; then x0 y0 = t R - m n, and
//     Z = t + n z1,  z1 = (x0 y1 + x1 y0 - m) / R mod n,
// satisfies Z R = X Y (mod n^2): a Montgomery product modulo n^2 with the half-length radix, from one
// half-length Montgomery product (whose quotient digits are kept) and one half-length Montgomery reduction
// of a sum of two products: 5 NL^2 limb products instead of the 8 NL^2 of a full-length product on 2 NL
// limbs, and 3.6 NL^2 instead of 6.2 NL^2 for a squaring (x0^2 by sq_weight, 2 x0 x1 as one product with a
// doubled limb). Both run in the same word-serial loop: step i adds a0 b0_i to window A and
// a0 b1_i + a1 b0_i to window B, takes A's quotient digit q, hands its complement 2^29 - 1 - q to the
// lowest column of B on lane 0 (the digits of R - 1 - m; a one in column 0 makes it R - m, and the -R that
// is left turns into -1 after the division, which the final + (n - 1) absorbs), then takes B's digit.
//   a0, a1, b0, b1: limbs < 2^29 + 2^8, values < 4n.  out0 < 2n, out1 < 2n (1 + 2^-30), limbs < 2^29 + 2^5.
// Where two operands' limbs come from: registers (ds_bpermute) or two NL-limb arrays in memory, as for
// the single product.
template <int LPT, int T>
struct BRegs2 {
  const u32 (&b0)[LPT];
  const u32 (&b1)[LPT];
  static constexpr int kAhead = BRegs<LPT, T>::kAhead;
  __device__ __forceinline__ u32 limb0(int o, int rr, const Grp<T>& g) const {
    if (T == 1) return b0[rr % LPT];
    if (Grp<T>::kWhole) return (u32)__builtin_amdgcn_readlane((int)b0[rr % LPT], o + rr / LPT);
    return (u32)__builtin_amdgcn_ds_bpermute(g.base_addr + ((o + rr / LPT) << 2), (int)b0[rr % LPT]);
  }
  __device__ __forceinline__ u32 limb1(int o, int rr, const Grp<T>& g) const {
    if (T == 1) return b1[rr % LPT];
    if (Grp<T>::kWhole) return (u32)__builtin_amdgcn_readlane((int)b1[rr % LPT], o + rr / LPT);
    return (u32)__builtin_amdgcn_ds_bpermute(g.base_addr + ((o + rr / LPT) << 2), (int)b1[rr % LPT]);
  }
};
template <int LPT, int T>
struct BMem2 {
  const u32* p;  // [b0: NL limbs][b1: NL limbs]
  static constexpr int kAhead = 0;
  __device__ __forceinline__ u32 limb0(int o, int rr, const Grp<T>& g) const {
    (void)g;
    return p[o * LPT + rr];
  }
  __device__ __forceinline__ u32 limb1(int o, int rr, const Grp<T>& g) const {
    (void)g;
    return p[LPT * T + o * LPT + rr];
  }
};

// B1X2: the source hands out the limbs of b1 already doubled (a squaring that doubled them once, outside the steps)
template <int LPT, int T, class BSrc, bool SQ, bool B1X2 = false>
__device__ __forceinline__ void pairmul_core(u32 (&out0)[LPT], u32 (&out1)[LPT], const u32 (&a0)[LPT],
                                             const u32 (&a1)[LPT], const BSrc& bsrc, const u32 (&n)[LPT], u32 n0inv,
                                             const Grp<T>& g) {
  static_assert(LPT <= 9, "a column of the second window takes three products per step");
  const u32 eight = opaque_eight();
  [[maybe_unused]] const u32 maskv = opaque_mask();
  u64 A[LPT], B[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    A[j] = 0;
    B[j] = 0;
  }
  if (g.k == 0) B[0] = 1;
  // a squaring doubles x0 once as the multiplicand of its doubled products, instead of the broadcast limb per step
  constexpr bool kDoubledA0 = SQ && T > 1 && !Grp<T>::kWhole;
  [[maybe_unused]] u32 a0d[LPT];
  if constexpr (kDoubledA0) {
#pragma unroll
    for (int j = 0; j < LPT; ++j) a0d[j] = a0[j] + a0[j];
  }
  u32 first = (g.k == 0) ? 1u : 0u;  // the lane that holds the lowest column of the whole integer
  // Hide that `first` is 0 or 1, so that the term it selects stays one multiply-add instead of a move, a
  // select and a 64-bit add: these kernels are bound by vector issue slots, one per instruction whatever it
  // is, at one wavefront per SIMD and at four alike (measured on both).
  if constexpr (T > 1) asm volatile("" : "+v"(first));
  constexpr int D = BSrc::kAhead;
  constexpr int RING = D > 0 ? D : 1;
  static_assert(LPT % RING == 0, "ring size");
  u32 ring0[RING], ring1[RING];
#pragma unroll
  for (int d = 0; d < D; ++d) {
    ring0[d] = bsrc.limb0(0, d, g);
    ring1[d] = bsrc.limb1(0, d, g);
  }
  constexpr int kLanesPerRound = Grp<T>::kWhole ? 4 : 1;
#pragma unroll kLanesPerRound
  for (int o = 0; o < T; ++o) {
    static_for<0, LPT>([&](auto rc) {
      constexpr int r = decltype(rc)::value;
      u32 b0i, b1i;
      if (D > 0) {
        b0i = ring0[r % RING];
        b1i = ring1[r % RING];
        ring0[r % RING] = bsrc.limb0(o, r + D, g);
        ring1[r % RING] = bsrc.limb1(o, r + D, g);
      } else {
        b0i = bsrc.limb0(o, r, g);
        b1i = bsrc.limb1(o, r, g);
      }
      [[maybe_unused]] const u32 b0i2 = (SQ && !kDoubledA0) ? b0i + b0i : b0i;
      const u32 b1x = (SQ && !B1X2) ? b1i + b1i : b1i;  // squaring: 2 x0 x1 as x0 times the doubled limb of x1
      // window A: a0 * b0 (for a squaring the products sq_weight selects)
      auto product_a = [&](auto jc) {
        constexpr int j = decltype(jc)::value;
        constexpr int w = SQ ? sq_weight(LPT, j, r) : 1;
        if constexpr (w == 1) A[j] = mad64(a0[j], b0i, A[j]);
        else if constexpr (w == 2) A[j] = kDoubledA0 ? mad64(a0d[j], b0i, A[j]) : mad64(a0[j], b0i2, A[j]);
      };
      product_a(std::integral_constant<int, 0>{});
      const u32 qav = Grp<T>::kWhole ? ((u32)A[0] * n0inv) & maskv : 0u;  // used by whole-wavefront groups only
      const u32 qa = Grp<T>::kWhole ? g.bcast0(qav) : g.bcast0_masked((u32)A[0] * n0inv, maskv);
      static_for<1, LPT>(product_a);
      // window B: a0 * b1 + a1 * b0, minus the quotient digit of A on the lowest column of the integer
      B[0] = mad64(a0[0], b1x, B[0]);
      if (!SQ) B[0] = mad64(a1[0], b0i, B[0]);
      // only the lowest lane's term counts, and that lane's own digit is the broadcast one: a whole-wavefront
      // group takes it from the vector register, so that no scalar instruction waits on the broadcast
      B[0] = mad64(Grp<T>::kWhole ? (qav ^ maskv) : LIMB_MASK - qa, first, B[0]);
      const u32 qb = g.bcast0_masked((u32)B[0] * n0inv, maskv);
#pragma unroll
      for (int j = 1; j < LPT; ++j) {
        B[j] = mad64(a0[j], b1x, B[j]);
        if (!SQ) B[j] = mad64(a1[j], b0i, B[j]);
      }
      // both windows: add the multiple of n, hand the lowest column down, slide
      const u64 ta = mad64(qa, n[0], A[0]);
      const u64 tb = mad64(qb, n[0], B[0]);
      const u32 recv_a = g.from_upper_raw((u32)ta) & maskv;
      const u32 recv_b = g.from_upper_raw((u32)tb) & maskv;
      if (LPT > 1) {
        A[0] = mad64(qa, n[LPT > 1 ? 1 : 0], A[LPT > 1 ? 1 : 0]) + (ta >> LIMB_BITS);
        B[0] = mad64(qb, n[LPT > 1 ? 1 : 0], B[LPT > 1 ? 1 : 0]) + (tb >> LIMB_BITS);
#pragma unroll
        for (int j = 2; j < LPT; ++j) {
          A[j - 1] = mad64(qa, n[j], A[j]);
          B[j - 1] = mad64(qb, n[j], B[j]);
        }
        A[LPT - 1] = (u64)recv_a;
        B[LPT - 1] = (u64)recv_b;
      } else {
        A[0] = (u64)recv_a + (ta >> LIMB_BITS);
        B[0] = (u64)recv_b + (tb >> LIMB_BITS);
      }
    });
  }
  // B holds (x0 y1 + x1 y0 - m) / R + 1 modulo n: add n - 1
#pragma unroll
  for (int j = 0; j < LPT; ++j) B[j] += (u64)n[j];
  B[0] -= (u64)first;  // n is odd, so its lowest limb is at least 1
  hi_normalise<LPT, T>(A, g, eight);
  hi_normalise<LPT, T>(B, g, eight);
  u64 ca = 0, cb = 0;
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    const u64 va = A[j] + ca, vb = B[j] + cb;
    out0[j] = (u32)va & LIMB_MASK;
    out1[j] = (u32)vb & LIMB_MASK;
    ca = va >> LIMB_BITS;
    cb = vb >> LIMB_BITS;
  }
  if (T > 1) {
    out0[0] += g.from_lower((u32)ca);
    out1[0] += g.from_lower((u32)cb);
  }
}

// The pair product for a whole-wavefront group of 2 limbs per lane with both windows of column accumulators held
// at 8 times their value (see montmul_whole_x8: no masks, the carries as multiply-adds): 11 multiply-adds and 9
// other instructions per step where pairmul_core has 9 and 16. A column of the second window takes 3 products
// per step for 2 steps (or 2, one of them doubled), which 8 times over still fits 64 bits; with 3 limbs per
// lane it would not. Same result as pairmul_core, bit for bit.
template <int T, bool SQ>
__device__ __forceinline__ void pairmul_whole_x8(u32 (&out0)[2], u32 (&out1)[2], const u32 (&a0)[2], const u32 (&a1)[2],
                                                 const u32 (&b0)[2], const u32 (&b1)[2], const u32 (&n)[2], u32 n0inv,
                                                 const Grp<T>& g) {
  static_assert(Grp<T>::kWhole, "one integer per wavefront");
  constexpr int LPT = 2;
  const u32 eight = opaque_eight();
  // multiplicands times 2, multipliers times 4; a squaring forms 2 x0 x1 as (4 x0) (4 x1)
  u32 a0s[LPT], a1s[LPT], b0q[LPT], b1q[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    a0s[j] = a0[j] << 1;
    a1s[j] = a1[j] << 1;
    b0q[j] = b0[j] << 2;
    b1q[j] = b1[j] << 2;
  }
  u64 A[LPT] = {0, 0}, B[LPT] = {0, 0};
  if (g.k == 0) B[0] = 8;
  u32 first = (g.k == 0) ? 1u : 0u;
  asm volatile("" : "+v"(first));  // keeps the term below one multiply-add
#pragma unroll 4
  for (int o = 0; o < T; ++o) {
    static_for<0, LPT>([&](auto rc) {
      constexpr int r = decltype(rc)::value;
      const u32 b0i = (u32)__builtin_amdgcn_readlane((int)b0q[r], o);
      const u32 b1i = (u32)__builtin_amdgcn_readlane((int)b1q[r], o);
      A[0] = mad64(a0s[0], b0i, A[0]);
      const u32 qav = (u32)A[0] * n0inv;  // 8 q on the lowest lane, exactly
      const u32 qa = g.bcast0(qav);
      A[1] = mad64(a0s[1], b0i, A[1]);
      if (SQ) {
        B[0] = mad64(b0q[0], b1i, B[0]);
      } else {
        B[0] = mad64(a0s[0], b1i, B[0]);
        B[0] = mad64(a1s[0], b0i, B[0]);
      }
      B[0] = mad64(qav ^ (LIMB_MASK << 3), first, B[0]);  // 8 (2^29 - 1 - q) on the lowest lane
      const u32 qb = g.bcast0((u32)B[0] * n0inv);
      if (SQ) {
        B[1] = mad64(b0q[1], b1i, B[1]);
      } else {
        B[1] = mad64(a0s[1], b1i, B[1]);
        B[1] = mad64(a1s[1], b0i, B[1]);
      }
      const u64 ta = mad64(qa, n[0], A[0]);
      const u64 tb = mad64(qb, n[0], B[0]);
      const u32 recv_a = g.from_upper_raw((u32)ta);
      const u32 recv_b = g.from_upper_raw((u32)tb);
      A[0] = mad64((u32)(ta >> 32), eight, mad64(qa, n[1], A[1]));
      B[0] = mad64((u32)(tb >> 32), eight, mad64(qb, n[1], B[1]));
      A[1] = (u64)recv_a;
      B[1] = (u64)recv_b;
    });
  }
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    A[j] >>= 3;
    B[j] >>= 3;
  }
  // from here on as in pairmul_core: B holds (x0 y1 + x1 y0 - m) / R + 1 modulo n, add n - 1
#pragma unroll
  for (int j = 0; j < LPT; ++j) B[j] += (u64)n[j];
  B[0] -= (u64)first;
  hi_normalise<LPT, T>(A, g, eight);
  hi_normalise<LPT, T>(B, g, eight);
  u64 ca = 0, cb = 0;
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    const u64 va = A[j] + ca, vb = B[j] + cb;
    out0[j] = (u32)va & LIMB_MASK;
    out1[j] = (u32)vb & LIMB_MASK;
    ca = va >> LIMB_BITS;
    cb = vb >> LIMB_BITS;
  }
  out0[0] += g.from_lower((u32)ca);
  out1[0] += g.from_lower((u32)cb);
}

// (out0, out1) = (a0, a1) * (b0, b1) / R modulo n^2, b in registers (out may alias a and b)
template <int LPT, int T>
__device__ __forceinline__ void pairmul(u32 (&out0)[LPT], u32 (&out1)[LPT], const u32 (&a0)[LPT], const u32 (&a1)[LPT],
                                        const u32 (&b0)[LPT], const u32 (&b1)[LPT], const u32 (&n)[LPT], u32 n0inv,
                                        const Grp<T>& g) {
  if constexpr (Grp<T>::kWhole && LPT == 2) {
    pairmul_whole_x8<T, false>(out0, out1, a0, a1, b0, b1, n, n0inv, g);
  } else {
    BRegs2<LPT, T> src = {b0, b1};
    pairmul_core<LPT, T, BRegs2<LPT, T>, false>(out0, out1, a0, a1, src, n, n0inv, g);
  }
}
// b = 2 NL limbs at `bmem` ([b0][b1]), the same array for every lane of the group
template <int LPT, int T>
__device__ __forceinline__ void pairmul_mem(u32 (&out0)[LPT], u32 (&out1)[LPT], const u32 (&a0)[LPT],
                                            const u32 (&a1)[LPT], const u32* bmem, const u32 (&n)[LPT], u32 n0inv,
                                            const Grp<T>& g) {
  BMem2<LPT, T> src = {bmem};
  pairmul_core<LPT, T, BMem2<LPT, T>, false>(out0, out1, a0, a1, src, n, n0inv, g);
}
// (out0, out1) = (a0, a1)^2 / R modulo n^2
template <int LPT, int T>
__device__ __forceinline__ void pairsqr(u32 (&out0)[LPT], u32 (&out1)[LPT], const u32 (&a0)[LPT], const u32 (&a1)[LPT],
                                        const u32 (&n)[LPT], u32 n0inv, const Grp<T>& g) {
  if constexpr (Grp<T>::kWhole && LPT == 2) {
    pairmul_whole_x8<T, true>(out0, out1, a0, a1, a0, a1, n, n0inv, g);
  } else if constexpr (T > 1) {
    // double x1 once, not limb by limb as it is read
    u32 a1d[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) a1d[j] = a1[j] + a1[j];
    BRegs2<LPT, T> src = {a0, a1d};
    pairmul_core<LPT, T, BRegs2<LPT, T>, true, true>(out0, out1, a0, a1, src, n, n0inv, g);
  } else {
    BRegs2<LPT, T> src = {a0, a1};
    pairmul_core<LPT, T, BRegs2<LPT, T>, true>(out0, out1, a0, a1, src, n, n0inv, g);
  }
}

// Full carry propagation of signed lazy limbs (|x[j]| < 2^30): afterwards every
// limb is in [0, 2^29) and the return value (the same on all lanes of the
// group) is the carry out of the top limb: 0 for a value in [0, 2^(29*NL)),
// -1 for a negative value (then the limbs hold value + 2^(29*NL)).
template <int LPT, int T>
__device__ __forceinline__ int resolve(s32 (&x)[LPT], const Grp<T>& g) {
  int top = 0;
  bool more;
  do {
    s32 c = 0;
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
      s32 v = x[j] + c;
      x[j] = v & (s32)LIMB_MASK;
      c = v >> LIMB_BITS;  // arithmetic
    }
    if (T == 1) {
      top += c;
      more = false;
    } else {
      if (g.k == T - 1) top += c;
      s32 cin = (s32)g.from_lower((u32)c);
      x[0] += cin;
      more = wave_any(cin != 0);
    }
  } while (more);
  if (T > 1) top = (int)g.bcast((u32)top, T - 1);
  return top;
}

template <int LPT, int T>
__device__ __forceinline__ int resolve(u32 (&x)[LPT], const Grp<T>& g) {
  s32 t[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) t[j] = (s32)x[j];
  int top = resolve<LPT, T>(t, g);
#pragma unroll
  for (int j = 0; j < LPT; ++j) x[j] = (u32)t[j];
  return top;
}

// x mod n for a lazy x < 2n: canonical limbs, value in [0, n).
template <int LPT, int T>
__device__ __forceinline__ void canonicalise(u32 (&x)[LPT], const u32 (&n)[LPT], const Grp<T>& g) {
  resolve<LPT, T>(x, g);
  s32 d[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) d[j] = (s32)x[j] - (s32)n[j];
  int top = resolve<LPT, T>(d, g);
  if (top >= 0) {
#pragma unroll
    for (int j = 0; j < LPT; ++j) x[j] = (u32)d[j];
  }
}

// out = (a - b) mod n for canonical a, b in [0, n).
template <int LPT, int T>
__device__ __forceinline__ void sub_mod(u32 (&out)[LPT], const u32 (&a)[LPT], const u32 (&b)[LPT],
                                        const u32 (&n)[LPT], const Grp<T>& g) {
  s32 d[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) d[j] = (s32)a[j] - (s32)b[j];
  int top = resolve<LPT, T>(d, g);
  // every group of the wave takes the same path through the cross-lane code
#pragma unroll
  for (int j = 0; j < LPT; ++j) d[j] += (top < 0) ? (s32)n[j] : 0;
  resolve<LPT, T>(d, g);
#pragma unroll
  for (int j = 0; j < LPT; ++j) out[j] = (u32)d[j];
}

// Plain product of canonical a and b (2*NL limbs): lo = low NL limbs, and when
// WANT_HI also hi = high NL limbs, both canonical. Same sliding window as
// montmul without the modulus: step i emits result limb i from lane 0's
// lowest column; what is left in the window at the end is the high half.
template <int LPT, int T, bool WANT_HI>
__device__ __forceinline__ void mul_plain(u32 (&lo)[LPT], u32 (&hi)[LPT], const u32 (&a)[LPT], const u32 (&b)[LPT],
                                          const Grp<T>& g) {
  static_assert(LPT <= 18, "a column must not collect more than 36 products");
  const u32 eight = opaque_eight();
  [[maybe_unused]] const u32 maskv = opaque_mask();
  u64 A[LPT];
  u32 res[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    A[j] = 0;
    res[j] = 0;
  }
#pragma unroll 1
  for (int o = 0; o < T; ++o) {
    const int src = g.base_addr + (o << 2);
#pragma unroll
    for (int r = 0; r < LPT; ++r) {
      u32 bi = (T == 1) ? b[r] : (u32)__builtin_amdgcn_ds_bpermute(src, (int)b[r]);
#pragma unroll
      for (int j = 0; j < LPT; ++j) A[j] = mad64(a[j], bi, A[j]);
      u32 low = (u32)A[0] & LIMB_MASK;
      u64 carry = A[0] >> LIMB_BITS;
      u32 digit = g.bcast(low, 0);
      if (g.k == o) res[r] = digit;
      u32 recv = g.from_upper(low);  // nothing enters above the top lane
      if (LPT > 1) {
        A[0] = A[1] + carry;
#pragma unroll
        for (int j = 2; j < LPT; ++j) A[j - 1] = A[j];
        A[LPT - 1] = (u64)recv;
      } else {
        A[0] = (u64)recv + carry;
      }
    }
  }
  // One product per column and step here, so the bound of montmul_core holds with room to spare;
  // one pass before the compression keeps the limbs and the carry to the next lane small.
  hi_normalise<LPT, T>(A, g, eight);
  if (WANT_HI) {
    u64 c = 0;
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
      u64 v = A[j] + c;
      hi[j] = (u32)v & LIMB_MASK;
      c = v >> LIMB_BITS;
    }
    if (T > 1) hi[0] += g.from_lower((u32)c);
    resolve<LPT, T>(hi, g);
  }
#pragma unroll
  for (int j = 0; j < LPT; ++j) lo[j] = res[j];
}

// out = a * b mod 2^(29*NL)
template <int LPT, int T>
__device__ __forceinline__ void mullo(u32 (&out)[LPT], const u32 (&a)[LPT], const u32 (&b)[LPT], const Grp<T>& g) {
  u32 unused[LPT];
  mul_plain<LPT, T, false>(out, unused, a, b, g);
}

// (hi, lo) = a * b
template <int LPT, int T>
__device__ __forceinline__ void mulwide(u32 (&lo)[LPT], u32 (&hi)[LPT], const u32 (&a)[LPT], const u32 (&b)[LPT],
                                        const Grp<T>& g) {
  mul_plain<LPT, T, true>(lo, hi, a, b, g);
}

// ---------------------------------------------------------------------------
// memory <-> registers
// ---------------------------------------------------------------------------

// limbs [k*LPT, (k+1)*LPT) of a limb array (internal format)
template <int LPT, int T>
__device__ __forceinline__ void load_limbs(u32 (&x)[LPT], const u32* p, const Grp<T>& g) {
  const u32* q = p + g.k * LPT;
  const bool live = g.live();
#pragma unroll
  for (int j = 0; j < LPT; ++j) x[j] = live ? q[j] : 0u;
}
template <int LPT, int T>
__device__ __forceinline__ void store_limbs(u32* p, const u32 (&x)[LPT], const Grp<T>& g) {
  u32* q = p + g.k * LPT;
  if (g.live()) {
#pragma unroll
    for (int j = 0; j < LPT; ++j) q[j] = x[j];
  }
}
template <int LPT>
__device__ __forceinline__ void zero_limbs(u32 (&x)[LPT]) {
#pragma unroll
  for (int j = 0; j < LPT; ++j) x[j] = 0;
}

// limbs [k*LPT, (k+1)*LPT) of an array that holds only `valid` limbs (zero above them)
template <int LPT, int T>
__device__ __forceinline__ void load_limbs_below(u32 (&x)[LPT], const u32* p, int valid, const Grp<T>& g) {
#pragma unroll
  for (int j = 0; j < LPT; ++j) x[j] = (g.live() && g.k * LPT + j < valid) ? p[g.k * LPT + j] : 0u;
}

// This lane's 29-bit limbs, counted from limb `first_limb` of the integer, cut out of an array
// of `nwords` little-endian 32-bit words (bits past the array read as zero).
template <int LPT, int T>
__device__ __forceinline__ void load_words_as_limbs(u32 (&x)[LPT], const u32* wp, int nwords, const Grp<T>& g,
                                                    int first_limb = 0) {
#pragma unroll
  for (int j = 0; j < LPT; ++j) {
    int bitpos = (first_limb + g.k * LPT + j) * LIMB_BITS;
    int wi = bitpos >> 5;
    int sh = bitpos & 31;
    u32 lo = (wi < nwords) ? wp[wi] : 0u;
    u32 hi = (wi + 1 < nwords) ? wp[wi + 1] : 0u;
    u64 v = ((u64)hi << 32) | lo;
    x[j] = g.live() ? (u32)(v >> sh) & LIMB_MASK : 0u;
  }
}

// 32-bit word `wi` of the integer whose canonical 29-bit limbs are limbs[0..nl)
__device__ __forceinline__ u32 word_from_limbs(const u32* limbs, int nl, int wi) {
  int bitpos = wi << 5;
  int li = bitpos / LIMB_BITS;
  int sh = bitpos - li * LIMB_BITS;  // 0..28
  u64 v = 0;
  if (li < nl) v = (u64)limbs[li] >> sh;
  if (li + 1 < nl) v |= (u64)limbs[li + 1] << (LIMB_BITS - sh);
  if (li + 2 < nl) v |= (u64)limbs[li + 2] << (2 * LIMB_BITS - sh);
  return (u32)v;
}

}  // namespace dev
}  // namespace haflo
