// Exponentiation-bound operators: encryption, decryption through p^2 and q^2,
// ciphertext-by-scalar multiplication. Kernels and their C entry points.
#include "kernels_common.hpp"

using namespace haflo;
using namespace haflo::dev;

namespace {

constexpr int kModexpBlocksPerCu = 4;  // resident blocks assumed when sizing window-table workspace

// E(m) = (1 + m n) r^n mod n^2, output in internal form.
//   r^n: fixed-exponent sliding-window power in Montgomery form.
//   (1 + m n) R = montmul(m, n R^2) + R, formed lazily and folded in with one
//   more Montgomery product.
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_encrypt(ModRef M, SchedRef S, const u32* __restrict__ k1,
                                                           const u32* __restrict__ plain, const u32* __restrict__ rnd,
                                                           int lp, u32* __restrict__ out, u32* __restrict__ tables,
                                                           size_t count) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  u32* table = tables + bt.slot() * (size_t)S.table_len * NL;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 x[LPT], acc[LPT], t[LPT];
    if (active) load_words_as_limbs<LPT, T>(x, rnd + item * (size_t)lp, lp, g);
    else zero_limbs<LPT>(x);
    load_limbs<LPT, T>(t, M.r2, g);
    montmul<LPT, T>(x, x, t, mod.n, mod.n0inv, g);
    modexp_fixed<LPT, T>(acc, x, mod, S, table, M.r1, g);
    if (active) load_words_as_limbs<LPT, T>(x, plain + item * (size_t)lp, lp, g);
    else zero_limbs<LPT>(x);
    load_limbs<LPT, T>(t, k1, g);
    montmul<LPT, T>(x, x, t, mod.n, mod.n0inv, g);
    load_limbs<LPT, T>(t, M.r1, g);
#pragma unroll
    for (int j = 0; j < LPT; ++j) x[j] += t[j];
    partial_norm<LPT, T>(x, g);
    montmul<LPT, T>(acc, acc, x, mod.n, mod.n0inv, g);
    canonicalise<LPT, T>(acc, mod.n, g);
    if (active) store_limbs<LPT, T>(out + item * (size_t)NL, acc, g);
  }
}

// c^k mod n^2 with one exponent plan for the whole batch
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_pow_bcast(ModRef M, SchedInline S, const u32* __restrict__ in,
                                                             u32* __restrict__ out, u32* __restrict__ tables,
                                                             size_t count) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  u32* table = tables + bt.slot() * (size_t)S.table_len * NL;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 x[LPT], acc[LPT];
    if (active) load_limbs<LPT, T>(x, in + item * (size_t)NL, g);
    else zero_limbs<LPT>(x);
    modexp_fixed<LPT, T>(acc, x, mod, S, table, M.r1, g);
    canonicalise<LPT, T>(acc, mod.n, g);
    if (active) store_limbs<LPT, T>(out + item * (size_t)NL, acc, g);
  }
}

// c^k mod n^2 with one unsigned 64-bit exponent per element: fixed 4-bit
// windows over a 16-entry table (entry 0 is the Montgomery one, so every
// window multiplies and lanes never diverge on the digit).
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_pow_u64(ModRef M, const u32* __restrict__ in,
                                                           const unsigned long long* __restrict__ kk,
                                                           u32* __restrict__ out, u32* __restrict__ tables,
                                                           size_t count) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  u32* table = tables + bt.slot() * (size_t)16 * NL;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 x[LPT], acc[LPT], t[LPT];
    u64 k = 0;
    if (active) {
      load_limbs<LPT, T>(x, in + item * (size_t)NL, g);
      k = kk[item];
    } else {
      zero_limbs<LPT>(x);
    }
    load_limbs<LPT, T>(t, M.r1, g);
    store_limbs<LPT, T>(table, t, g);
    store_limbs<LPT, T>(table + NL, x, g);
#pragma unroll
    for (int j = 0; j < LPT; ++j) t[j] = x[j];
#pragma unroll 1
    for (int i = 2; i < 16; ++i) {
      montmul<LPT, T>(t, t, x, mod.n, mod.n0inv, g);
      store_limbs<LPT, T>(table + (size_t)i * NL, t, g);
    }
    load_limbs<LPT, T>(acc, table + (size_t)(k >> 60) * NL, g);
#pragma unroll 1
    for (int wi = 14; wi >= 0; --wi) {
#pragma unroll 1
      for (int s = 0; s < 4; ++s) montmul<LPT, T>(acc, acc, acc, mod.n, mod.n0inv, g);
      u32 d = (u32)(k >> (4 * wi)) & 15u;
      load_limbs<LPT, T>(t, table + (size_t)d * NL, g);
      montmul<LPT, T>(acc, acc, t, mod.n, mod.n0inv, g);
    }
    canonicalise<LPT, T>(acc, mod.n, g);
    if (active) store_limbs<LPT, T>(out + item * (size_t)NL, acc, g);
  }
}

// Decryption stage A: internal ciphertext -> canonical residue mod n^2 in
// 29-bit limbs (workspace), ready to be split in halves.
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_dec_unmont(ModRef M, const u32* __restrict__ in,
                                                              u32* __restrict__ canon29, size_t count) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  u32 one[LPT];
  zero_limbs<LPT>(one);
  if (g.k == 0) one[0] = 1u;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 x[LPT];
    if (active) load_limbs<LPT, T>(x, in + item * (size_t)NL, g);
    else zero_limbs<LPT>(x);
    montmul<LPT, T>(x, x, one, mod.n, mod.n0inv, g);
    canonicalise<LPT, T>(x, mod.n, g);
    if (active) store_limbs<LPT, T>(canon29 + item * (size_t)NL, x, g);
  }
}

// Decryption stage B for one prime s (modulus s^2 of NL limbs): reduce the
// 2*NL-limb residue c = c_hi * R + c_lo into Montgomery form mod s^2
// (c R = c_lo R + c_hi R^2 = montmul(c_lo, R^2) + montmul(c_hi, R^3)), raise
// to s - 1, leave the Montgomery domain and store the canonical result.
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_dec_pow(ModRef M, SchedRef S, const u32* __restrict__ canon29,
                                                           u32* __restrict__ ypow, u32* __restrict__ tables,
                                                           size_t count) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  u32* table = tables + bt.slot() * (size_t)S.table_len * NL;
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 lo[LPT], hi[LPT], t[LPT], acc[LPT];
    if (active) {
      load_limbs<LPT, T>(lo, canon29 + item * (size_t)(2 * NL), g);
      load_limbs<LPT, T>(hi, canon29 + item * (size_t)(2 * NL) + NL, g);
    } else {
      zero_limbs<LPT>(lo);
      zero_limbs<LPT>(hi);
    }
    load_limbs<LPT, T>(t, M.r2, g);
    montmul<LPT, T>(lo, lo, t, mod.n, mod.n0inv, g);
    load_limbs<LPT, T>(t, M.r3, g);
    montmul<LPT, T>(hi, hi, t, mod.n, mod.n0inv, g);
#pragma unroll
    for (int j = 0; j < LPT; ++j) lo[j] += hi[j];
    partial_norm<LPT, T>(lo, g);
    modexp_fixed<LPT, T>(acc, lo, mod, S, table, M.r1, g);
    zero_limbs<LPT>(t);
    if (g.k == 0) t[0] = 1u;
    montmul<LPT, T>(acc, acc, t, mod.n, mod.n0inv, g);
    canonicalise<LPT, T>(acc, mod.n, g);
    if (active) store_limbs<LPT, T>(ypow + item * (size_t)NL, acc, g);
  }
}

// m_s = L_s(y) * h_s mod s for y = c^(s-1) mod s^2 (canonical, 2*NL limbs of
// which only the low NL matter): L_s(y) = (y - 1)/s is an exact quotient below
// s < 2^(29 NL), so it equals (y - 1) * s^-1 modulo 2^(29 NL).
template <int LPT, int T>
__device__ __forceinline__ void crt_branch(u32 (&ms)[LPT], const u32* ylow, bool active, const ModRegs<LPT>& mod,
                                           const u32* sinv, const u32* hsR, const Grp<T>& g) {
  u32 x[LPT], t[LPT];
  if (active) load_limbs<LPT, T>(x, ylow, g);
  else zero_limbs<LPT>(x);
  s32 d[LPT];
#pragma unroll
  for (int j = 0; j < LPT; ++j) d[j] = (s32)x[j];
  if (g.k == 0) d[0] -= 1;
  resolve<LPT, T>(d, g);  // modulo 2^(29 NL): a borrow out of the top is dropped
#pragma unroll
  for (int j = 0; j < LPT; ++j) x[j] = (u32)d[j];
  load_limbs<LPT, T>(t, sinv, g);
  mullo<LPT, T>(x, x, t, g);
  load_limbs<LPT, T>(t, hsR, g);
  montmul<LPT, T>(ms, x, t, mod.n, mod.n0inv, g);
  canonicalise<LPT, T>(ms, mod.n, g);
}

// Decryption stage C: both branches, then the Chinese remainder
// m = m_p + p * ((m_q - m_p) * p^-1 mod q), written as Lp 32-bit words.
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_dec_crt(ModRef MP, ModRef MQ, const u32* __restrict__ pinv2,
                                                           const u32* __restrict__ qinv2, const u32* __restrict__ hpR,
                                                           const u32* __restrict__ hqR, const u32* __restrict__ pinvqR,
                                                           const u32* __restrict__ yp, const u32* __restrict__ yq,
                                                           u32* __restrict__ plain, int lp, size_t count) {
  constexpr int NL = LPT * T;
  __shared__ u32 stage[kBlockThreads * LPT * 2];
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mp, mq;
  load_mod<LPT, T>(mp, MP, g);
  load_mod<LPT, T>(mq, MQ, g);
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 a[LPT], b[LPT], t[LPT], u[LPT];
    crt_branch<LPT, T>(a, yp + item * (size_t)(2 * NL), active, mp, pinv2, hpR, g);  // m_p
    crt_branch<LPT, T>(b, yq + item * (size_t)(2 * NL), active, mq, qinv2, hqR, g);  // m_q
    // (m_q - m_p) mod q; m_p < p < 2q so one conditional subtraction reduces it
#pragma unroll
    for (int j = 0; j < LPT; ++j) t[j] = a[j];
    canonicalise<LPT, T>(t, mq.n, g);
    sub_mod<LPT, T>(u, b, t, mq.n, g);
    load_limbs<LPT, T>(t, pinvqR, g);
    montmul<LPT, T>(u, u, t, mq.n, mq.n0inv, g);
    canonicalise<LPT, T>(u, mq.n, g);
    // p * u as a 2*NL-limb product: low half, then high half
    u32 lo[LPT], hi[LPT];
    mulwide<LPT, T>(lo, hi, mp.n, u, g);
#pragma unroll
    for (int j = 0; j < LPT; ++j) lo[j] += a[j];
    int carry = resolve<LPT, T>(lo, g);
    if (g.k == 0) hi[0] += (u32)carry;
    resolve<LPT, T>(hi, g);
    u32* mine = stage + bt.gib * (2 * NL);
#pragma unroll
    for (int j = 0; j < LPT; ++j) {
      mine[g.k * LPT + j] = lo[j];
      mine[NL + g.k * LPT + j] = hi[j];
    }
    __syncthreads();
    if (active)
      for (int w = g.k; w < lp; w += T) plain[item * (size_t)lp + w] = word_from_limbs(mine, 2 * NL, w);
    __syncthreads();
  }
}

void inline_schedule(SchedInline& si, const HostSched& h) {
  si.nsteps = (int)h.steps.size();
  for (int i = 0; i < si.nsteps && i < 64; ++i) si.steps[i] = h.steps[i];
  si.first = h.first;
  si.table_len = h.table_len;
  si.is_zero = h.is_zero;
}

LaunchShape modexp_shape(const haflo_ctx* ctx, size_t count, int t) {
  return launch_shape(ctx, count, t, kModexpBlocksPerCu);
}

}  // namespace

namespace haflo {
// window tables: one slot per resident lane group
size_t ws_encrypt(const haflo_ctx* ctx, size_t count) {
  return modexp_shape(ctx, count, ctx->N.t).slots() * (size_t)ctx->sched_n.h.table_len * ctx->N.nl * 4;
}
// sized for the per-element variant (16 entries); the broadcast variant never needs more
size_t ws_scalar_mul(const haflo_ctx* ctx, size_t count) {
  return modexp_shape(ctx, count, ctx->N.t).slots() * (size_t)16 * ctx->N.nl * 4;
}
// layout: [canon29: count*N.nl][yp: count*P2.nl][yq: count*Q2.nl][tables]
size_t ws_decrypt(const haflo_ctx* ctx, size_t count) {
  if (!ctx->has_priv) return 0;
  size_t tl = (size_t)std::max(ctx->sched_pm1.h.table_len, ctx->sched_qm1.h.table_len);
  return (count * (size_t)ctx->N.nl + 2 * count * (size_t)ctx->P2.nl +
          modexp_shape(ctx, count, ctx->P2.t).slots() * tl * ctx->P2.nl) * 4;
}
}  // namespace haflo

extern "C" {

int haflo_encrypt(const haflo_ctx* ctx, const uint32_t* d_plain, const uint32_t* d_r, void* d_cipher, size_t count,
                  void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx || (count && (!d_plain || !d_r || !d_cipher))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  if (!d_workspace || workspace_bytes < ws_encrypt(ctx, count)) return HAFLO_EINVAL;
  const ModHost& m = ctx->N;
  const LaunchShape sh = modexp_shape(ctx, count, m.t);
  hipStream_t st = (hipStream_t)stream;
#define CALL(LPT, T)                                                                                          \
  HAFLO_LAUNCH((k_encrypt<LPT, T>), sh, st, m.ref(), ctx->sched_n.ref(), ctx->d_k1, d_plain, d_r, ctx->lp,    \
               (u32*)d_cipher, (u32*)d_workspace, count)
  HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  return hip_status(hipGetLastError());
}

int haflo_scalar_mul_u64(const haflo_ctx* ctx, const void* d_c, const uint64_t* d_k, void* d_out, size_t count,
                         void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx || (count && (!d_c || !d_k || !d_out))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  if (!d_workspace || workspace_bytes < ws_scalar_mul(ctx, count)) return HAFLO_EINVAL;
  const ModHost& m = ctx->N;
  const LaunchShape sh = modexp_shape(ctx, count, m.t);
  hipStream_t st = (hipStream_t)stream;
#define CALL(LPT, T)                                                                                   \
  HAFLO_LAUNCH((k_pow_u64<LPT, T>), sh, st, m.ref(), (const u32*)d_c, (const unsigned long long*)d_k,  \
               (u32*)d_out, (u32*)d_workspace, count)
  HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  return hip_status(hipGetLastError());
}

int haflo_scalar_mul_i64_bcast(const haflo_ctx* ctx, const void* d_c, int64_t k, void* d_out, size_t count,
                               void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx || (count && (!d_c || !d_out))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  if (!d_workspace || workspace_bytes < ws_scalar_mul(ctx, count)) return HAFLO_EINVAL;
  const ModHost& m = ctx->N;
  hipStream_t st = (hipStream_t)stream;
  const u32* src = (const u32*)d_c;
  uint64_t mag = k < 0 ? 0ull - (uint64_t)k : (uint64_t)k;
  if (k < 0) {
    // a negative scalar is a power of the inverse: invert into d_out first
    int rc = invert_batch(ctx, src, (u32*)d_out, count, st);
    if (rc != HAFLO_OK) return rc;
    src = (const u32*)d_out;
  }
  SchedInline si;
  inline_schedule(si, make_schedule(Big(mag), 4));
  const LaunchShape sh = modexp_shape(ctx, count, m.t);
#define CALL(LPT, T) \
  HAFLO_LAUNCH((k_pow_bcast<LPT, T>), sh, st, m.ref(), si, src, (u32*)d_out, (u32*)d_workspace, count)
  HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  return hip_status(hipGetLastError());
}

int haflo_decrypt(const haflo_ctx* ctx, const void* d_cipher, uint32_t* d_plain, size_t count, void* d_workspace,
                  size_t workspace_bytes, void* stream) {
  if (!ctx || (count && (!d_cipher || !d_plain))) return HAFLO_EINVAL;
  if (!ctx->has_priv) return HAFLO_ENOPRIV;
  if (count == 0) return HAFLO_OK;
  if (!d_workspace || workspace_bytes < ws_decrypt(ctx, count)) return HAFLO_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  u32* canon29 = (u32*)d_workspace;
  u32* yp = canon29 + count * (size_t)ctx->N.nl;
  u32* yq = yp + count * (size_t)ctx->P2.nl;
  u32* tables = yq + count * (size_t)ctx->Q2.nl;
  {
    const ModHost& m = ctx->N;
    const LaunchShape sh = launch_shape(ctx, count, m.t, 8);
#define CALL(LPT, T) HAFLO_LAUNCH((k_dec_unmont<LPT, T>), sh, st, m.ref(), (const u32*)d_cipher, canon29, count)
    HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  }
  for (int side = 0; side < 2; ++side) {
    const ModHost& m = side ? ctx->Q2 : ctx->P2;
    const DevSched& s = side ? ctx->sched_qm1 : ctx->sched_pm1;
    u32* y = side ? yq : yp;
    const LaunchShape sh = modexp_shape(ctx, count, m.t);
#define CALL(LPT, T) HAFLO_LAUNCH((k_dec_pow<LPT, T>), sh, st, m.ref(), s.ref(), (const u32*)canon29, y, tables, count)
    HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  }
  {
    const ModHost& m = ctx->P;
    const LaunchShape sh = launch_shape(ctx, count, m.t, 8);
#define CALL(LPT, T)                                                                                            \
  HAFLO_LAUNCH((k_dec_crt<LPT, T>), sh, st, ctx->P.ref(), ctx->Q.ref(), ctx->d_pinv, ctx->d_qinv, ctx->d_hp,    \
               ctx->d_hq, ctx->d_pinvq, (const u32*)yp, (const u32*)yq, d_plain, ctx->lp, count)
    HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  }
  return hip_status(hipGetLastError());
}

}  // extern "C"
