// Import / export of ciphertexts, ciphertext addition, fixed-point encoding
// and decoding: kernels and their C entry points.
#include "kernels_common.hpp"

// launch and access tuning of the two HBM-bound kernels
#ifndef HAFLO_DECODE_BATCH
#define HAFLO_DECODE_BATCH 8
#endif
#ifndef HAFLO_DECODE_BLOCKS_PER_CU
#define HAFLO_DECODE_BLOCKS_PER_CU 32
#endif
#ifndef HAFLO_DECODE_NONTEMPORAL
#define HAFLO_DECODE_NONTEMPORAL 1
#endif
#ifndef HAFLO_ENCODE_NONTEMPORAL
#define HAFLO_ENCODE_NONTEMPORAL 1
#endif

using namespace haflo;
using namespace haflo::dev;

namespace {

// canonical 32-bit-limb ciphertexts -> internal (radix 2^29, Montgomery form)
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_import(ModRef M, const u32* __restrict__ canon, int nwords,
                                                          u32* __restrict__ out, u32* status, size_t count) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  u32 r2[LPT];
  load_limbs<LPT, T>(r2, M.r2, g);
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 x[LPT];
    if (active) load_words_as_limbs<LPT, T>(x, canon + item * (size_t)nwords, nwords, g);
    else zero_limbs<LPT>(x);
    s32 d[LPT];
#pragma unroll
    for (int j = 0; j < LPT; ++j) d[j] = (s32)x[j] - (s32)mod.n[j];
    int top = resolve<LPT, T>(d, g);
    if (top >= 0) {  // value >= n^2: not a residue
      zero_limbs<LPT>(x);
      if (active && g.k == 0 && status) atomicOr(status, HAFLO_ST_RANGE);
    }
    montmul<LPT, T>(x, x, r2, mod.n, mod.n0inv, g);
    canonicalise<LPT, T>(x, mod.n, g);
    if (active) store_limbs<LPT, T>(out + item * (size_t)NL, x, g);
  }
}

// internal -> canonical 32-bit limbs; the radix change goes through LDS
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_export(ModRef M, const u32* __restrict__ in, u32* __restrict__ canon,
                                                          int nwords, size_t count) {
  constexpr int NL = LPT * T;
  __shared__ u32 stage[kBlockThreads * LPT];
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
    u32* mine = stage + bt.gib * NL;
#pragma unroll
    for (int j = 0; j < LPT; ++j) mine[g.k * LPT + j] = x[j];
    __syncthreads();
    if (active)
      for (int w = g.k; w < nwords; w += T) canon[item * (size_t)nwords + w] = word_from_limbs(mine, NL, w);
    __syncthreads();
  }
}

// out = c1 * c2 mod n^2 on internal ciphertexts (one Montgomery product)
template <int LPT, int T>
__global__ __launch_bounds__(kBlockThreads) void k_add(ModRef M, const u32* __restrict__ c1, const u32* __restrict__ c2,
                                                       u32* __restrict__ out, size_t count) {
  constexpr int NL = LPT * T;
  Grp<T> g;
  Batch<T> bt;
  ModRegs<LPT> mod;
  load_mod<LPT, T>(mod, M, g);
  for (size_t base = bt.first(); base < count; base += bt.stride()) {
    size_t item = base + bt.gib;
    bool active = item < count;
    u32 a[LPT], b[LPT];
    if (active) {
      load_limbs<LPT, T>(a, c1 + item * (size_t)NL, g);
      load_limbs<LPT, T>(b, c2 + item * (size_t)NL, g);
    } else {
      zero_limbs<LPT>(a);
      zero_limbs<LPT>(b);
    }
    montmul<LPT, T>(a, a, b, mod.n, mod.n0inv, g);
    canonicalise<LPT, T>(a, mod.n, g);
    if (active) store_limbs<LPT, T>(out + item * (size_t)NL, a, g);
  }
}

// rint(v * 2^s) in binary64 with int64 range check; returns false when undefined
__device__ __forceinline__ bool quantise(float v, int scale_bits, long long& q) {
  double sc = __builtin_ldexp((double)v, scale_bits);
  // false for NaN, +-inf and anything outside [-2^63, 2^63)
  if (!(sc >= -9223372036854775808.0 && sc < 9223372036854775808.0)) {
    q = 0;
    return false;
  }
  q = (long long)__builtin_rint(sc);
  return true;
}

// Signed fixed-point encoding to residues mod n. A wavefront takes 64 elements at a time: every
// lane quantises one of them (one coalesced read of the inputs), then the wavefront writes the
// 64 * Lp words in Lp/4 fully coalesced stores of one 16-byte quad per lane, each lane fetching
// the quantised integer of the element its quad belongs to from the lane that holds it. 64 is a
// multiple of the quads per element, so a lane keeps its quad index, and with it its words of n.
// A negative q is n - |q|: |q| < 2^64 only touches the two lowest words, above them the borrow
// runs through zero words of n up to its first non-zero word `z`.
// With a second input v2 the encoded integer is q(v) - 2 q(v2) (the plaintext part of the fore
// gradient); both must then stay below 2^61 in magnitude.
__global__ __launch_bounds__(kBlockThreads) void k_encode(const float* __restrict__ v, const float* __restrict__ v2,
                                                          int scale_bits, const u32* __restrict__ nw, int lp, int z,
                                                          u32* __restrict__ plain, u32* __restrict__ status,
                                                          size_t count) {
  const int qpi = lp >> 2;  // quads per element: 4, 8, 16 or 32
  const int qshift = 31 - __builtin_clz((unsigned)qpi);
  const int lane = (int)(threadIdx.x & (WAVE - 1));
  const int quad = lane & (qpi - 1);
  const int per_store = WAVE >> qshift;  // elements one store of the wavefront covers
  const size_t wave = ((size_t)blockIdx.x * blockDim.x + threadIdx.x) / WAVE;
  const size_t nwaves = ((size_t)gridDim.x * blockDim.x) / WAVE;
  const u64 nlo = (u64)nw[0] | ((u64)nw[1] << 32);
  u32 nq[4];  // this quad's words of n
#pragma unroll
  for (int i = 0; i < 4; ++i) nq[i] = nw[quad * 4 + i];
  const size_t tiles = (count + WAVE - 1) / WAVE;
  for (size_t tile = wave; tile < tiles; tile += nwaves) {
    const size_t mine = tile * WAVE + (size_t)lane;
    long long q = 0;
    bool ok = true;
    if (mine < count) {
      ok = quantise(v[mine], scale_bits, q);
      if (v2) {
        long long q2;
        const long long lim = 1ll << 61;
        ok = quantise(v2[mine], scale_bits, q2) && ok && q > -lim && q < lim && q2 > -lim && q2 < lim;
        q = ok ? q - 2 * q2 : 0;
      }
      if (status) status[mine] = ok ? HAFLO_ST_OK : HAFLO_ST_RANGE;
    }
    const int qlo = (int)(u32)(u64)q, qhi = (int)(u32)((u64)q >> 32);
#pragma unroll 1
    for (int t = 0; t < qpi; ++t) {
      const int src = t * per_store + (lane >> qshift);  // the lane that quantised this quad's element
      const u64 sq = (u64)(u32)__builtin_amdgcn_ds_bpermute(src << 2, qlo) |
                     ((u64)(u32)__builtin_amdgcn_ds_bpermute(src << 2, qhi) << 32);
      const size_t item = tile * WAVE + (size_t)src;
      if (item >= count) continue;
      u32 w[4] = {0u, 0u, 0u, 0u};
      if ((long long)sq >= 0) {
        if (quad == 0) {
          w[0] = (u32)sq;
          w[1] = (u32)(sq >> 32);
        }
      } else {
        const u64 a = 0ull - sq;  // |q| <= 2^63
        const u32 borrow = nlo < a ? 1u : 0u;
        if (quad == 0) {
          const u64 d = nlo - a;
          w[0] = (u32)d;
          w[1] = (u32)(d >> 32);
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int j = quad * 4 + i;
          if (j >= 2) w[i] = (j < z) ? (0u - borrow) : (j == z ? nq[i] - borrow : nq[i]);
        }
      }
      typedef u32 quad_t __attribute__((vector_size(16)));
      const quad_t o = {w[0], w[1], w[2], w[3]};
      quad_t* dst = reinterpret_cast<quad_t*>(plain) + (item * (size_t)qpi + (size_t)quad);
      if (HAFLO_ENCODE_NONTEMPORAL) __builtin_nontemporal_store(o, dst);
      else *dst = o;
    }
  }
}

__global__ __launch_bounds__(kBlockThreads) void k_encode_exponents(const float* __restrict__ x, int scale_bits,
                                                                    int* __restrict__ e, u32* __restrict__ status,
                                                                    size_t count) {
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < count;
       idx += (size_t)gridDim.x * blockDim.x) {
    long long q;
    bool ok = quantise(x[idx], scale_bits, q);
    if (ok && (q < -2147483648ll || q > 2147483647ll)) ok = false;
    e[idx] = ok ? (int)q : 0;
    if (status) status[idx] = ok ? HAFLO_ST_OK : HAFLO_ST_RANGE;
  }
}

// Decoding: LPI = Lp/4 lanes read one element's words as 16-byte quads (coalesced). A decodable residue is
// either below 2^63 (q = m) or within 2^63 of n (q = m - n); everything else leaves int64 and is flagged,
// including the whole middle of [0, n) around floor(n/2), so the comparison with floor(n/2) itself never has
// to be made: m < 2^64 iff all words above the low two are zero, and n - m < 2^64 iff the words above the
// low two equal those of n (no borrow out of the low two words) or of n - 2^64 (borrow). A lane group takes
// B = min(LPI, 8) consecutive elements per pass: their loads are all issued before the first is used
// (enough bytes in flight per compute unit to cover the HBM latency), and lane u of the group ends up
// holding the result of the group's element u, so that q, q / 2^scale and the status leave the wavefront as
// contiguous runs instead of one word per group.
constexpr int kDecodeBatchMax = HAFLO_DECODE_BATCH;
constexpr int decode_batch(int lpi) { return lpi < kDecodeBatchMax ? lpi : kDecodeBatchMax; }
template <int LPI>
__global__ __launch_bounds__(kBlockThreads) void k_decode(const u32* __restrict__ plain, const u32* __restrict__ nw,
                                                          const u32* __restrict__ nbw, int scale_bits,
                                                          long long* __restrict__ qout, double* __restrict__ vout,
                                                          u32* __restrict__ status, size_t count) {
  static_assert(LPI >= 4 && LPI <= 32 && (LPI & (LPI - 1)) == 0, "lanes per item");
  constexpr int B = decode_batch(LPI);
  const int lane = (int)(threadIdx.x & (WAVE - 1));
  const int li = lane & (LPI - 1);       // quad index inside the element
  const int gbase = lane - li;           // first lane of this element's group
  const u64 gmask = (LPI == 64) ? ~0ull : ((1ull << LPI) - 1ull);
  const int gpb = (int)blockDim.x / LPI;  // lane groups per block
  const int gib = (int)threadIdx.x / LPI;
  // this quad of n and of n - 2^64; the low two words of the element do not take part in the comparisons
  uint4 n4 = reinterpret_cast<const uint4*>(nw)[li];
  uint4 b4 = reinterpret_cast<const uint4*>(nbw)[li];
  const u64 nlo = (u64)n4.x | ((u64)n4.y << 32);  // used on lane 0 only
  const u32 keep = li == 0 ? 0u : ~0u;
  n4.x &= keep, n4.y &= keep, b4.x &= keep, b4.y &= keep;
  for (size_t base0 = (size_t)blockIdx.x * gpb * B; base0 < count; base0 += (size_t)gridDim.x * gpb * B) {
    const size_t first = base0 + (size_t)gib * B;  // this group's elements: first .. first + B - 1
    uint4 loaded[B];
#pragma unroll
    for (int u = 0; u < B; ++u) {
      loaded[u] = make_uint4(0u, 0u, 0u, 0u);
      if (first + u < count) {
        typedef u32 quad_t __attribute__((vector_size(16)));
        const quad_t* src = reinterpret_cast<const quad_t*>(plain) + ((first + u) * (size_t)LPI + li);
        const quad_t v = HAFLO_DECODE_NONTEMPORAL ? __builtin_nontemporal_load(src) : *src;
        loaded[u] = make_uint4(v[0], v[1], v[2], v[3]);
      }
    }
    long long my_q = 0;  // lane u < B: value and validity of element first + u
    bool my_ok = false;
#pragma unroll
    for (int u = 0; u < B; ++u) {
      const uint4 m4 = loaded[u];
      const u64 mlo = (u64)m4.x | ((u64)m4.y << 32);  // meaningful on lane 0
      const u32 hx = m4.x & keep, hy = m4.y & keep;
      const bool zero = (hx | hy | m4.z | m4.w) == 0u;
      const bool like_n = ((hx ^ n4.x) | (hy ^ n4.y) | (m4.z ^ n4.z) | (m4.w ^ n4.w)) == 0u;
      const bool like_b = ((hx ^ b4.x) | (hy ^ b4.y) | (m4.z ^ b4.z) | (m4.w ^ b4.w)) == 0u;
      const bool all_zero = ((__builtin_amdgcn_ballot_w64(zero) >> gbase) & gmask) == gmask;
      const bool all_n = ((__builtin_amdgcn_ballot_w64(like_n) >> gbase) & gmask) == gmask;
      const bool all_b = ((__builtin_amdgcn_ballot_w64(like_b) >> gbase) & gmask) == gmask;
      // lane 0: the low 64 bits of m and of n - m, and whether that subtraction borrows
      const u64 dlo = nlo - mlo;
      const bool borrow = nlo < mlo;
      const bool near_n = borrow ? all_b : all_n;  // n - m = dlo exactly
      const bool ok = all_zero ? (mlo < 0x8000000000000000ull) : (near_n && dlo <= 0x8000000000000000ull);
      const long long q = !ok ? 0ll : (all_zero ? (long long)mlo : (long long)(0ull - dlo));
      // hand lane 0's verdict to lane u
      const u32 q_lo = (u32)__builtin_amdgcn_ds_bpermute(gbase << 2, (int)(u32)(u64)q);
      const u32 q_hi = (u32)__builtin_amdgcn_ds_bpermute(gbase << 2, (int)(u32)((u64)q >> 32));
      const u32 ok0 = (u32)__builtin_amdgcn_ds_bpermute(gbase << 2, ok ? 1 : 0);
      if (li == u) {
        my_q = (long long)((u64)q_lo | ((u64)q_hi << 32));
        my_ok = ok0 != 0u;
      }
    }
    const size_t item = first + (size_t)li;
    if (li < B && item < count) {
      if (qout) __builtin_nontemporal_store(my_q, qout + item);
      if (vout) __builtin_nontemporal_store(__builtin_ldexp((double)my_q, -scale_bits), vout + item);
      if (status) __builtin_nontemporal_store((u32)(my_ok ? HAFLO_ST_OK : HAFLO_ST_RANGE), status + item);
    }
  }
}

}  // namespace

extern "C" {

int haflo_import_cipher(const haflo_ctx* ctx, const uint32_t* d_canon, void* d_cipher, uint32_t* d_status,
                        size_t count, void* stream) {
  if (!ctx || (count && (!d_canon || !d_cipher))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  const ModHost& m = ctx->N;
  const LaunchShape sh = launch_shape(ctx, count, m.t, 8);
  hipStream_t st = (hipStream_t)stream;
#define CALL(LPT, T) \
  HAFLO_LAUNCH((k_import<LPT, T>), sh, st, m.ref(), d_canon, ctx->lc, (u32*)d_cipher, d_status, count)
  HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  return hip_status(hipGetLastError());
}

int haflo_export_cipher(const haflo_ctx* ctx, const void* d_cipher, uint32_t* d_canon, size_t count, void* stream) {
  if (!ctx || (count && (!d_canon || !d_cipher))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  const ModHost& m = ctx->N;
  const LaunchShape sh = launch_shape(ctx, count, m.t, 8);
  hipStream_t st = (hipStream_t)stream;
#define CALL(LPT, T) HAFLO_LAUNCH((k_export<LPT, T>), sh, st, m.ref(), (const u32*)d_cipher, d_canon, ctx->lc, count)
  HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  return hip_status(hipGetLastError());
}

int haflo_add(const haflo_ctx* ctx, const void* d_c1, const void* d_c2, void* d_out, size_t count, void* stream) {
  if (!ctx || (count && (!d_c1 || !d_c2 || !d_out))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  const ModHost& m = ctx->N;
  const LaunchShape sh = launch_shape(ctx, count, m.t, 8);
  hipStream_t st = (hipStream_t)stream;
#define CALL(LPT, T) \
  HAFLO_LAUNCH((k_add<LPT, T>), sh, st, m.ref(), (const u32*)d_c1, (const u32*)d_c2, (u32*)d_out, count)
  HAFLO_DISPATCH_GEOMETRY(m, CALL);
#undef CALL
  return hip_status(hipGetLastError());
}

int haflo_encode_f32(const haflo_ctx* ctx, const float* d_v, uint32_t scale_bits, uint32_t* d_plain,
                     uint32_t* d_status, size_t count, void* stream) {
  if (!ctx || scale_bits > 62 || (count && (!d_v || !d_plain))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  int z = 2;
  while (z < ctx->lp && ctx->n.word(z) == 0) ++z;
  // the residues are written once and read by a later kernel: non-temporal stores from few, long-running
  // wavefronts (a plain device fill is fastest the same way: more blocks per compute unit write slower)
  const LaunchShape sh = launch_shape(ctx, count, 1, ctx->lp <= 32 ? 2 : 1);
  HAFLO_LAUNCH(k_encode, sh, (hipStream_t)stream, d_v, (const float*)nullptr, (int)scale_bits, ctx->d_n_words,
               ctx->lp, z, d_plain, d_status, count);
  return hip_status(hipGetLastError());
}

int haflo_fore_gradient(const haflo_ctx* ctx, const void* d_c_host, const float* d_logits_guest,
                        const float* d_label, const uint32_t* d_r, uint32_t scale_bits, void* d_out,
                        uint32_t* d_status, size_t count, void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx || scale_bits > 60 || (count && (!d_c_host || !d_logits_guest || !d_label || !d_r || !d_out)))
    return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  // workspace: [guest plaintexts][their encryptions][encryption workspace]
  const size_t plain_bytes = (count * (size_t)ctx->lp * 4 + 255) & ~(size_t)255;
  const size_t cipher_bytes = (count * (size_t)ctx->N.nl * 4 + 255) & ~(size_t)255;
  const size_t enc_bytes = haflo_workspace_bytes(ctx, HAFLO_OP_ENCRYPT, count, 0);
  if (!d_workspace || workspace_bytes < plain_bytes + cipher_bytes + enc_bytes) return HAFLO_EINVAL;
  uint32_t* plain = (uint32_t*)d_workspace;
  char* guest = (char*)d_workspace + plain_bytes;
  int z = 2;
  while (z < ctx->lp && ctx->n.word(z) == 0) ++z;
  const LaunchShape sh = launch_shape(ctx, count, 1, ctx->lp <= 32 ? 2 : 1);
  HAFLO_LAUNCH(k_encode, sh, (hipStream_t)stream, d_logits_guest, d_label, (int)scale_bits, ctx->d_n_words, ctx->lp,
               z, plain, d_status, count);
  int rc = haflo_encrypt(ctx, plain, d_r, guest, count, guest + cipher_bytes, enc_bytes, stream);
  if (rc != HAFLO_OK) return rc;
  return haflo_add(ctx, d_c_host, guest, d_out, count, stream);
}

int haflo_encode_exponents_f32(const float* d_x, uint32_t scale_bits, int32_t* d_e, uint32_t* d_status, size_t count,
                               void* stream) {
  if (scale_bits > 62 || (count && (!d_x || !d_e))) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  size_t need = (count + kBlockThreads - 1) / kBlockThreads;
  LaunchShape sh;
  sh.threads = kBlockThreads;
  sh.gpb = kBlockThreads;
  sh.blocks = (int)(need < 16384 ? need : 16384);
  HAFLO_LAUNCH(k_encode_exponents, sh, (hipStream_t)stream, d_x, (int)scale_bits, d_e, d_status, count);
  return hip_status(hipGetLastError());
}

int haflo_decode(const haflo_ctx* ctx, const uint32_t* d_plain, uint32_t scale_bits, int64_t* d_q, double* d_v,
                 uint32_t* d_status, size_t count, void* stream) {
  if (!ctx || scale_bits > 1000 || (count && !d_plain)) return HAFLO_EINVAL;
  if (count == 0) return HAFLO_OK;
  const int lpi = ctx->lp / 4;
  const LaunchShape sh = launch_shape(ctx, (count + decode_batch(lpi) - 1) / decode_batch(lpi), lpi, HAFLO_DECODE_BLOCKS_PER_CU);
  hipStream_t st = (hipStream_t)stream;
#define DECODE(LPI)                                                                                        \
  HAFLO_LAUNCH((k_decode<LPI>), sh, st, d_plain, ctx->d_n_words, ctx->d_nb_words, (int)scale_bits,         \
               (long long*)d_q, d_v, d_status, count)
  switch (lpi) {
    case 4: DECODE(4); break;
    case 8: DECODE(8); break;
    case 16: DECODE(16); break;
    case 32: DECODE(32); break;
    default: return HAFLO_EINVAL;
  }
#undef DECODE
  return hip_status(hipGetLastError());
}

}  // extern "C"
