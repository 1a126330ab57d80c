// Import / export of ciphertexts, ciphertext addition, fixed-point encoding
// and decoding: kernels and their C entry points.
#include "kernels_common.hpp"

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
      uint4 o;
      o.x = w[0];
      o.y = w[1];
      o.z = w[2];
      o.w = w[3];
      reinterpret_cast<uint4*>(plain)[item * (size_t)qpi + (size_t)quad] = o;
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

// Decoding: LPI = Lp/4 lanes read one element's words as 16-byte quads
// (coalesced), decide m > floor(n/2) with a ballot, form n - m with a
// generate/propagate borrow look-ahead across the lanes, and lane 0 of the
// element checks the int64 range and writes q and q / 2^scale.
template <int LPI>
__global__ __launch_bounds__(kBlockThreads) void k_decode(const u32* __restrict__ plain, const u32* __restrict__ nw,
                                                          const u32* __restrict__ halfw, int scale_bits,
                                                          long long* __restrict__ qout, double* __restrict__ vout,
                                                          u32* __restrict__ status, size_t count) {
  static_assert(LPI >= 4 && LPI <= 32 && (LPI & (LPI - 1)) == 0, "lanes per item");
  const int lane = (int)(threadIdx.x & (WAVE - 1));
  const int li = lane & (LPI - 1);       // quad index inside the element
  const int gbase = lane - li;           // first lane of this element's group
  const u64 gmask = (LPI == 64) ? ~0ull : ((1ull << LPI) - 1ull);
  const int ipb = (int)blockDim.x / LPI;  // items per block
  const int iib = (int)threadIdx.x / LPI;
  const uint4 n4 = reinterpret_cast<const uint4*>(nw)[li];
  const uint4 h4 = reinterpret_cast<const uint4*>(halfw)[li];
  for (size_t base = (size_t)blockIdx.x * ipb; base < count; base += (size_t)gridDim.x * ipb) {
    size_t item = base + iib;
    bool active = item < count;
    uint4 m4 = make_uint4(0u, 0u, 0u, 0u);
    if (active) m4 = reinterpret_cast<const uint4*>(plain)[item * (size_t)LPI + li];
    // lexicographic compare of this quad with floor(n/2), most significant word first
    int cmp = 0;
    if (m4.w != h4.w) cmp = m4.w > h4.w ? 1 : -1;
    else if (m4.z != h4.z) cmp = m4.z > h4.z ? 1 : -1;
    else if (m4.y != h4.y) cmp = m4.y > h4.y ? 1 : -1;
    else if (m4.x != h4.x) cmp = m4.x > h4.x ? 1 : -1;
    u64 gt = (__builtin_amdgcn_ballot_w64(cmp > 0) >> gbase) & gmask;
    u64 lt = (__builtin_amdgcn_ballot_w64(cmp < 0) >> gbase) & gmask;
    bool neg = gt > lt;  // higher lanes hold more significant words
    // d = n - m, quad-local with borrow-in 0
    u64 nlo = (u64)n4.x | ((u64)n4.y << 32), nhi = (u64)n4.z | ((u64)n4.w << 32);
    u64 mlo = (u64)m4.x | ((u64)m4.y << 32), mhi = (u64)m4.z | ((u64)m4.w << 32);
    u64 dlo = nlo - mlo;
    u64 b0 = nlo < mlo ? 1ull : 0ull;
    u64 dhi = nhi - mhi - b0;
    bool gen = (nhi < mhi) || (nhi == mhi && b0);  // borrow out with borrow-in 0
    bool prop = (dlo == 0ull && dhi == 0ull);      // a borrow-in would pass through
    u64 G = (__builtin_amdgcn_ballot_w64(gen) >> gbase) & gmask;
    u64 P = (__builtin_amdgcn_ballot_w64(prop) >> gbase) & gmask;
    // carries of the addition U + V with U = G|P, V = G are the borrows into each lane
    u64 U = G | P, V = G;
    u64 bin = ((U + V) ^ U ^ V) >> li & 1ull;
    if (bin) {
      u64 t = dlo;
      dlo = t - 1ull;
      if (t == 0ull) dhi -= 1ull;
    }
    u64 rlo = neg ? dlo : mlo;
    u64 rhi = neg ? dhi : mhi;
    // magnitude must fit 64 bits: everything above the low two words is zero
    bool high_nonzero = (li == 0) ? (rhi != 0ull) : ((rlo | rhi) != 0ull);
    u64 nz = (__builtin_amdgcn_ballot_w64(high_nonzero) >> gbase) & gmask;
    if (active && li == 0) {
      bool ok = (nz == 0ull) && (neg ? (rlo <= 0x8000000000000000ull) : (rlo < 0x8000000000000000ull));
      long long q = 0;
      if (ok) q = neg ? (long long)(0ull - rlo) : (long long)rlo;
      if (qout) qout[item] = q;
      if (vout) vout[item] = __builtin_ldexp((double)q, -scale_bits);
      if (status) status[item] = ok ? HAFLO_ST_OK : HAFLO_ST_RANGE;
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
  const LaunchShape sh = launch_shape(ctx, count, 1, 8);
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
  const LaunchShape sh = launch_shape(ctx, count, 1, 8);
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
  const LaunchShape sh = launch_shape(ctx, count, lpi, 16);
  hipStream_t st = (hipStream_t)stream;
#define DECODE(LPI)                                                                                        \
  HAFLO_LAUNCH((k_decode<LPI>), sh, st, d_plain, ctx->d_n_words, ctx->d_halfn_words, (int)scale_bits,      \
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
