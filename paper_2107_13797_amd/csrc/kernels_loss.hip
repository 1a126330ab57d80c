// Encrypted second-order Taylor loss of logistic regression, built from the ciphertext operators:
// a launch sequence with every intermediate on the device.
//
//   sum_i ( -1/2 y_i u_i + 1/8 u_i^2 ),  u_i = u_host,i + u_guest,i
// scaled by 8 * 2^(2 s) is, with q = rint(. * 2^s),
//   sum_i ( m2_i + (2 q_guest,i - 4 q_y,i) m1_i + q_guest,i^2 - 4 q_y,i q_guest,i )
// where m1_i = q(u_host,i) and m2_i = m1_i^2 are the host's plaintexts. On ciphertexts:
//   out = prod_i c2_i  *  prod_i c1_i^(k_i)  *  E(P; r),
//   k_i = 2 q_guest,i - 4 q_y,i,   P = sum_i q_guest,i (q_guest,i - 4 q_y,i) mod n,
// i.e. one summation, one single-column X^T [[d]] with the k_i as exponents, one encryption.
#include "kernels_common.hpp"

using namespace haflo;
using namespace haflo::dev;

namespace {

constexpr int kLossBlocks = 1024;

// rint(v * 2^s) in binary64; false when undefined or at least 2^limit_bits in magnitude
__device__ __forceinline__ bool quantise_below(float v, int scale_bits, int limit_bits, long long& q) {
  double sc = __builtin_ldexp((double)v, scale_bits);
  double lim = __builtin_ldexp(1.0, limit_bits);
  if (!(sc > -lim && sc < lim)) {
    q = 0;
    return false;
  }
  q = (long long)__builtin_rint(sc);
  return q > -(1ll << limit_bits) && q < (1ll << limit_bits);
}

struct Wide {  // signed 128-bit integer as two's complement (lo, hi)
  unsigned long long lo;
  long long hi;
};
__device__ __forceinline__ void wide_add(Wide& a, long long v) {
  unsigned long long lo = a.lo + (unsigned long long)v;
  a.hi += (v < 0 ? -1ll : 0ll) + (lo < a.lo ? 1ll : 0ll);
  a.lo = lo;
}
__device__ __forceinline__ void wide_add(Wide& a, const Wide& b) {
  unsigned long long lo = a.lo + b.lo;
  a.hi += b.hi + (lo < a.lo ? 1ll : 0ll);
  a.lo = lo;
}

// k[i] = 2 q_guest - 4 q_y, partial[block] = sum over the block's elements of q_guest (q_guest - 4 q_y).
// Elements that are not finite or too large (|q_guest| >= 2^28, |q_y| >= 2^27) count as zero and set *status.
__global__ __launch_bounds__(kBlockThreads) void k_loss_terms(const float* __restrict__ u_guest,
                                                              const float* __restrict__ label, int scale_bits,
                                                              size_t count, int* __restrict__ k,
                                                              Wide* __restrict__ partial, u32* __restrict__ status) {
  __shared__ Wide red[kBlockThreads];
  Wide mine = {0ull, 0ll};
  bool bad = false;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < count; i += (size_t)gridDim.x * blockDim.x) {
    long long qg, qy;
    bool ok = quantise_below(u_guest[i], scale_bits, 28, qg);
    ok = quantise_below(label[i], scale_bits, 27, qy) && ok;
    if (!ok) {
      qg = 0;
      qy = 0;
      bad = true;
    }
    k[i] = (int)(2 * qg - 4 * qy);
    wide_add(mine, qg * (qg - 4 * qy));
  }
  red[threadIdx.x] = mine;
  __syncthreads();
  for (int step = kBlockThreads >> 1; step >= 1; step >>= 1) {
    if ((int)threadIdx.x < step) wide_add(red[threadIdx.x], red[threadIdx.x + step]);
    __syncthreads();
  }
  if (threadIdx.x == 0) partial[blockIdx.x] = red[0];
  if (status && __builtin_amdgcn_ballot_w64(bad) != 0ull && (threadIdx.x & (WAVE - 1)) == 0)
    atomicOr(status, HAFLO_ST_RANGE);
}

// plain[0..lp) = (sum of the partials) mod n, as 32-bit words (a negative sum S is n - |S|).
__global__ __launch_bounds__(WAVE) void k_loss_plain(const Wide* __restrict__ partial, int nparts,
                                                     const u32* __restrict__ nw, int lp, u32* __restrict__ plain) {
  if (threadIdx.x != 0 || blockIdx.x != 0) return;
  Wide s = {0ull, 0ll};
  for (int i = 0; i < nparts; ++i) wide_add(s, partial[i]);
  const bool neg = s.hi < 0;
  if (neg) {  // magnitude
    s.lo = ~s.lo + 1ull;
    s.hi = ~s.hi + (s.lo == 0ull ? 1ll : 0ll);
  }
  const u32 mag[4] = {(u32)s.lo, (u32)(s.lo >> 32), (u32)(unsigned long long)s.hi,
                      (u32)((unsigned long long)s.hi >> 32)};
  u32 borrow = 0;
  for (int j = 0; j < lp; ++j) {
    const u32 m = j < 4 ? mag[j] : 0u;
    if (!neg) {
      plain[j] = m;
    } else {
      const unsigned long long d = (unsigned long long)nw[j] - m - borrow;
      plain[j] = (u32)d;
      borrow = (u32)(d >> 63);
    }
  }
}

size_t align256(size_t b) { return (b + 255) & ~(size_t)255; }

struct LossPlan {
  size_t off_k, off_partial, off_plain, off_t1, off_t2, off_t3, off_ws, ws_bytes, total;
};
LossPlan loss_plan(const haflo_ctx* ctx, size_t count) {
  LossPlan p;
  const size_t cipher = align256((size_t)ctx->N.nl * 4);
  size_t b = 0;
  p.off_k = b;        b += align256(count * 4);
  p.off_partial = b;  b += align256((size_t)kLossBlocks * sizeof(Wide));
  p.off_plain = b;    b += align256((size_t)ctx->lp * 4);
  p.off_t1 = b;       b += cipher;
  p.off_t2 = b;       b += cipher;
  p.off_t3 = b;       b += cipher;
  p.off_ws = b;
  size_t w = haflo_workspace_bytes(ctx, HAFLO_OP_MATVEC_XT_D, count, 1);
  size_t e = haflo_workspace_bytes(ctx, HAFLO_OP_ENCRYPT, 1, 0);
  if (e > w) w = e;
  e = haflo_workspace_bytes(ctx, HAFLO_OP_ENCRYPT_OBFUSCATOR, 1, 0);
  if (e > w) w = e;
  p.ws_bytes = w;
  p.total = b + w;
  return p;
}

}  // namespace

namespace haflo {
size_t ws_taylor_loss(const haflo_ctx* ctx, size_t count) { return loss_plan(ctx, count).total; }
}  // namespace haflo

extern "C" {

int haflo_taylor_loss(const haflo_ctx* ctx, const void* d_c_u, const void* d_c_u2, const float* d_u_guest,
                      const float* d_label, const uint32_t* d_r, uint32_t scale_bits, void* d_out,
                      uint32_t* d_status, size_t count, void* d_workspace, size_t workspace_bytes, void* stream) {
  if (!ctx || scale_bits > 27 || !d_out || (count && (!d_c_u || !d_c_u2 || !d_u_guest || !d_label)))
    return HAFLO_EINVAL;
  if (count > 0xFFFFFFFFull) return HAFLO_EINVAL;
  const LossPlan p = loss_plan(ctx, count);
  if (!d_workspace || workspace_bytes < p.total) return HAFLO_EINVAL;
  hipStream_t st = (hipStream_t)stream;
  char* base = (char*)d_workspace;
  int* k = (int*)(base + p.off_k);
  Wide* partial = (Wide*)(base + p.off_partial);
  uint32_t* plain = (uint32_t*)(base + p.off_plain);
  void* t1 = base + p.off_t1;
  void* t2 = base + p.off_t2;
  void* t3 = base + p.off_t3;
  void* ws = base + p.off_ws;
  LaunchShape sh;
  sh.threads = kBlockThreads;
  sh.gpb = kBlockThreads;
  size_t need = (count + kBlockThreads - 1) / kBlockThreads;
  sh.blocks = (int)(need < 1 ? 1 : (need < (size_t)kLossBlocks ? need : (size_t)kLossBlocks));
  HAFLO_LAUNCH(k_loss_terms, sh, st, d_u_guest, d_label, (int)scale_bits, count, k, partial, d_status);
  LaunchShape one;
  one.blocks = 1;
  one.threads = WAVE;
  one.gpb = WAVE;
  HAFLO_LAUNCH(k_loss_plain, one, st, (const Wide*)partial, sh.blocks, (const u32*)ctx->d_n_words, ctx->lp, plain);
  int rc = haflo_cipher_matvec(ctx, 0, d_c_u, k, count, 1, t1, ws, p.ws_bytes, stream);
  if (rc != HAFLO_OK) return rc;
  rc = haflo_cipher_sum(ctx, d_c_u2, count, t2, ws, p.ws_bytes, stream);
  if (rc != HAFLO_OK) return rc;
  // without an r the plaintext part enters as g^P = 1 + P n (obfuscator 1): two products instead of a
  // full exponentiation; the result is still randomised by the host's ciphertexts
  rc = d_r ? haflo_encrypt(ctx, plain, d_r, t3, 1, ws, p.ws_bytes, stream)
           : haflo_encrypt_with_obfuscator(ctx, plain, ctx->N.ref().r1, t3, 1, ws, p.ws_bytes, stream);
  if (rc != HAFLO_OK) return rc;
  rc = haflo_add(ctx, t1, t2, t1, 1, stream);
  if (rc != HAFLO_OK) return rc;
  return haflo_add(ctx, t1, t3, d_out, 1, stream);
}

}  // extern "C"
