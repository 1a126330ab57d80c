// Internal declarations shared by the translation units of libhaflo: the key
// context, per-modulus constant tables, exponent schedules and launch helpers.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <vector>

#include "../../include/haflo.h"
#include "hostbig.hpp"

namespace haflo {

constexpr int kLimbBits = 29;
constexpr int kBlockThreads = 256;

// Device view of one odd modulus in radix 2^29 with NL limbs. All pointers are
// device memory owned by the context; every table has NL limbs.
struct ModRef {
  const uint32_t* n;   // the modulus
  const uint32_t* r1;  // R mod n, R = 2^(29*NL): the Montgomery form of 1
  const uint32_t* r2;  // R^2 mod n
  const uint32_t* r3;  // R^3 mod n
  uint32_t n0inv;      // -n^-1 mod 2^29
  int nl;              // limbs
};

// Sliding-window exponentiation plan for one fixed exponent, shared by every
// element of a batch. The table holds the odd powers x^1, x^3, ...,
// x^(2*table_len-1). Execution: acc = table[first]; then for each step square
// `nsq` times and, unless idx == kNoMul, multiply by table[idx].
constexpr uint32_t kNoMul = 0xFFFFu;
struct SchedRef {
  const uint32_t* steps;  // device: (nsq << 16) | idx
  int nsteps;
  int first;      // table index of the leading window
  int table_len;  // entries to precompute (>= 1)
  int is_zero;    // exponent == 0: result is 1
};

struct HostSched {
  std::vector<uint32_t> steps;
  int first = 0;
  int table_len = 1;
  int is_zero = 0;
  uint64_t nsquare = 0, nmul = 0;  // Montgomery products the plan executes (table build included)
};
HostSched make_schedule(const Big& e, int window);

struct ModHost {
  Big mod;
  int nl = 0;   // 29-bit limbs
  int lpt = 0;  // limbs per lane
  int t = 0;    // lanes per big integer
  uint32_t n0inv = 0;
  uint32_t* d_tab = nullptr;  // device: n | r1 | r2 | r3, nl limbs each
  ModRef ref() const {
    ModRef r;
    r.n = d_tab;
    r.r1 = d_tab + nl;
    r.r2 = d_tab + 2 * nl;
    r.r3 = d_tab + 3 * nl;
    r.n0inv = n0inv;
    r.nl = nl;
    return r;
  }
};

struct DevSched {
  HostSched h;
  uint32_t* d_steps = nullptr;
  SchedRef ref() const {
    SchedRef r;
    r.steps = d_steps;
    r.nsteps = (int)h.steps.size();
    r.first = h.first;
    r.table_len = h.table_len;
    r.is_zero = h.is_zero;
    return r;
  }
};

}  // namespace haflo

struct haflo_ctx {
  uint32_t n_bits = 0;
  bool has_priv = false;
  int lc = 0, lp = 0;  // canonical 32-bit limbs of a ciphertext / plaintext
  int num_cu = 0;
  haflo::Big n, nsq, p, q;
  haflo::ModHost N;            // n^2
  haflo::ModHost P2, Q2;       // p^2, q^2 (private)
  haflo::ModHost P, Q;         // p, q (private)
  haflo::DevSched sched_n;     // exponent n modulo n^2 (encryption)
  haflo::DevSched sched_pm1;   // exponent p-1 modulo p^2
  haflo::DevSched sched_qm1;   // exponent q-1 modulo q^2
  // device constants
  uint32_t* d_k1 = nullptr;      // n * R^2 mod n^2 (N.nl limbs): montmul(m, k1) = m*n*R
  uint32_t* d_n_words = nullptr; // n as lp 32-bit words
  uint32_t* d_halfn_words = nullptr;  // floor(n/2) as lp words
  uint32_t* d_priv = nullptr;    // private-key tables, see ctx.cpp
  // offsets (in limbs) into d_priv, each P.nl limbs
  const uint32_t* d_pinv = nullptr;    // p^-1 mod 2^(29*P.nl)
  const uint32_t* d_qinv = nullptr;
  const uint32_t* d_hp = nullptr;      // h_p * R_p mod p
  const uint32_t* d_hq = nullptr;
  const uint32_t* d_pinvq = nullptr;   // (p^-1 mod q) * R_q mod q
  std::vector<void*> dev_allocs;
};

namespace haflo {

// Launch shape for a grid-stride kernel over `groups` lane groups of `t` lanes:
// 256-lane blocks capped at blocks_per_cu per compute unit; a batch too small
// to give every compute unit four wavefronts uses single-wavefront blocks so
// that it still spreads over the chip.
struct LaunchShape {
  int blocks;
  int threads;
  int gpb;  // groups per block
  size_t slots() const { return (size_t)blocks * gpb; }
};
inline LaunchShape launch_shape(const haflo_ctx* ctx, size_t groups, int t, int blocks_per_cu) {
  LaunchShape s;
  size_t small_limit = (size_t)ctx->num_cu * 4 * (64 / t);
  s.threads = (groups <= small_limit) ? 64 : kBlockThreads;
  s.gpb = s.threads / t;
  size_t need = (groups + s.gpb - 1) / s.gpb;
  size_t cap = (size_t)ctx->num_cu * blocks_per_cu * (kBlockThreads / s.threads);
  if (need < 1) need = 1;
  s.blocks = (int)(need < cap ? need : cap);
  return s;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? HAFLO_OK : HAFLO_EHIP; }

// 29-bit limbs of a host integer
std::vector<uint32_t> to_limbs29(const Big& x, int nl);

// workspace sizes in bytes (kernels_modexp.hip)
size_t ws_encrypt(const haflo_ctx* ctx, size_t count);
size_t ws_scalar_mul(const haflo_ctx* ctx, size_t count);
size_t ws_decrypt(const haflo_ctx* ctx, size_t count);

// out[i] = in[i]^-1 mod n^2 on internal ciphertexts; out may alias in (kernels_matvec.hip)
int invert_batch(const haflo_ctx* ctx, const uint32_t* in, uint32_t* out, size_t count, hipStream_t st);

}  // namespace haflo
