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
  const uint32_t* one; // the integer 1
  uint32_t n0inv;      // -n^-1 mod 2^29
  int nl;              // limbs
};

// Sliding-window exponentiation plan for one fixed exponent, shared by every
// element of a batch. The table holds the odd powers x^1, x^3, ...,
// x^(2*table_len-1). Execution: acc = table[first]; then for each step square
// `nsq` times and, unless idx == kNoMul, multiply by table[idx].
constexpr uint32_t kNoMul = 0xFFFFu;
struct HostSched {
  std::vector<uint32_t> steps;  // (nsq << 16) | idx
  int first = 0;
  int table_len = 1;
  int is_zero = 0;
  uint64_t nsquare = 0, nmul = 0;  // Montgomery products the plan executes (table build included)
};
HostSched make_schedule(const Big& e, int window);

// The exponentiation kernels run a small batch-uniform program, one
// instruction per Montgomery product or register/table move, so that the whole
// operator goes through a single unrolled product loop. An instruction is
// op | a << 8 | b << 20. `acc` is the running value (lazy Montgomery form),
// table[] the group's scratch slots of NL limbs, constant[] per-modulus limb
// arrays (kConst*), k the element's own 64-bit exponent where one is given.
enum EngOp : uint32_t {
  ENG_SQ = 0,        // acc = acc * acc
  ENG_MUL_T = 1,     // acc = acc * table[a]
  ENG_MUL_T_ST = 2,  // acc = acc * table[a]; table[b] = acc
  ENG_MUL_C = 3,     // acc = acc * constant[a]
  ENG_MUL_TD = 4,    // acc = acc * table[(k >> a) & 15]
  // no product below this line
  ENG_LOAD_T = 8,    // acc = table[a]
  ENG_STORE_T = 9,   // table[a] = acc
  ENG_LOAD_C = 10,   // acc = constant[a]
  ENG_ADD_C = 11,    // acc += constant[a]  (lazy, limbs renormalised)
  ENG_ADD_T = 12,    // acc += table[a]
  ENG_LOAD_W = 13,   // acc = the element's 32-bit-word input a (0 or 1), cut into limbs
  ENG_LOAD_L = 14,   // acc = limbs [a*NL, (a+1)*NL) of the element's limb input
  ENG_LOAD_TD = 15,  // acc = table[(k >> a) & 15]
  ENG_LOAD_WH = 16,  // acc = limbs [NL, 2 NL) of the element's 32-bit-word input a: the part above ENG_LOAD_W's
  ENG_LOAD_W1 = 17   // pair engine only: acc = 1 + n w for the element's 32-bit-word input a
};
enum { kConstR1 = 0, kConstR2 = 1, kConstR3 = 2, kConstOne = 3, kConstExtra = 4, kConstR4 = 5, kConstR5 = 6, kNumConst = 7 };
inline uint32_t eng_ins(uint32_t op, uint32_t a = 0, uint32_t b = 0) { return op | (a << 8) | (b << 20); }

// acc = acc^e for the plan `h`, using table slots [0, h.table_len] (the last one as scratch)
void append_modexp(std::vector<uint32_t>& prog, const HostSched& h);
// table[d] = x^d for d < entries from acc = x (leaves acc = 1 in Montgomery form)
void append_power_table(std::vector<uint32_t>& prog, int entries);

struct DevProg {
  std::vector<uint32_t> host;
  uint32_t* d_ins = nullptr;
  int table_entries = 1;  // table slots the program touches
  HostSched sched;        // the exponent plan inside it, for cost accounting
};

struct ModHost {
  Big mod;
  int nl = 0;   // 29-bit limbs
  int lpt = 0;  // limbs per lane
  int t = 0;    // lanes per big integer
  uint32_t n0inv = 0;
  uint32_t* d_tab = nullptr;  // device: n | r1 | r2 | r3 | one, nl limbs each
  // Pair arithmetic modulo mod^2 (residues x0 + mod x1, see pairmul_core): kNumConst constants of 2 nl limbs
  // each, [x0 | x1], indexed by kConst*: R, R^2, R^3, 1, an operator-specific one, R^4, R^5, all modulo
  // mod^2 with R = 2^(29 nl). Null where the modulus is not used that way.
  uint32_t* d_pairs = nullptr;
  ModRef ref() const {
    ModRef r;
    r.n = d_tab;
    r.r1 = d_tab + nl;
    r.r2 = d_tab + 2 * nl;
    r.r3 = d_tab + 3 * nl;
    r.one = d_tab + 4 * nl;
    r.n0inv = n0inv;
    r.nl = nl;
    return r;
  }
};

}  // namespace haflo

struct haflo_ctx {
  uint32_t n_bits = 0;
  bool has_priv = false;
  int lc = 0, lp = 0;  // canonical 32-bit limbs of a ciphertext / plaintext
  int num_cu = 0;
  int device = -1;  // the HIP device that was current when the context was created
  size_t xtd_bucket_min_rows = HAFLO_XTD_BUCKET_MIN_ROWS_DEFAULT;  // X^T [[d]]: bucket method from this many rows on
  haflo::Big n, nsq, p, q;
  haflo::ModHost N;            // n^2
  haflo::ModHost Nw;           // n, at the limb count (and Montgomery radix) of n^2
  haflo::ModHost P2, Q2;       // p^2, q^2 (private)
  haflo::ModHost P, Q;         // p, q (private)
  // n at half the limbs of n^2: the modulus of the pair arithmetic modulo n^2. Its operator-specific pair
  // constants: [kConstExtra] R R_N, [kConstR3] R_N, [kConstR4] R^2 / R_N, [kConstR5] R^3 / R_N (R_N = 2^(29 N.nl),
  // the radix of the stored ciphertexts): out of and into the pair form
  haflo::ModHost Nh;
  haflo::DevProg prog_enc_pairs;   // encryption with the public key on pairs modulo n
  haflo::DevProg prog_dec_pairs_p, prog_dec_pairs_q;    // decryption branches on pairs modulo p, q
  haflo::DevProg prog_lift_pairs_p, prog_lift_pairs_q;  // key owner's encryption, second stage, on pairs modulo p, q
  haflo::DevProg prog_enc;     // encryption: r^n modulo n^2 and the (1 + m n) factor
  haflo::DevProg prog_dec_p;   // decryption branch: c^(p-1) modulo p^2
  haflo::DevProg prog_dec_q;   // decryption branch: c^(q-1) modulo q^2
  haflo::DevProg prog_enc_p;   // key owner's encryption, first stage: r^(n mod (p-1)) modulo p
  haflo::DevProg prog_enc_q;   //   and r^(n mod (q-1)) modulo q
  haflo::DevProg prog_lift_p;  // second stage: y^p modulo p^2
  haflo::DevProg prog_lift_q;  //   and y^q modulo q^2
  uint32_t* d_p2inv = nullptr; // ((p^2)^-1 mod q^2) * R mod q^2 (P2.nl limbs)
  // device constants
  uint32_t* d_k1 = nullptr;      // n * R^2 mod n^2 (N.nl limbs): montmul(m, k1) = m*n*R
  uint32_t* d_n_words = nullptr; // n as lp 32-bit words
  uint32_t* d_nb_words = nullptr;  // n - 2^64 as lp words
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
enum { kGeoPlain = 0, kGeoWide = 1, kGeoWave = 2 };  // lanes per big integer: as the modulus says, twice that, a wavefront
struct LaunchShape {
  int blocks;
  int threads;
  int gpb;  // groups per block
  int geo = kGeoPlain;
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

// device address of the static scratch array on the current device (kernels_modexp.hip)
int static_scratch_init();

// workspace sizes in bytes (kernels_modexp.hip)
size_t ws_encrypt(const haflo_ctx* ctx, size_t count);
size_t ws_scalar_mul(const haflo_ctx* ctx, size_t count);
size_t ws_encrypt_obf(const haflo_ctx* ctx, size_t count);
size_t ws_decrypt(const haflo_ctx* ctx, size_t count);
// workspace of the Taylor-loss sequence in bytes (kernels_loss.hip)
size_t ws_taylor_loss(const haflo_ctx* ctx, size_t count);

// tables[i][d] = c_i^d for d < entries (kernels_modexp.hip)
int power_tables(const haflo_ctx* ctx, const uint32_t* d_c, uint32_t* d_tables, int entries, size_t count,
                 hipStream_t st);

// out[i] = in[i]^-1 mod n^2 on internal ciphertexts; out may alias in (kernels_matvec.hip)
int invert_batch(const haflo_ctx* ctx, const uint32_t* in, uint32_t* out, size_t count, hipStream_t st);

// X^T [[d]] by the bucket method (kernels_buckets.hip). Workspace layout in 32-bit words.
struct XtdBucketPlan {
  int rounds;
  int chunk_bits;  // a reduction round multiplies chunks of at most 2^chunk_bits items
  size_t keys, scan_blocks;
  size_t off_cnt, off_totals, off_offs, off_sorted, off_arena[2], off_G, off_AT, off_R, off_pairs, off_order, total;
  bool pairs;  // the products run on pairs of residues modulo n
};
bool xtd_buckets_fit(size_t rows, size_t cols);
XtdBucketPlan xtd_bucket_plan(const haflo_ctx* ctx, size_t rows, size_t cols);
// d_P[j][sign] = product of c_i^|x_ij| over the entries of column j with that sign (lazy Montgomery form).
// ws: xtd_bucket_plan(...).total words.
int xtd_buckets(const haflo_ctx* ctx, const uint32_t* d_c, const int32_t* d_X, size_t rows, size_t cols,
                uint32_t* ws, uint32_t* d_P, hipStream_t st);

// Segmented summation through the bucket reduction rounds (kernels_buckets.hip). Workspace layout in 32-bit words.
struct SegSumPlan {
  int rounds;
  int chunk_bits;
  size_t scan_blocks, off_cnt, off_totals, off_offs, off_arena[2], total;
};
SegSumPlan seg_sum_plan(const haflo_ctx* ctx, size_t count, size_t nseg);
// d_out[k] = product of d_c[offsets[k] .. offsets[k+1]) (canonical internal elements); ws: seg_sum_plan(...).total words
int seg_sum(const haflo_ctx* ctx, const uint32_t* d_c, const uint32_t* d_offsets, size_t count, size_t nseg,
            uint32_t* d_out, uint32_t* d_status, uint32_t* ws, hipStream_t st);

}  // namespace haflo
