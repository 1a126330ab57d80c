// Host side of libhaflo: deterministic key generation, key contexts and the
// per-key constant tables the kernels read (Montgomery constants in radix
// 2^29, exponent schedules, constants of decryption through p^2 and q^2).
#include <cstdio>
#include <cstdlib>
#include <new>

#include "haflo_internal.hpp"

namespace haflo {

std::vector<uint32_t> to_limbs29(const Big& x, int nl) {
  std::vector<uint32_t> r(nl, 0);
  for (int i = 0; i < nl; ++i) r[i] = x.extract((size_t)i * kLimbBits, kLimbBits);
  return r;
}

// Sliding-window plan for a fixed exponent (left to right, odd-power table).
static HostSched plan_with_window(const Big& e, int w) {
  HostSched s;
  if (e.is_zero()) {
    s.is_zero = 1;
    return s;
  }
  long i = (long)e.bits() - 1;
  auto take_window = [&](long hi, long& lo_out) -> uint32_t {
    long lo = hi - w + 1;
    if (lo < 0) lo = 0;
    while (!e.bit((size_t)lo)) ++lo;
    lo_out = lo;
    return e.extract((size_t)lo, (unsigned)(hi - lo + 1));
  };
  long lo;
  uint32_t v = take_window(i, lo);
  s.first = (int)((v - 1) / 2);
  int max_idx = s.first;
  // bits below the leading window that it skipped over (trailing zeros of the
  // window were excluded, so none) - continue below `lo`
  i = lo - 1;
  uint32_t pending = 0;
  while (i >= 0) {
    if (!e.bit((size_t)i)) {
      ++pending;
      --i;
      continue;
    }
    v = take_window(i, lo);
    uint32_t nsq = pending + (uint32_t)(i - lo + 1);
    int idx = (int)((v - 1) / 2);
    if (idx > max_idx) max_idx = idx;
    s.steps.push_back((nsq << 16) | (uint32_t)idx);
    s.nsquare += nsq;
    s.nmul += 1;
    pending = 0;
    i = lo - 1;
  }
  if (pending) {
    s.steps.push_back((pending << 16) | kNoMul);
    s.nsquare += pending;
  }
  s.table_len = max_idx + 1;
  if (s.table_len > 1) {
    s.nsquare += 1;                 // x^2
    s.nmul += s.table_len - 1;      // x^3, x^5, ...
  }
  return s;
}

HostSched make_schedule(const Big& e, int window) {
  if (window > 0) return plan_with_window(e, window);
  HostSched best = plan_with_window(e, 1);
  for (int w = 2; w <= 7; ++w) {
    HostSched c = plan_with_window(e, w);
    if (c.nsquare + c.nmul < best.nsquare + best.nmul) best = c;
  }
  return best;
}

void append_modexp(std::vector<uint32_t>& prog, const HostSched& h) {
  if (h.is_zero) {
    prog.push_back(eng_ins(ENG_LOAD_C, kConstR1));
    return;
  }
  const uint32_t tmp = (uint32_t)h.table_len;
  prog.push_back(eng_ins(ENG_STORE_T, 0));
  if (h.table_len > 1) {
    prog.push_back(eng_ins(ENG_SQ));
    prog.push_back(eng_ins(ENG_STORE_T, tmp));
    prog.push_back(eng_ins(ENG_LOAD_T, 0));
    for (int i = 1; i < h.table_len; ++i) prog.push_back(eng_ins(ENG_MUL_T_ST, tmp, (uint32_t)i));
  }
  prog.push_back(eng_ins(ENG_LOAD_T, (uint32_t)h.first));
  for (uint32_t st : h.steps) {
    for (uint32_t i = 0; i < (st >> 16); ++i) prog.push_back(eng_ins(ENG_SQ));
    if ((st & 0xFFFFu) != kNoMul) prog.push_back(eng_ins(ENG_MUL_T, st & 0xFFFFu));
  }
}

void append_power_table(std::vector<uint32_t>& prog, int entries) {
  prog.push_back(eng_ins(ENG_STORE_T, 1));
  for (uint32_t d = 2; d < (uint32_t)entries; ++d) prog.push_back(eng_ins(ENG_MUL_T_ST, 1, d));
  prog.push_back(eng_ins(ENG_LOAD_C, kConstR1));
  prog.push_back(eng_ins(ENG_STORE_T, 0));
}

static const std::vector<uint32_t>& small_primes() {
  static std::vector<uint32_t> pr;
  if (pr.empty()) {
    for (uint32_t c = 2; c < 2000; ++c) {
      bool ok = true;
      for (uint32_t d = 2; d * d <= c; ++d)
        if (c % d == 0) {
          ok = false;
          break;
        }
      if (ok) pr.push_back(c);
    }
  }
  return pr;
}

// one strong-probable-prime round of odd cand to `base`
static bool mr_round(const MontHost& mh, const Big& cand, const Big& cm1, const Big& d, size_t s, const Big& base) {
  Big x = mh.powmod(base, d);
  if (x == Big(1) || x == cm1) return true;
  for (size_t i = 1; i < s; ++i) {
    x = mh.from_mont(mh.mul(mh.to_mont(x), mh.to_mont(x)));
    if (x == cm1) return true;
  }
  (void)cand;
  return false;
}

static Big next_prime_from_stream(SplitMix64& rng, size_t half_bits) {
  size_t nwords = half_bits / 64;
  for (;;) {
    Big cand = rng.words(nwords);
    cand.w.resize(half_bits / 32, 0);
    cand.w[half_bits / 32 - 1] |= 0xC0000000u;
    cand.w[0] |= 1u;
    cand.trim();
    bool divisible = false;
    for (uint32_t sp : small_primes())
      if (cand.mod_small(sp) == 0) {
        divisible = true;
        break;
      }
    if (divisible) continue;
    MontHost mh(cand);
    Big cm1 = Big::sub(cand, Big(1));
    Big d = cm1;
    size_t s = 0;
    while (!d.is_odd()) {
      d = d.shr1();
      ++s;
    }
    Big cm3 = Big::sub(cand, Big(3));
    bool ok = true;
    for (int round = 0; round < 40; ++round) {
      Big base = rng.words(nwords);
      // base < 2^half_bits < 2*(cand-3): one conditional subtraction reduces it
      if (base >= cm3) base = Big::sub(base, cm3);
      base = Big::add(base, Big(2));
      if (!mr_round(mh, cand, cm1, d, s, base)) {
        ok = false;
        break;
      }
    }
    if (ok) return cand;
  }
}

static bool valid_bits(uint32_t n_bits) { return n_bits == 512 || n_bits == 1024 || n_bits == 2048 || n_bits == 4096; }

static bool choose_geometry(ModHost& m) {
  if (m.nl % 18 == 0) {
    m.lpt = 18;
    m.t = m.nl / 18;
  } else if (m.nl == 9) {
    m.lpt = 9;
    m.t = 1;
  } else {
    return false;
  }
  return m.t == 1 || m.t == 2 || m.t == 4 || m.t == 8 || m.t == 16;
}

struct Uploader {
  haflo_ctx* ctx;
  bool ok = true;
  uint32_t* put(const std::vector<uint32_t>& v) {
    if (!ok) return nullptr;
    void* d = nullptr;
    size_t bytes = v.size() * sizeof(uint32_t);
    if (bytes == 0) bytes = 4;
    if (hipMalloc(&d, bytes) != hipSuccess) {
      ok = false;
      return nullptr;
    }
    ctx->dev_allocs.push_back(d);
    if (!v.empty() && hipMemcpy(d, v.data(), v.size() * sizeof(uint32_t), hipMemcpyHostToDevice) != hipSuccess) {
      ok = false;
      return nullptr;
    }
    return (uint32_t*)d;
  }
};

static void build_modulus(ModHost& m, const Big& mod, int nl, Uploader& up) {
  m.mod = mod;
  m.nl = nl;
  if (!choose_geometry(m)) {
    up.ok = false;
    return;
  }
  m.n0inv = neg_inv32(mod.w[0]) & ((1u << kLimbBits) - 1u);
  Big r1 = Big::mod(Big::pow2((size_t)kLimbBits * nl), mod);
  Big r2 = Big::mod(Big::mul(r1, r1), mod);
  Big r3 = Big::mod(Big::mul(r2, r1), mod);
  Big one(1);
  std::vector<uint32_t> tab;
  for (const Big* b : {(const Big*)&mod, (const Big*)&r1, (const Big*)&r2, (const Big*)&r3, (const Big*)&one}) {
    std::vector<uint32_t> l = to_limbs29(*b, nl);
    tab.insert(tab.end(), l.begin(), l.end());
  }
  m.d_tab = up.put(tab);
}

// encryption: acc = r (word input 1) -> r R -> (r R)^n -> times ((m n) R + R), m = word input 0
static void build_prog_encrypt(DevProg& p, const Big& n, Uploader& up) {
  p.sched = make_schedule(n, 0);
  p.host.clear();
  p.host.push_back(eng_ins(ENG_LOAD_W, 1));
  p.host.push_back(eng_ins(ENG_MUL_C, kConstR2));
  append_modexp(p.host, p.sched);
  p.host.push_back(eng_ins(ENG_STORE_T, 0));
  p.host.push_back(eng_ins(ENG_LOAD_W, 0));
  p.host.push_back(eng_ins(ENG_MUL_C, kConstExtra));  // montmul(m, n R^2) = m n R
  p.host.push_back(eng_ins(ENG_ADD_C, kConstR1));
  p.host.push_back(eng_ins(ENG_MUL_T, 0));
  p.table_entries = p.sched.table_len + 1;
  p.d_ins = up.put(p.host);
}

// The same on pairs of residues modulo n (engine_run_pairs): r -> r R -> (r R)^n = r^n R -> times (1 + m n)
// (the pair (1, m)) = the ciphertext -> times R 2^(29 N.nl): its Montgomery form modulo n^2 at the radix of
// the other operators. Constants: [0] R, [1] R^2, [4] R 2^(29 N.nl), all modulo n^2 and as pairs.
static void build_prog_encrypt_pairs(DevProg& p, const HostSched& sched, Uploader& up) {
  p.sched = sched;
  p.host.clear();
  p.host.push_back(eng_ins(ENG_LOAD_W, 1));
  p.host.push_back(eng_ins(ENG_MUL_C, kConstR2));
  append_modexp(p.host, p.sched);
  p.host.push_back(eng_ins(ENG_STORE_T, 0));
  p.host.push_back(eng_ins(ENG_LOAD_W1, 0));
  p.host.push_back(eng_ins(ENG_MUL_T, 0));
  p.host.push_back(eng_ins(ENG_MUL_C, kConstExtra));
  p.table_entries = p.sched.table_len + 1;
  p.d_ins = up.put(p.host);
}

// x < s^2 as the pair (x mod s, x div s), nl limbs each
static std::vector<uint32_t> pair_limbs(const Big& x, const Big& n, int nl) {
  const Big lo = Big::mod(x, n);
  const Big hi = Big::div(x, n);
  std::vector<uint32_t> v = to_limbs29(lo, nl), h = to_limbs29(hi, nl);
  v.insert(v.end(), h.begin(), h.end());
  return v;
}

// The constants of the pair arithmetic modulo s^2 for the modulus `ms` = s (ModHost::d_pairs): R .. R^5 and 1
// in their slots; `special` replaces the slots it names (operator-specific constants).
static void build_pair_consts(ModHost& ms, const Big& s, const Big& s2,
                              const std::vector<std::pair<int, Big>>& special, Uploader& up) {
  std::vector<Big> c(kNumConst);
  c[kConstR1] = Big::mod(Big::pow2((size_t)kLimbBits * ms.nl), s2);
  c[kConstR2] = Big::mod(Big::mul(c[kConstR1], c[kConstR1]), s2);
  c[kConstR3] = Big::mod(Big::mul(c[kConstR2], c[kConstR1]), s2);
  c[kConstR4] = Big::mod(Big::mul(c[kConstR3], c[kConstR1]), s2);
  c[kConstR5] = Big::mod(Big::mul(c[kConstR4], c[kConstR1]), s2);
  c[kConstOne] = Big(1);
  c[kConstExtra] = Big(1);
  for (const std::pair<int, Big>& sp : special) c[sp.first] = sp.second;
  std::vector<uint32_t> tab;
  for (const Big& b : c) {
    std::vector<uint32_t> l = pair_limbs(b, s, ms.nl);
    tab.insert(tab.end(), l.begin(), l.end());
  }
  ms.d_pairs = up.put(tab);
}

// Decryption branch for a prime s on pairs modulo s: the canonical residue c modulo n^2 in four quarters,
// c = c_0 + c_1 R + c_2 R^2 + c_3 R^3 (R = 2^(29 nl(s))), goes to the pair form of c R modulo s^2 as the sum
// of the products of (c_k, 0) with R^(k+2), is raised to s - 1 and leaves the Montgomery domain. The result
// is 1 + s L with L the quotient the decryption needs: the engine stores the second half of the pair.
static void build_prog_decrypt_pairs(DevProg& p, const HostSched& sched, Uploader& up) {
  p.sched = sched;
  p.host.clear();
  const uint32_t power[4] = {kConstR2, kConstR3, kConstR4, kConstR5};
  for (uint32_t k = 0; k < 4; ++k) {
    p.host.push_back(eng_ins(ENG_LOAD_L, k));
    p.host.push_back(eng_ins(ENG_MUL_C, power[k]));
    if (k) p.host.push_back(eng_ins(ENG_ADD_T, 0));
    if (k < 3) p.host.push_back(eng_ins(ENG_STORE_T, 0));
  }
  append_modexp(p.host, p.sched);
  p.host.push_back(eng_ins(ENG_MUL_C, kConstOne));
  p.table_entries = p.sched.table_len + 1;
  p.d_ins = up.put(p.host);
}
// Key owner's encryption, second stage, on pairs modulo s: y (limb input, below s) to the power s modulo s^2
static void build_prog_lift_pairs(DevProg& p, const HostSched& sched, Uploader& up) {
  p.sched = sched;
  p.host.clear();
  p.host.push_back(eng_ins(ENG_LOAD_L, 0));
  p.host.push_back(eng_ins(ENG_MUL_C, kConstR2));
  append_modexp(p.host, p.sched);
  p.host.push_back(eng_ins(ENG_MUL_C, kConstOne));
  p.table_entries = p.sched.table_len + 1;
  p.d_ins = up.put(p.host);
}

// Key owner's encryption, one prime-power branch in two stages. With n = s t (s, t the primes,
// gcd(t, s - 1) = 1) the n-th powers modulo s^2 are the subgroup of order s - 1, whose elements are
// determined by their residues modulo s: the one that is a modulo s is a^s mod s^2. Hence
//   r^n mod s^2 = (r^(n mod (s-1)) mod s)^s mod s^2:
// a half-length exponent on the quarter-size modulus s, then a half-length exponent on s^2, instead
// of a full-length exponent on s^2.
// Stage 1: r (word input 1, below n) = r_hi R + r_lo goes to Montgomery form modulo s as
// montmul(r_lo, R^2) + montmul(r_hi, R^3), is raised to e = n mod (s - 1) and leaves the Montgomery
// domain.
static void build_prog_encrypt_low(DevProg& p, const Big& e, Uploader& up) {
  p.sched = make_schedule(e, 0);
  p.host.clear();
  p.host.push_back(eng_ins(ENG_LOAD_WH, 1));
  p.host.push_back(eng_ins(ENG_MUL_C, kConstR3));
  p.host.push_back(eng_ins(ENG_STORE_T, 0));
  p.host.push_back(eng_ins(ENG_LOAD_W, 1));
  p.host.push_back(eng_ins(ENG_MUL_C, kConstR2));
  p.host.push_back(eng_ins(ENG_ADD_T, 0));
  append_modexp(p.host, p.sched);
  p.host.push_back(eng_ins(ENG_MUL_C, kConstOne));
  p.table_entries = p.sched.table_len + 1;
  p.d_ins = up.put(p.host);
}
// Stage 2: y (limb input, the canonical result of stage 1, zero-extended) to the power s modulo s^2;
// the result leaves the Montgomery domain.
static void build_prog_encrypt_lift(DevProg& p, const Big& s, Uploader& up) {
  p.sched = make_schedule(s, 0);
  p.host.clear();
  p.host.push_back(eng_ins(ENG_LOAD_L, 0));
  p.host.push_back(eng_ins(ENG_MUL_C, kConstR2));
  append_modexp(p.host, p.sched);
  p.host.push_back(eng_ins(ENG_MUL_C, kConstOne));
  p.table_entries = p.sched.table_len + 1;
  p.d_ins = up.put(p.host);
}

// decryption branch for a prime s: the canonical residue c = c_hi R + c_lo (two halves of the
// limb input) goes to Montgomery form mod s^2 as montmul(c_lo, R^2) + montmul(c_hi, R^3),
// is raised to s - 1 and leaves the Montgomery domain
static void build_prog_decrypt(DevProg& p, const Big& e, Uploader& up) {
  p.sched = make_schedule(e, 0);
  p.host.clear();
  p.host.push_back(eng_ins(ENG_LOAD_L, 0));
  p.host.push_back(eng_ins(ENG_MUL_C, kConstR2));
  p.host.push_back(eng_ins(ENG_STORE_T, 0));
  p.host.push_back(eng_ins(ENG_LOAD_L, 1));
  p.host.push_back(eng_ins(ENG_MUL_C, kConstR3));
  p.host.push_back(eng_ins(ENG_ADD_T, 0));
  append_modexp(p.host, p.sched);
  p.host.push_back(eng_ins(ENG_MUL_C, kConstOne));
  p.table_entries = p.sched.table_len + 1;
  p.d_ins = up.put(p.host);
}

static std::vector<uint32_t> to_words(const Big& x, int nw) {
  std::vector<uint32_t> r(nw, 0);
  for (int i = 0; i < nw; ++i) r[i] = x.word(i);
  return r;
}

static int ctx_build(haflo_ctx* ctx, const Big& n, const Big* p, const Big* q, uint32_t n_bits) {
  ctx->n_bits = n_bits;
  ctx->lc = (int)(n_bits / 16);
  ctx->lp = (int)(n_bits / 32);
  ctx->n = n;
  ctx->nsq = Big::mul(n, n);
  int dev = 0;
  hipDeviceProp_t prop;
  if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return HAFLO_EHIP;
  ctx->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 1;
  ctx->device = dev;
  if (int rc = static_scratch_init()) return rc;

  Uploader up{ctx};
  const int nl_n2 = (int)(n_bits * 9 / 128);
  build_modulus(ctx->N, ctx->nsq, nl_n2, up);
  build_modulus(ctx->Nw, n, nl_n2, up);
  if (!up.ok) return HAFLO_ENOMEM;
  build_prog_encrypt(ctx->prog_enc, n, up);
  {
    // k1 = n * R^2 mod n^2
    Big r1 = Big::mod(Big::pow2((size_t)kLimbBits * nl_n2), ctx->nsq);
    Big r2 = Big::mod(Big::mul(r1, r1), ctx->nsq);
    Big k1 = Big::mod(Big::mul(n, r2), ctx->nsq);
    ctx->d_k1 = up.put(to_limbs29(k1, nl_n2));
  }
  {
    // pair arithmetic modulo n^2: n at half the limbs, and the constants of the pair engine
    const int nl_h = nl_n2 / 2;
    build_modulus(ctx->Nh, n, nl_h, up);
    const Big R = Big::mod(Big::pow2((size_t)kLimbBits * nl_h), ctx->nsq);
    const Big RN = Big::mod(Big::pow2((size_t)kLimbBits * nl_n2), ctx->nsq);
    // 1 / R_N modulo n^2: ((n^2 + 1) / 2)^(29 N.nl)
    MontHost mn2(ctx->nsq);
    const Big half = Big::add(ctx->nsq, Big(1)).shr1();
    const Big rn_inv = mn2.powmod(half, Big((uint64_t)kLimbBits * (uint64_t)nl_n2));
    const Big r2 = Big::mod(Big::mul(R, R), ctx->nsq), r3 = Big::mod(Big::mul(r2, R), ctx->nsq);
    // out of the pair form: times R R_N from a plain pair, times R_N from a pair in Montgomery form; into it
    // from a stored ciphertext W = w_lo + R w_hi (= c R_N): w_lo times R^2 / R_N plus w_hi times R^3 / R_N
    build_pair_consts(ctx->Nh, n, ctx->nsq,
                      {{kConstExtra, Big::mod(Big::mul(R, RN), ctx->nsq)},
                       {kConstR3, RN},
                       {kConstR4, Big::mod(Big::mul(r2, rn_inv), ctx->nsq)},
                       {kConstR5, Big::mod(Big::mul(r3, rn_inv), ctx->nsq)}},
                      up);
    build_prog_encrypt_pairs(ctx->prog_enc_pairs, ctx->prog_enc.sched, up);
  }
  ctx->d_n_words = up.put(to_words(n, ctx->lp));
  ctx->d_nb_words = up.put(to_words(Big::sub(n, Big::pow2(64)), ctx->lp));

  if (p && q) {
    ctx->has_priv = true;
    ctx->p = *p;
    ctx->q = *q;
    const int nl_h = nl_n2 / 2, nl_q = nl_n2 / 4;
    build_modulus(ctx->P2, Big::mul(*p, *p), nl_h, up);
    build_modulus(ctx->Q2, Big::mul(*q, *q), nl_h, up);
    build_modulus(ctx->P, *p, nl_q, up);
    build_modulus(ctx->Q, *q, nl_q, up);
    if (!up.ok) return HAFLO_ENOMEM;
    build_prog_decrypt(ctx->prog_dec_p, Big::sub(*p, Big(1)), up);
    build_prog_decrypt(ctx->prog_dec_q, Big::sub(*q, Big(1)), up);
    build_pair_consts(ctx->P, *p, ctx->P2.mod, {}, up);
    build_pair_consts(ctx->Q, *q, ctx->Q2.mod, {}, up);
    build_prog_decrypt_pairs(ctx->prog_dec_pairs_p, ctx->prog_dec_p.sched, up);
    build_prog_decrypt_pairs(ctx->prog_dec_pairs_q, ctx->prog_dec_q.sched, up);
    {
      Big pm1 = Big::sub(*p, Big(1)), qm1 = Big::sub(*q, Big(1));
      Big ordq = Big::mul(*q, qm1);  // |(Z/q^2)*|
      build_prog_encrypt_low(ctx->prog_enc_p, Big::mod(n, pm1), up);
      build_prog_encrypt_low(ctx->prog_enc_q, Big::mod(n, qm1), up);
      build_prog_encrypt_lift(ctx->prog_lift_p, *p, up);
      build_prog_encrypt_lift(ctx->prog_lift_q, *q, up);
      build_prog_lift_pairs(ctx->prog_lift_pairs_p, ctx->prog_lift_p.sched, up);
      build_prog_lift_pairs(ctx->prog_lift_pairs_q, ctx->prog_lift_q.sched, up);
      // (p^2)^-1 mod q^2 = (p^2)^(q(q-1)-1) mod q^2 (p is a unit there), kept in Montgomery form
      const Big& q2 = ctx->Q2.mod;
      MontHost mq2(q2);
      Big p2_mod_q2 = Big::mod(ctx->P2.mod, q2);
      Big inv = mq2.powmod(p2_mod_q2, Big::sub(ordq, Big(1)));
      Big rq2 = Big::mod(Big::pow2((size_t)kLimbBits * nl_h), q2);
      ctx->d_p2inv = up.put(to_limbs29(Big::mod(Big::mul(inv, rq2), q2), nl_h));
    }
    // With g = n + 1: g^(p-1) mod p^2 = 1 + (p-1)*n mod p^2, so
    // L_p(g^(p-1) mod p^2) = -q mod p and h_p = -(q^-1) mod p (p, q prime).
    MontHost mp(*p), mq(*q);
    Big q_mod_p = (*q >= *p) ? Big::sub(*q, *p) : *q;
    Big p_mod_q = (*p >= *q) ? Big::sub(*p, *q) : *p;
    Big qinv_p = mp.powmod(q_mod_p, Big::sub(*p, Big(2)));
    Big pinv_q = mq.powmod(p_mod_q, Big::sub(*q, Big(2)));
    Big hp = Big::sub(*p, qinv_p);
    Big hq = Big::sub(*q, pinv_q);
    Big rp = Big::mod(Big::pow2((size_t)kLimbBits * nl_q), *p);
    Big rq = Big::mod(Big::pow2((size_t)kLimbBits * nl_q), *q);
    Big hpR = Big::mod(Big::mul(hp, rp), *p);
    Big hqR = Big::mod(Big::mul(hq, rq), *q);
    Big pinvqR = Big::mod(Big::mul(pinv_q, rq), *q);
    Big pinv2 = inv_mod_pow2(*p, (size_t)kLimbBits * nl_q);
    Big qinv2 = inv_mod_pow2(*q, (size_t)kLimbBits * nl_q);
    std::vector<uint32_t> tab;
    for (const Big* b : {(const Big*)&pinv2, (const Big*)&qinv2, (const Big*)&hpR, (const Big*)&hqR, (const Big*)&pinvqR}) {
      std::vector<uint32_t> l = to_limbs29(*b, nl_q);
      tab.insert(tab.end(), l.begin(), l.end());
    }
    ctx->d_priv = up.put(tab);
    if (!up.ok) return HAFLO_ENOMEM;
    ctx->d_pinv = ctx->d_priv;
    ctx->d_qinv = ctx->d_priv + nl_q;
    ctx->d_hp = ctx->d_priv + 2 * nl_q;
    ctx->d_hq = ctx->d_priv + 3 * nl_q;
    ctx->d_pinvq = ctx->d_priv + 4 * nl_q;
  }
  if (!up.ok) return HAFLO_ENOMEM;
  if (hipDeviceSynchronize() != hipSuccess) return HAFLO_EHIP;
  return HAFLO_OK;
}

}  // namespace haflo

using namespace haflo;

extern "C" {

const char* haflo_strerror(int code) {
  switch (code) {
    case HAFLO_OK: return "ok";
    case HAFLO_EINVAL: return "invalid argument";
    case HAFLO_EKEY: return "unusable key material";
    case HAFLO_ENOPRIV: return "operation needs the private key";
    case HAFLO_EHIP: return "HIP runtime error";
    case HAFLO_ENOMEM: return "allocation failed";
    case HAFLO_ETOOBIG: return "batch needs more than the fixed scratch of the allocation-free entry point";
    default: return "unknown error";
  }
}

int haflo_keygen(uint32_t n_bits, uint64_t seed, uint8_t* p_le, uint8_t* q_le) {
  if (!valid_bits(n_bits) || !p_le || !q_le) return HAFLO_EINVAL;
  try {
    SplitMix64 rng(seed);
    size_t half = n_bits / 2;
    Big p = next_prime_from_stream(rng, half);
    for (;;) {
      Big q = next_prime_from_stream(rng, half);
      if (q == p) continue;
      Big n = Big::mul(p, q);
      Big phi = Big::mul(Big::sub(p, Big(1)), Big::sub(q, Big(1)));
      if (Big::gcd(n, phi) != Big(1)) continue;
      p.to_bytes_le(p_le, n_bits / 16);
      q.to_bytes_le(q_le, n_bits / 16);
      return HAFLO_OK;
    }
  } catch (const std::bad_alloc&) {
    return HAFLO_ENOMEM;
  }
}

int haflo_ctx_destroy(haflo_ctx* ctx) {
  if (!ctx) return HAFLO_EINVAL;
  int rc = HAFLO_OK;
  for (void* d : ctx->dev_allocs)
    if (hipFree(d) != hipSuccess) rc = HAFLO_EHIP;
  delete ctx;
  return rc;
}

int haflo_ctx_create_private(const uint8_t* p_le, const uint8_t* q_le, uint32_t n_bits, haflo_ctx** out) {
  if (!p_le || !q_le || !out || !valid_bits(n_bits)) return HAFLO_EINVAL;
  *out = nullptr;
  try {
    Big p = Big::from_bytes_le(p_le, n_bits / 16), q = Big::from_bytes_le(q_le, n_bits / 16);
    if (!p.is_odd() || !q.is_odd() || p == q || p.bits() != n_bits / 2 || q.bits() != n_bits / 2) return HAFLO_EKEY;
    Big n = Big::mul(p, q);
    if (n.bits() != n_bits) return HAFLO_EKEY;
    Big phi = Big::mul(Big::sub(p, Big(1)), Big::sub(q, Big(1)));
    if (Big::gcd(n, phi) != Big(1)) return HAFLO_EKEY;
    haflo_ctx* ctx = new haflo_ctx();
    int rc = ctx_build(ctx, n, &p, &q, n_bits);
    if (rc != HAFLO_OK) {
      haflo_ctx_destroy(ctx);
      return rc;
    }
    *out = ctx;
    return HAFLO_OK;
  } catch (const std::bad_alloc&) {
    return HAFLO_ENOMEM;
  }
}

int haflo_ctx_create_public(const uint8_t* n_le, uint32_t n_bits, haflo_ctx** out) {
  if (!n_le || !out || !valid_bits(n_bits)) return HAFLO_EINVAL;
  *out = nullptr;
  try {
    Big n = Big::from_bytes_le(n_le, n_bits / 8);
    if (!n.is_odd() || n.bits() != n_bits) return HAFLO_EKEY;
    haflo_ctx* ctx = new haflo_ctx();
    int rc = ctx_build(ctx, n, nullptr, nullptr, n_bits);
    if (rc != HAFLO_OK) {
      haflo_ctx_destroy(ctx);
      return rc;
    }
    *out = ctx;
    return HAFLO_OK;
  } catch (const std::bad_alloc&) {
    return HAFLO_ENOMEM;
  }
}

int haflo_ctx_info(const haflo_ctx* ctx, uint32_t* n_bits, uint32_t* cipher_limbs, uint32_t* plain_limbs,
                   size_t* cipher_bytes_internal, size_t* plain_bytes) {
  if (!ctx) return HAFLO_EINVAL;
  if (n_bits) *n_bits = ctx->n_bits;
  if (cipher_limbs) *cipher_limbs = (uint32_t)ctx->lc;
  if (plain_limbs) *plain_limbs = (uint32_t)ctx->lp;
  if (cipher_bytes_internal) *cipher_bytes_internal = (size_t)ctx->N.nl * 4;
  if (plain_bytes) *plain_bytes = (size_t)ctx->lp * 4;
  return HAFLO_OK;
}

int haflo_ctx_set_xtd_bucket_min_rows(haflo_ctx* ctx, size_t min_rows) {
  if (!ctx) return HAFLO_EINVAL;
  ctx->xtd_bucket_min_rows = min_rows ? min_rows : (size_t)HAFLO_XTD_BUCKET_MIN_ROWS_DEFAULT;
  return HAFLO_OK;
}

int haflo_op_cost(const haflo_ctx* ctx, int op, uint64_t* montmuls, uint32_t* modulus_limbs) {
  if (!ctx) return HAFLO_EINVAL;
  uint64_t mm = 0;
  uint32_t limbs = 0;
  if (op == HAFLO_OP_ENCRYPT) {
    if (ctx->has_priv) {
      // through p^2 and q^2, counted in products of the half-size moduli: per branch the second
      // stage (into Montgomery form, the power, out of it) and the first stage on the quarter-size
      // modulus (three products into Montgomery form, the power, one out), a quarter-size product
      // being (2 L^2 + L) / (2 (2L)^2 + 2L) of a half-size one; then one half-size product and one
      // plain product to recombine and three full-size products (= 12 half-size ones) for the
      // (1 + m n) factor and the Montgomery form of the result
      const uint64_t lift = ctx->prog_lift_p.sched.nsquare + ctx->prog_lift_p.sched.nmul +
                            ctx->prog_lift_q.sched.nsquare + ctx->prog_lift_q.sched.nmul + 4;
      const uint64_t low = ctx->prog_enc_p.sched.nsquare + ctx->prog_enc_p.sched.nmul +
                           ctx->prog_enc_q.sched.nsquare + ctx->prog_enc_q.sched.nmul + 8;
      const uint64_t lq = (uint64_t)ctx->lc / 4, lh = (uint64_t)ctx->lc / 2;
      mm = lift + (low * (2 * lq * lq + lq) + (2 * lh * lh + lh) - 1) / (2 * lh * lh + lh) + 2 + 12;
      limbs = (uint32_t)ctx->lc / 2;
    } else {
      // into Montgomery form, the power r^n, (1 + m n) R, the final product
      mm = ctx->prog_enc.sched.nsquare + ctx->prog_enc.sched.nmul + 3;
      limbs = (uint32_t)ctx->lc;
    }
  } else if (op == HAFLO_OP_DECRYPT) {
    if (!ctx->has_priv) return HAFLO_ENOPRIV;
    // per branch: two products to reduce into Montgomery form, the power, one product out
    mm = ctx->prog_dec_p.sched.nsquare + ctx->prog_dec_p.sched.nmul + ctx->prog_dec_q.sched.nsquare +
         ctx->prog_dec_q.sched.nmul + 6;
    limbs = (uint32_t)ctx->lc / 2;
  } else {
    return HAFLO_EINVAL;
  }
  if (montmuls) *montmuls = mm;
  if (modulus_limbs) *modulus_limbs = limbs;
  return HAFLO_OK;
}

// executed multiply-adds of one product on `nl` 29-bit limbs, all lanes of its group together
namespace {
uint64_t sq_products(int lpt) {  // limb products per step a squaring forms with lpt limbs per lane
  uint64_t c = 0;
  for (int j = 0; j < lpt; ++j) {
    const int d = j;  // distance from the broadcast limb 0
    if (d == 0 || (lpt % 2 == 0 && d == lpt / 2) || d <= (lpt - 1) / 2) ++c;
  }
  return c;
}
uint64_t plain_mul_mads(uint64_t nl, int lpt) { return nl * (nl / lpt) * (2 * (uint64_t)lpt) + nl; }
uint64_t plain_sqr_mads(uint64_t nl, int lpt) { return nl * (nl / lpt) * (sq_products(lpt) + (uint64_t)lpt) + nl; }
// the pair arithmetic runs with 9 limbs per lane: two windows, three (two for a squaring) products and two reductions
uint64_t pair_mul_mads(uint64_t nl) { return nl * (nl / 9) * 45 + 2 * nl; }
uint64_t pair_sqr_mads(uint64_t nl) { return nl * (nl / 9) * (sq_products(9) + 27) + 2 * nl; }
}  // namespace

int haflo_op_work(const haflo_ctx* ctx, int op, uint64_t* mads_executed) {
  if (!ctx) return HAFLO_EINVAL;
  uint64_t w = 0;
  if (op == HAFLO_OP_ENCRYPT && !ctx->has_priv) {
    // pairs modulo n: the power, three more products (into Montgomery form, the (1 + m n) factor, out of the
    // pair form) and the plain product n x1 of the stored integer
    const uint64_t nl = (uint64_t)ctx->Nh.nl;
    w = ctx->prog_enc.sched.nsquare * pair_sqr_mads(nl) + (ctx->prog_enc.sched.nmul + 3) * pair_mul_mads(nl) + nl * nl;
  } else if (op == HAFLO_OP_DECRYPT) {
    if (!ctx->has_priv) return HAFLO_ENOPRIV;
    // out of Montgomery form modulo n^2; per prime: four products into the pair form, the power, one out;
    // then three half-size products and one plain product for the recombination
    const uint64_t nl = (uint64_t)ctx->P.nl;
    w = plain_mul_mads((uint64_t)ctx->N.nl, ctx->N.lpt);
    for (const haflo::DevProg* dp : {&ctx->prog_dec_p, &ctx->prog_dec_q})
      w += dp->sched.nsquare * pair_sqr_mads(nl) + (dp->sched.nmul + 5) * pair_mul_mads(nl);
    w += 3 * plain_mul_mads(nl, ctx->P.lpt) + nl * nl;
  } else {
    return HAFLO_EINVAL;
  }
  if (mads_executed) *mads_executed = w;
  return HAFLO_OK;
}

}  // extern "C"
