// Host-side unsigned big integers for key handling: key generation, the
// per-key constants of Montgomery arithmetic and of decryption through the
// prime-power factors. Plain schoolbook algorithms on 32-bit words; nothing
// here runs per ciphertext.
#pragma once
#include <algorithm>
#include <cstdint>
#include <cstring>
#include <vector>

namespace haflo {

class Big {
 public:
  std::vector<uint32_t> w;  // little-endian words, no trailing zero words

  Big() {}
  explicit Big(uint64_t v) {
    if (v) w.push_back((uint32_t)v);
    if (v >> 32) w.push_back((uint32_t)(v >> 32));
  }
  static Big from_bytes_le(const uint8_t* b, size_t nbytes) {
    Big r;
    r.w.assign((nbytes + 3) / 4, 0);
    for (size_t i = 0; i < nbytes; ++i) r.w[i / 4] |= (uint32_t)b[i] << (8 * (i % 4));
    r.trim();
    return r;
  }
  static Big from_words(const uint32_t* p, size_t n) {
    Big r;
    r.w.assign(p, p + n);
    r.trim();
    return r;
  }
  static Big pow2(size_t k) {
    Big r;
    r.w.assign(k / 32 + 1, 0);
    r.w[k / 32] = 1u << (k % 32);
    return r;
  }
  void to_bytes_le(uint8_t* b, size_t nbytes) const {
    for (size_t i = 0; i < nbytes; ++i) b[i] = (i / 4 < w.size()) ? (uint8_t)(w[i / 4] >> (8 * (i % 4))) : 0;
  }
  void trim() {
    while (!w.empty() && w.back() == 0) w.pop_back();
  }
  bool is_zero() const { return w.empty(); }
  bool is_odd() const { return !w.empty() && (w[0] & 1); }
  uint32_t word(size_t i) const { return i < w.size() ? w[i] : 0; }
  size_t bits() const {
    if (w.empty()) return 0;
    return 32 * (w.size() - 1) + (32 - __builtin_clz(w.back()));
  }
  bool bit(size_t i) const { return (word(i / 32) >> (i % 32)) & 1; }
  // bits [pos, pos+len) as an integer, len <= 32
  uint32_t extract(size_t pos, unsigned len) const {
    uint64_t v = (uint64_t)word(pos / 32) | ((uint64_t)word(pos / 32 + 1) << 32);
    v >>= (pos % 32);
    return len >= 32 ? (uint32_t)v : (uint32_t)(v & ((1ull << len) - 1));
  }

  static int cmp(const Big& a, const Big& b) {
    if (a.w.size() != b.w.size()) return a.w.size() < b.w.size() ? -1 : 1;
    for (size_t i = a.w.size(); i-- > 0;)
      if (a.w[i] != b.w[i]) return a.w[i] < b.w[i] ? -1 : 1;
    return 0;
  }
  bool operator==(const Big& o) const { return cmp(*this, o) == 0; }
  bool operator!=(const Big& o) const { return cmp(*this, o) != 0; }
  bool operator<(const Big& o) const { return cmp(*this, o) < 0; }
  bool operator>=(const Big& o) const { return cmp(*this, o) >= 0; }

  static Big add(const Big& a, const Big& b) {
    Big r;
    size_t n = std::max(a.w.size(), b.w.size());
    r.w.resize(n + 1);
    uint64_t c = 0;
    for (size_t i = 0; i < n; ++i) {
      c += (uint64_t)a.word(i) + b.word(i);
      r.w[i] = (uint32_t)c;
      c >>= 32;
    }
    r.w[n] = (uint32_t)c;
    r.trim();
    return r;
  }
  // a - b, requires a >= b
  static Big sub(const Big& a, const Big& b) {
    Big r;
    r.w.resize(a.w.size());
    int64_t c = 0;
    for (size_t i = 0; i < a.w.size(); ++i) {
      c += (int64_t)a.w[i] - b.word(i);
      r.w[i] = (uint32_t)c;
      c >>= 32;
    }
    r.trim();
    return r;
  }
  static Big mul(const Big& a, const Big& b) {
    Big r;
    if (a.is_zero() || b.is_zero()) return r;
    r.w.assign(a.w.size() + b.w.size(), 0);
    for (size_t i = 0; i < a.w.size(); ++i) {
      uint64_t c = 0;
      for (size_t j = 0; j < b.w.size(); ++j) {
        c += (uint64_t)a.w[i] * b.w[j] + r.w[i + j];
        r.w[i + j] = (uint32_t)c;
        c >>= 32;
      }
      r.w[i + b.w.size()] = (uint32_t)c;
    }
    r.trim();
    return r;
  }
  Big shl1() const {
    Big r;
    r.w.resize(w.size() + 1);
    uint32_t c = 0;
    for (size_t i = 0; i < w.size(); ++i) {
      r.w[i] = (w[i] << 1) | c;
      c = w[i] >> 31;
    }
    r.w[w.size()] = c;
    r.trim();
    return r;
  }
  Big shr1() const {
    Big r;
    r.w.resize(w.size());
    for (size_t i = 0; i < w.size(); ++i) r.w[i] = (w[i] >> 1) | (word(i + 1) << 31);
    r.trim();
    return r;
  }
  // low k bits
  Big low_bits(size_t k) const {
    Big r;
    size_t nw = (k + 31) / 32;
    r.w.assign(nw, 0);
    for (size_t i = 0; i < nw; ++i) r.w[i] = word(i);
    if (k % 32) r.w[nw - 1] &= (1u << (k % 32)) - 1;
    r.trim();
    return r;
  }
  uint32_t mod_small(uint32_t d) const {
    uint64_t r = 0;
    for (size_t i = w.size(); i-- > 0;) r = ((r << 32) | w[i]) % d;
    return (uint32_t)r;
  }
  // a mod m by binary shift-and-subtract (only used for per-key constants)
  static Big mod(const Big& a, const Big& m) {
    Big r;
    for (size_t i = a.bits(); i-- > 0;) {
      r = r.shl1();
      if (a.bit(i)) {
        if (r.w.empty()) r.w.push_back(1);
        else r.w[0] |= 1;
      }
      if (r >= m) r = sub(r, m);
    }
    return r;
  }
  // floor(a / m) by the same shift-and-subtract
  static Big div(const Big& a, const Big& m) {
    Big r, q;
    q.w.assign((a.bits() + 31) / 32, 0);
    for (size_t i = a.bits(); i-- > 0;) {
      r = r.shl1();
      if (a.bit(i)) {
        if (r.w.empty()) r.w.push_back(1);
        else r.w[0] |= 1;
      }
      if (r >= m) {
        r = sub(r, m);
        q.w[i / 32] |= 1u << (i % 32);
      }
    }
    q.trim();
    return q;
  }
  static Big gcd(Big a, Big b) {
    if (a.is_zero()) return b;
    if (b.is_zero()) return a;
    size_t shift = 0;
    while (!a.is_odd() && !b.is_odd()) {
      a = a.shr1();
      b = b.shr1();
      ++shift;
    }
    while (!a.is_odd()) a = a.shr1();
    while (!b.is_zero()) {
      while (!b.is_odd()) b = b.shr1();
      if (b < a) std::swap(a, b);
      b = sub(b, a);
    }
    for (size_t i = 0; i < shift; ++i) a = a.shl1();
    return a;
  }
};

// -m^-1 mod 2^32 for odd m0 (Newton iteration on the low word).
inline uint32_t neg_inv32(uint32_t m0) {
  uint32_t x = m0;  // correct to 3 bits
  for (int i = 0; i < 5; ++i) x *= 2 - m0 * x;
  return (uint32_t)(0u - x);
}

// Word-serial Montgomery arithmetic modulo an odd m (host side, 32-bit words).
class MontHost {
 public:
  Big m;
  size_t k;  // words
  uint32_t m0inv;
  Big r1, r2;  // R mod m, R^2 mod m, R = 2^(32k)

  explicit MontHost(const Big& mod_) : m(mod_) {
    k = m.w.size();
    m0inv = neg_inv32(m.w[0]);
    r1 = Big::mod(Big::pow2(32 * k), m);
    r2 = Big::mod(Big::mul(r1, r1), m);
  }
  Big mul(const Big& a, const Big& b) const {
    std::vector<uint32_t> t(k + 2, 0);
    for (size_t i = 0; i < k; ++i) {
      uint64_t c = 0;
      uint32_t bi = b.word(i);
      for (size_t j = 0; j < k; ++j) {
        c += (uint64_t)a.word(j) * bi + t[j];
        t[j] = (uint32_t)c;
        c >>= 32;
      }
      c += t[k];
      t[k] = (uint32_t)c;
      t[k + 1] = (uint32_t)(c >> 32);
      uint32_t q = t[0] * m0inv;
      c = (uint64_t)q * m.w[0] + t[0];
      c >>= 32;
      for (size_t j = 1; j < k; ++j) {
        c += (uint64_t)q * m.w[j] + t[j];
        t[j - 1] = (uint32_t)c;
        c >>= 32;
      }
      c += t[k];
      t[k - 1] = (uint32_t)c;
      t[k] = t[k + 1] + (uint32_t)(c >> 32);
    }
    Big r = Big::from_words(t.data(), k + 1);
    if (r >= m) r = Big::sub(r, m);
    return r;
  }
  Big to_mont(const Big& a) const { return mul(a, r2); }
  Big from_mont(const Big& a) const { return mul(a, Big(1)); }
  // a^e mod m, plain values in and out, a < m
  Big powmod(const Big& a, const Big& e) const {
    Big base = to_mont(a);
    Big acc = r1;
    for (size_t i = e.bits(); i-- > 0;) {
      acc = mul(acc, acc);
      if (e.bit(i)) acc = mul(acc, base);
    }
    return from_mont(acc);
  }
};

// x^-1 mod 2^bits for odd x (Newton doubling on truncated products).
inline Big inv_mod_pow2(const Big& x, size_t bits) {
  Big inv(1);
  size_t have = 1;
  Big two(2);
  while (have < bits) {
    have = std::min(bits, have * 2);
    // inv = inv * (2 - x*inv) mod 2^have
    Big xi = Big::mul(x.low_bits(have), inv).low_bits(have);
    Big t = Big::sub(Big::add(Big::pow2(have), two), xi).low_bits(have);  // 2 - xi mod 2^have
    inv = Big::mul(inv, t).low_bits(have);
  }
  return inv;
}

// SplitMix64 (Steele, Lea, Flood): the stream behind deterministic key generation.
struct SplitMix64 {
  uint64_t s;
  explicit SplitMix64(uint64_t seed) : s(seed) {}
  uint64_t next() {
    s += 0x9E3779B97F4A7C15ull;
    uint64_t z = s;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
  Big words(size_t n64) {
    Big r;
    r.w.resize(2 * n64);
    for (size_t i = 0; i < n64; ++i) {
      uint64_t v = next();
      r.w[2 * i] = (uint32_t)v;
      r.w[2 * i + 1] = (uint32_t)(v >> 32);
    }
    r.trim();
    return r;
  }
};

}  // namespace haflo
