// Test-only C wrapper around the host big-integer helpers of the library (hostbig.hpp), so that
// tests can compare them with Python integers. Built with g++ by tests/test_hostbig.py.
#include <stdint.h>
#include <string.h>

#include "../paper_2107_13797_amd/csrc/hostbig.hpp"

using haflo::Big;

namespace {
Big get(const uint8_t* p, size_t n) { return Big::from_bytes_le(p, n); }
}

extern "C" {

enum { OP_ADD = 0, OP_SUB, OP_MUL, OP_MOD, OP_GCD, OP_POWMOD, OP_INV_POW2, OP_SHL1, OP_SHR1, OP_LOW_BITS, OP_MONTMUL, OP_DIV };

// out (nout bytes, little-endian) = op(a, b, c); k is a small integer argument. Returns the bit
// length of the result, or -1 for an unknown op.
long hostbig_op(int op, const uint8_t* a, size_t na, const uint8_t* b, size_t nb, const uint8_t* c, size_t nc,
                uint64_t k, uint8_t* out, size_t nout) {
  Big x = get(a, na), y = get(b, nb), z = get(c, nc), r;
  switch (op) {
    case OP_ADD: r = Big::add(x, y); break;
    case OP_SUB: r = Big::sub(x, y); break;
    case OP_MUL: r = Big::mul(x, y); break;
    case OP_MOD: r = Big::mod(x, y); break;
    case OP_GCD: r = Big::gcd(x, y); break;
    case OP_POWMOD: r = haflo::MontHost(z).powmod(x, y); break;   // x^y mod z, z odd, x < z
    case OP_INV_POW2: r = haflo::inv_mod_pow2(x, (size_t)k); break;
    case OP_SHL1: r = x.shl1(); break;
    case OP_SHR1: r = x.shr1(); break;
    case OP_LOW_BITS: r = x.low_bits((size_t)k); break;
    case OP_MONTMUL: r = haflo::MontHost(z).mul(x, y); break;     // x y R^-1 mod z, R = 2^(32 words(z))
    case OP_DIV: r = Big::div(x, y); break;
    default: return -1;
  }
  r.to_bytes_le(out, nout);
  return (long)r.bits();
}

uint32_t hostbig_neg_inv32(uint32_t m0) { return haflo::neg_inv32(m0); }
uint32_t hostbig_mod_small(const uint8_t* a, size_t na, uint32_t d) { return get(a, na).mod_small(d); }
int hostbig_cmp(const uint8_t* a, size_t na, const uint8_t* b, size_t nb) { return Big::cmp(get(a, na), get(b, nb)); }
uint32_t hostbig_extract(const uint8_t* a, size_t na, uint64_t pos, unsigned len) { return get(a, na).extract((size_t)pos, len); }

}  // extern "C"
