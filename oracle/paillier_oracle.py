"""Plain, slow, arbitrary-precision Paillier: the checker for the HIP path.

TEST INFRASTRUCTURE ONLY. Imported by tests, by the smoke check and by the
benchmark's CPU-baseline leg; never by the product path. It shares no code,
table or constant with the HIP library.

Every operation below is the plain definition written with Python integers:

* encrypt, scalar multiply, add, summation: the operator formulas of the
  paper's Table 1 (all modulo n^2; the identities printed "mod n" in the
  paper's Section 2.3 are a typo for the same formulas).
* key generation and decryption: the paper does not restate them; they are
  Paillier's original scheme (the paper's Section 2.1 cites it) with g = n + 1:
  lambda = lcm(p-1, q-1), mu = L(g^lambda mod n^2)^-1 mod n,
  D(c) = L(c^lambda mod n^2) * mu mod n, L(x) = (x - 1) / n.
* fixed-point encoding: signed fixed point, value * 2^scale rounded to nearest
  (ties to even), negatives stored as n - |q|.
* matrix-vector products: the paper's "Homomorphic Matrix Multiplication" row
  of Table 2 is scalar multiply followed by summation along one axis; signed
  integer exponents, a negative exponent meaning a power of the inverse.

All results are canonical residues, so any correct evaluation order (Montgomery
form, windows, CRT, product trees) must agree with these bit for bit.

Parity pins (see tests/test_oracle_pins.py): exhaustive brute force on tiny keys
(every plaintext, every unit r; discrete-log decryption), additive and scalar
homomorphism, closed-form plaintext sums for the matvecs, CRT == plain
decryption, sympy primality of generated keys, fixed-point round trips and
hand-computed golden values under tests/golden/.
"""
from __future__ import annotations

import math
from dataclasses import dataclass
from typing import Iterable, List, Optional, Sequence, Tuple

MASK64 = (1 << 64) - 1


# --------------------------------------------------------------------------
# deterministic key generation
# --------------------------------------------------------------------------
class SplitMix64:
    """The SplitMix64 counter-based generator (public-domain algorithm by
    Steele, Lea and Flood): state += golden gamma, then two xor-shift-multiply
    rounds. Key generation draws every random word from one such stream."""

    def __init__(self, seed: int):
        self.state = seed & MASK64

    def next(self) -> int:
        self.state = (self.state + 0x9E3779B97F4A7C15) & MASK64
        z = self.state
        z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & MASK64
        z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & MASK64
        return z ^ (z >> 31)

    def words(self, count: int) -> int:
        """`count` 64-bit draws assembled little-endian (first draw = least
        significant word)."""
        v = 0
        for i in range(count):
            v |= self.next() << (64 * i)
        return v


def _small_primes(limit: int) -> List[int]:
    sieve = bytearray([1]) * limit
    sieve[0:2] = b"\x00\x00"
    for i in range(2, int(limit ** 0.5) + 1):
        if sieve[i]:
            sieve[i * i :: i] = bytearray(len(sieve[i * i :: i]))
    return [i for i in range(limit) if sieve[i]]


SMALL_PRIMES = _small_primes(2000)
MR_ROUNDS = 40


def _miller_rabin_round(cand: int, base: int) -> bool:
    """One strong-probable-prime test of odd `cand` to `base`."""
    d = cand - 1
    s = 0
    while d % 2 == 0:
        d //= 2
        s += 1
    x = pow(base, d, cand)
    if x == 1 or x == cand - 1:
        return True
    for _ in range(s - 1):
        x = x * x % cand
        if x == cand - 1:
            return True
    return False


def _next_prime_from_stream(rng: SplitMix64, half_bits: int) -> int:
    """Draw candidates until one passes.

    A candidate is half_bits/64 stream words with the two top bits and the low
    bit forced to one (so a product of two has exactly 2*half_bits bits).
    A candidate divisible by a prime below 2000 is dropped without drawing
    anything else. Otherwise up to 40 Miller-Rabin rounds run, each with a
    base drawn from the stream as (words mod (cand - 3)) + 2; the first failing
    round drops the candidate.
    """
    nwords = half_bits // 64
    while True:
        cand = rng.words(nwords)
        cand |= (3 << (half_bits - 2)) | 1
        if any(cand % sp == 0 for sp in SMALL_PRIMES):
            continue
        ok = True
        for _ in range(MR_ROUNDS):
            base = rng.words(nwords) % (cand - 3) + 2
            if not _miller_rabin_round(cand, base):
                ok = False
                break
        if ok:
            return cand


def keygen(n_bits: int, seed: int) -> Tuple[int, int]:
    """Two primes of n_bits/2 bits each from one SplitMix64 stream: the first
    passing candidate is p; the stream continues for q, redrawn while q == p
    or gcd(pq, (p-1)(q-1)) != 1."""
    if n_bits % 128 != 0 or n_bits < 128:
        raise ValueError("n_bits must be a positive multiple of 128")
    rng = SplitMix64(seed)
    half = n_bits // 2
    p = _next_prime_from_stream(rng, half)
    while True:
        q = _next_prime_from_stream(rng, half)
        if q != p and math.gcd(p * q, (p - 1) * (q - 1)) == 1:
            return p, q


# --------------------------------------------------------------------------
# keys
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class PublicKey:
    n: int

    @property
    def nsq(self) -> int:
        return self.n * self.n

    @property
    def g(self) -> int:
        return self.n + 1


@dataclass(frozen=True)
class PrivateKey:
    p: int
    q: int

    @property
    def n(self) -> int:
        return self.p * self.q

    @property
    def public(self) -> PublicKey:
        return PublicKey(self.n)

    @property
    def lam(self) -> int:
        return math.lcm(self.p - 1, self.q - 1)

    @property
    def mu(self) -> int:
        n = self.n
        return pow(L_function(pow(n + 1, self.lam, n * n), n), -1, n)


def L_function(x: int, n: int) -> int:
    """L(x) = (x - 1) / n, defined where x = 1 mod n."""
    assert (x - 1) % n == 0
    return (x - 1) // n


# --------------------------------------------------------------------------
# operators (Table 1 of the paper, plus decryption)
# --------------------------------------------------------------------------
def encrypt(pk: PublicKey, m: int, r: int) -> int:
    """E(m) = g^m * r^n mod n^2 with 0 <= m < n and r a unit in [1, n)."""
    n, nsq = pk.n, pk.nsq
    if not (0 <= m < n):
        raise ValueError("plaintext out of range")
    if not (1 <= r < n) or math.gcd(r, n) != 1:
        raise ValueError("r must be a unit in [1, n)")
    return pow(pk.g, m, nsq) * pow(r, n, nsq) % nsq


def decrypt(sk: PrivateKey, c: int) -> int:
    """D(c) = L(c^lambda mod n^2) * mu mod n."""
    n = sk.n
    return L_function(pow(c, sk.lam, n * n), n) * sk.mu % n


def decrypt_crt(sk: PrivateKey, c: int) -> int:
    """The same plaintext through the two prime-power factors: for each prime
    s in (p, q), m_s = L_s(c^(s-1) mod s^2) * h_s mod s with
    h_s = L_s(g^(s-1) mod s^2)^-1 mod s, then the Chinese remainder."""
    p, q = sk.p, sk.q
    n = p * q
    res = []
    for s in (p, q):
        hs = pow(L_function(pow(n + 1, s - 1, s * s), s), -1, s)
        res.append(L_function(pow(c % (s * s), s - 1, s * s), s) * hs % s)
    mp, mq = res
    return (mp + p * ((mq - mp) * pow(p, -1, q) % q)) % n


def add(pk: PublicKey, c1: int, c2: int) -> int:
    """E(m1 + m2) = E(m1) * E(m2) mod n^2."""
    return c1 * c2 % pk.nsq


def scalar_mul(pk: PublicKey, c: int, k: int) -> int:
    """E(m * k) = E(m)^k mod n^2; a negative k is a power of the inverse."""
    if k >= 0:
        return pow(c, k, pk.nsq)
    return pow(pow(c, -1, pk.nsq), -k, pk.nsq)


def summation(pk: PublicKey, cs: Iterable[int]) -> int:
    """E(sum m_i) = prod E(m_i) mod n^2; the empty product is 1."""
    acc = 1
    for c in cs:
        acc = acc * c % pk.nsq
    return acc


def summation_segments(pk: PublicKey, cs: Sequence[int], offsets: Sequence[int]) -> List[int]:
    """The summation of Table 1 over consecutive slices of one array: output i
    is the product of cs[offsets[i]:offsets[i+1]] modulo n^2 (1 for an empty
    slice). offsets is non-decreasing and stays within the array."""
    assert all(0 <= a <= b <= len(cs) for a, b in zip(offsets, offsets[1:]))
    return [summation(pk, cs[a:b]) for a, b in zip(offsets, offsets[1:])]


def matvec(pk: PublicKey, orientation: int, cs: Sequence[int], X: Sequence[Sequence[int]]) -> List[int]:
    """Ciphertext matrix-vector product with signed integer exponents.

    orientation 0 (encrypted gradient X^T [[d]]): len(cs) == rows,
        out[j] = prod_i cs[i]^X[i][j] mod n^2 for each column j.
    orientation 1 (encrypted forward pass X [[w]]): len(cs) == cols,
        out[i] = prod_j cs[j]^X[i][j] mod n^2 for each row i.
    """
    rows = len(X)
    cols = len(X[0]) if rows else 0
    if orientation == 0:
        assert len(cs) == rows
        return [summation(pk, (scalar_mul(pk, cs[i], int(X[i][j])) for i in range(rows))) for j in range(cols)]
    if orientation == 1:
        assert len(cs) == cols
        return [summation(pk, (scalar_mul(pk, cs[j], int(X[i][j])) for j in range(cols))) for i in range(rows)]
    raise ValueError("orientation must be 0 or 1")


def encrypt_with_obfuscator(pk: PublicKey, m: int, obfuscator: int) -> int:
    """Table 1's encryption g^m * r^n mod n^2 with the factor r^n supplied ready-made."""
    assert 0 <= m < pk.n and 0 <= obfuscator < pk.nsq
    return pow(pk.g, m, pk.nsq) * obfuscator % pk.nsq


def fore_gradient(pk: PublicKey, c_host: int, logit_guest: float, label: float, r: int,
                  scale_bits: int) -> Tuple[int, int]:
    """Guest's fore gradient of heterogeneous logistic regression, section 3.4 (workflow figure):
    [[0.25 * (logits_host + logits_guest) - 0.5 * label]].

    Fixed-point reading: c_host encrypts q(logits_host) at scale 2^scale_bits; the guest adds an
    encryption of q(logits_guest) - 2 q(label). The sum q_host + q_guest - 2 q_label is
    4 * 2^scale_bits times the fore gradient, so the result is read at scale 2^(scale_bits + 2)
    and the factor 0.25 needs no ciphertext operation.

    Returns (ciphertext, status): status 1 and a guest part of 0 when an input is not finite or a
    quantised input reaches 2^61 in magnitude, else status 0."""
    qg, ql = quantise(logit_guest, scale_bits), quantise(label, scale_bits)
    ok = qg is not None and ql is not None and abs(qg) < (1 << 61) and abs(ql) < (1 << 61)
    q = qg - 2 * ql if ok else 0
    return add(pk, c_host, encrypt(pk, q % pk.n, r)), (0 if ok else 1)


def taylor_loss(pk: PublicKey, c_u: Sequence[int], c_u2: Sequence[int], u_guest: Sequence[float],
                label: Sequence[float], r: int, scale_bits: int) -> Tuple[int, int]:
    """Encrypted second-order Taylor loss of section 2.1 (the approximated l_H) without its public
    parts (log 2 per instance, the factor 1/h):  sum_i ( -1/2 y_i u_i + 1/8 u_i^2 ),
    u_i = u_host,i + u_guest,i.

    c_u[i] encrypts m1_i = q(u_host,i), c_u2[i] encrypts m2_i = m1_i^2 (scale 2^s and 2^(2s)).
    Multiplying the sum by 8 * 2^(2s) gives sum_i ( m2_i + k_i m1_i + p_i ) with
    k_i = 2 q(u_guest,i) - 4 q(y_i) and p_i = q(u_guest,i) (q(u_guest,i) - 4 q(y_i)); on ciphertexts
    that is the summation of c_u2, the product of c_u[i]^(k_i) and one encryption of sum p_i.

    Returns (ciphertext, status): an element that is not finite or too large (|q(u_guest)| >= 2^28,
    |q(y)| >= 2^27) counts with k_i = p_i = 0 and sets status 1."""
    assert len(c_u) == len(c_u2) == len(u_guest) == len(label)
    status = 0
    ks, plain = [], 0
    for ug, y in zip(u_guest, label):
        qg, qy = quantise(ug, scale_bits), quantise(y, scale_bits)
        if qg is None or qy is None or abs(qg) >= (1 << 28) or abs(qy) >= (1 << 27):
            qg, qy, status = 0, 0, 1
        ks.append(2 * qg - 4 * qy)
        plain += qg * (qg - 4 * qy)
    out = summation(pk, c_u2)
    out = add(pk, out, summation(pk, (scalar_mul(pk, c, k) for c, k in zip(c_u, ks))))
    out = add(pk, out, encrypt(pk, plain % pk.n, r))
    return out, status


# --------------------------------------------------------------------------
# signed fixed point
# --------------------------------------------------------------------------
INT64_MIN = -(1 << 63)
INT64_MAX = (1 << 63) - 1


def quantise(v: float, scale_bits: int) -> Optional[int]:
    """rint(v * 2^scale) as an integer, ties to even, computed in binary64
    (a binary32 input widens exactly and the power-of-two product is exact
    short of overflow). None when v is not finite or the result leaves int64."""
    v = float(v)
    if math.isnan(v) or math.isinf(v):
        return None
    try:
        scaled = math.ldexp(v, scale_bits)
    except OverflowError:
        return None
    if math.isinf(scaled):
        return None
    # round half to even on an exactly representable binary64 value
    fl = math.floor(scaled)
    diff = scaled - fl
    if diff > 0.5 or (diff == 0.5 and (int(fl) & 1)):
        q = int(fl) + 1
    else:
        q = int(fl)
    if q < INT64_MIN or q > INT64_MAX:
        return None
    return q


def encode(pk: PublicKey, v: float, scale_bits: int) -> Tuple[int, int]:
    """(residue, status): residue = q mod n with q = quantise(v); status 1 and
    residue 0 when q is undefined."""
    q = quantise(v, scale_bits)
    if q is None:
        return 0, 1
    return q % pk.n, 0


def encode_exponent(v: float, scale_bits: int) -> Tuple[int, int]:
    """(exponent, status) for a matrix entry: the same quantisation, kept as a
    signed 32-bit integer; status 1 and exponent 0 when it does not fit."""
    q = quantise(v, scale_bits)
    if q is None or q < -(1 << 31) or q > (1 << 31) - 1:
        return 0, 1
    return q, 0


def decode(pk: PublicKey, m: int, scale_bits: int) -> Tuple[int, float, int]:
    """(q, value, status): signed lift (m > floor(n/2) means m - n), then
    value = q / 2^scale with q converted to binary64 by round-to-nearest-even.
    status 1 (q = 0, value = 0.0) when the lifted integer leaves int64."""
    n = pk.n
    q = m if m <= n // 2 else m - n
    if q < INT64_MIN or q > INT64_MAX:
        return 0, 0.0, 1
    return q, math.ldexp(float(q), -scale_bits), 0


# --------------------------------------------------------------------------
# interchange format helpers (little-endian 32-bit limbs)
# --------------------------------------------------------------------------
def to_limbs(x: int, nlimbs: int) -> List[int]:
    assert 0 <= x < (1 << (32 * nlimbs))
    return [(x >> (32 * i)) & 0xFFFFFFFF for i in range(nlimbs)]


def from_limbs(limbs: Sequence[int]) -> int:
    v = 0
    for i, w in enumerate(limbs):
        v |= int(w) << (32 * i)
    return v
