"""Pins for the CPU oracle: checks against things other than itself.

Brute force on tiny keys, the operator identities of the paper's Table 1,
closed forms on plaintexts, hand-worked golden values, independent primality
checks and fixed-point round trips. A dropped term, a wrong sign, modulus or
index anywhere in oracle/paillier_oracle.py fails at least one of these.
"""
import math
import os
import random

import numpy as np
import pytest
import sympy

from oracle import paillier_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "tiny_paillier.txt")

TINY_PRIMES = [(5, 7), (7, 11), (11, 13), (13, 17), (17, 19), (23, 29), (29, 31)]


def tiny_keys():
    return [O.PrivateKey(p, q) for p, q in TINY_PRIMES if math.gcd(p * q, (p - 1) * (q - 1)) == 1]


def read_golden():
    vals = {}
    with open(GOLDEN) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, v = line.split()
            vals[k] = int(v)
    return vals


def test_golden_hand_worked_values():
    g = read_golden()
    sk = O.PrivateKey(g["p"], g["q"])
    pk = sk.public
    assert pk.n == g["n"] and pk.nsq == g["nsq"]
    assert sk.lam == g["lambda"] and sk.mu == g["mu"]
    assert O.encrypt(pk, 0, 2) == g["enc_m0_r2"] == g["r2_pow_n"]
    assert O.encrypt(pk, 1, 2) == g["enc_m1_r2"]
    assert O.encrypt(pk, 5, 2) == g["enc_m5_r2"]
    assert O.add(pk, g["enc_m1_r2"], g["enc_m5_r2"]) == g["prod_m1_m5"]
    assert O.decrypt(sk, g["prod_m1_m5"]) == 6
    assert O.decrypt_crt(sk, g["prod_m1_m5"]) == 6


def brute_force_decrypt(pk, c):
    """Independent of lambda/mu: c = (1+n)^m r^n means c^phi-free search - find
    the unique m with c * (1+n)^-m an n-th power residue, by exhausting r."""
    n, nsq = pk.n, pk.nsq
    nth_powers = {pow(r, n, nsq) for r in range(1, n) if math.gcd(r, n) == 1}
    hits = [m for m in range(n) if (c * pow(pow(1 + n, m, nsq), -1, nsq)) % nsq in nth_powers]
    assert len(hits) == 1
    return hits[0]


@pytest.mark.parametrize("sk", tiny_keys()[:4], ids=lambda k: "p%dq%d" % (k.p, k.q))
def test_exhaustive_encrypt_decrypt_tiny(sk):
    pk = sk.public
    n, nsq = pk.n, pk.nsq
    units = [r for r in range(1, n) if math.gcd(r, n) == 1]
    seen = set()
    for m in range(n):
        for r in units:
            c = O.encrypt(pk, m, r)
            # definition vs binomial shortcut g^m = 1 + m n
            assert c == (1 + m * n) * pow(r, n, nsq) % nsq
            assert O.decrypt(sk, c) == m
            assert O.decrypt_crt(sk, c) == m
            seen.add(c)
    # encryption is a bijection Z_n x Z_n^* -> Z_{n^2}^*
    assert len(seen) == n * len(units)
    assert len(seen) == sum(1 for c in range(nsq) if math.gcd(c, nsq) == 1)


def test_decrypt_matches_discrete_log_brute_force():
    sk = O.PrivateKey(7, 11)
    pk = sk.public
    rng = random.Random(3)
    for _ in range(12):
        m = rng.randrange(pk.n)
        r = rng.choice([r for r in range(1, pk.n) if math.gcd(r, pk.n) == 1])
        c = O.encrypt(pk, m, r)
        assert brute_force_decrypt(pk, c) == m == O.decrypt(sk, c)


@pytest.mark.parametrize("sk", tiny_keys(), ids=lambda k: "p%dq%d" % (k.p, k.q))
def test_homomorphic_identities_tiny(sk):
    pk = sk.public
    n = pk.n
    rng = random.Random(n)
    units = [r for r in range(1, n) if math.gcd(r, n) == 1]
    for _ in range(60):
        a, b = rng.randrange(n), rng.randrange(n)
        ca, cb = O.encrypt(pk, a, rng.choice(units)), O.encrypt(pk, b, rng.choice(units))
        assert O.decrypt(sk, O.add(pk, ca, cb)) == (a + b) % n
        for k in (0, 1, 2, 3, n - 1, n, n + 5, -1, -2, -n - 3):
            assert O.decrypt(sk, O.scalar_mul(pk, ca, k)) == (a * k) % n
        assert O.scalar_mul(pk, ca, 0) == 1
        # a negative power is the inverse of the positive one
        assert O.scalar_mul(pk, ca, -3) * O.scalar_mul(pk, ca, 3) % pk.nsq == 1


def _real_key(bits):
    from conftest import oracle_key
    p, q = oracle_key(bits)
    return O.PrivateKey(p, q)


@pytest.mark.parametrize("bits", [512, 1024, 2048])
def test_keygen_properties(bits):
    sk = _real_key(bits)
    p, q = sk.p, sk.q
    assert sympy.isprime(p) and sympy.isprime(q) and p != q
    assert p.bit_length() == bits // 2 and q.bit_length() == bits // 2
    assert (p * q).bit_length() == bits
    assert math.gcd(p * q, (p - 1) * (q - 1)) == 1
    # deterministic in the seed, different across seeds
    from paper_2107_13797_amd import synth
    assert O.keygen(bits, synth.BASE_SEED + bits) == (p, q)
    if bits == 512:
        assert O.keygen(bits, 1) != (p, q)


def test_splitmix64_reference_values():
    # first outputs of SplitMix64 seeded with 0 as published with the algorithm
    # (widely reproduced test vector of the reference implementation)
    rng = O.SplitMix64(0)
    assert [rng.next() for _ in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_miller_rabin_against_sympy():
    rng = random.Random(9)
    for _ in range(300):
        cand = rng.getrandbits(48) | 1 | (1 << 47)
        verdict = all(O._miller_rabin_round(cand, b) for b in (2, 3, 5, 7, 11, 13, 17, 19, 23, 29, 31, 37))
        assert verdict == sympy.isprime(cand)


@pytest.mark.parametrize("bits", [512, 1024, 2048])
def test_roundtrip_and_crt_real_sizes(bits):
    sk = _real_key(bits)
    pk = sk.public
    n = pk.n
    rng = random.Random(bits)
    ms = [0, 1, n - 1, n // 2, n // 2 + 1] + [rng.randrange(n) for _ in range(3)]
    for m in ms:
        r = rng.randrange(1, n)
        c = O.encrypt(pk, m, r)
        assert c == (1 + m * n) * pow(r, n, pk.nsq) % pk.nsq
        assert O.decrypt(sk, c) == m
        assert O.decrypt_crt(sk, c) == m
    a, b = ms[-1], ms[-2]
    ca, cb = O.encrypt(pk, a, 2), O.encrypt(pk, b, 3)
    assert O.decrypt_crt(sk, O.add(pk, ca, cb)) == (a + b) % n
    k = rng.getrandbits(64)
    assert O.decrypt_crt(sk, O.scalar_mul(pk, ca, k)) == a * k % n
    assert O.decrypt_crt(sk, O.scalar_mul(pk, ca, -k)) == (-a * k) % n
    assert O.decrypt_crt(sk, O.summation(pk, [ca, cb, ca])) == (2 * a + b) % n
    assert O.summation(pk, []) == 1


def test_summation_segments_decrypt_to_slice_sums():
    """Every segment's product decrypts (through the brute-force-pinned decryption) to the sum of
    its slice of plaintexts; empty segments give the encryption-free 1; one segment over the whole
    array is the plain summation; on a tiny key the products are also checked by brute force."""
    sk = _real_key(512)
    pk = sk.public
    n = pk.n
    rng = random.Random(13)
    ms = [rng.randrange(n) for _ in range(23)]
    cs = [O.encrypt(pk, m, rng.randrange(1, n)) for m in ms]
    offsets = [0, 0, 1, 1, 9, 20, 20, 23]
    out = O.summation_segments(pk, cs, offsets)
    assert len(out) == len(offsets) - 1
    assert [O.decrypt_crt(sk, c) for c in out] == [sum(ms[a:b]) % n for a, b in zip(offsets, offsets[1:])]
    assert out[0] == 1 and out[2] == 1 and out[5] == 1 and out[1] == cs[0]
    assert O.summation_segments(pk, cs, [0, 23]) == [O.summation(pk, cs)]
    assert O.summation_segments(pk, cs, [4, 7]) == [cs[4] * cs[5] * cs[6] % pk.nsq]
    assert O.summation_segments(pk, cs, [5]) == [] and O.summation_segments(pk, [], [0, 0]) == [1]
    tiny = O.PrivateKey(11, 13)
    tcs = [O.encrypt(tiny.public, m, r) for m, r in ((3, 2), (140, 5), (0, 7), (77, 9))]
    got = O.summation_segments(tiny.public, tcs, [1, 3, 4])
    assert [brute_force_decrypt(tiny.public, c) for c in got] == [140 % 143, 77]


def test_matvec_closed_form_on_plaintexts():
    """D(out) must equal the integer matrix-vector product of the plaintexts
    (exact Python integers), for both orientations, with signed entries."""
    sk = _real_key(512)
    pk = sk.public
    n = pk.n
    rng = random.Random(11)
    rows, cols = 6, 4
    X = [[rng.randrange(-(1 << 18), 1 << 18) for _ in range(cols)] for _ in range(rows)]
    X[0][0] = 0
    X[1][1] = -1
    md = [rng.randrange(n) for _ in range(rows)]
    cd = [O.encrypt(pk, m, rng.randrange(1, n)) for m in md]
    out0 = O.matvec(pk, 0, cd, X)
    assert [O.decrypt_crt(sk, c) for c in out0] == [sum(X[i][j] * md[i] for i in range(rows)) % n for j in range(cols)]
    mw = [rng.randrange(n) for _ in range(cols)]
    cw = [O.encrypt(pk, m, rng.randrange(1, n)) for m in mw]
    out1 = O.matvec(pk, 1, cw, X)
    assert [O.decrypt_crt(sk, c) for c in out1] == [sum(X[i][j] * mw[j] for j in range(cols)) % n for i in range(rows)]


def test_matvec_special_cases():
    sk = _real_key(512)
    pk = sk.public
    rng = random.Random(12)
    cs = [O.encrypt(pk, rng.randrange(pk.n), rng.randrange(1, pk.n)) for _ in range(4)]
    ident = [[1 if i == j else 0 for j in range(4)] for i in range(4)]
    assert O.matvec(pk, 0, cs, ident) == cs
    assert O.matvec(pk, 1, cs, ident) == cs
    ones = [[1] for _ in range(4)]
    assert O.matvec(pk, 0, cs, ones) == [O.summation(pk, cs)]
    single_neg = [[0], [-1], [0], [0]]
    assert O.matvec(pk, 0, cs, single_neg) == [pow(cs[1], -1, pk.nsq)]
    zeros = [[0, 0] for _ in range(4)]
    assert O.matvec(pk, 0, cs, zeros) == [1, 1]
    assert O.matvec(pk, 1, cs, [[0, 0, 0, 0]]) == [1]
    # transposition: orientation 1 on X equals orientation 0 on X^T
    X = [[rng.randrange(-50, 50) for _ in range(4)] for _ in range(3)]
    Xt = [list(col) for col in zip(*X)]
    assert O.matvec(pk, 1, cs, X) == O.matvec(pk, 0, cs, Xt)


def test_tiny_matvec_brute_force():
    sk = O.PrivateKey(11, 13)
    pk = sk.public
    n = pk.n
    units = [r for r in range(1, n) if math.gcd(r, n) == 1]
    rng = random.Random(5)
    md = [rng.randrange(n) for _ in range(3)]
    cd = [O.encrypt(pk, m, rng.choice(units)) for m in md]
    X = [[2, -3], [-1, 0], [5, 7]]
    out = O.matvec(pk, 0, cd, X)
    for j, c in enumerate(out):
        assert brute_force_decrypt(pk, c) == sum(X[i][j] * md[i] for i in range(3)) % n


def test_fixed_point_matches_numpy_rint():
    pk = O.PublicKey(_real_key(512).n)
    rng = np.random.default_rng(1)
    vals = np.concatenate([
        rng.normal(0, 0.25, 2000).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 0.5, -0.5, 1.5 * 2.0 ** -24, 2.5 * 2.0 ** -24, -1.5 * 2.0 ** -24,
                  -2.5 * 2.0 ** -24, 2.0 ** -25, -(2.0 ** -25), 1e-40, -1e-40, 3.4e38, -3.4e38, 1e10, -1e10],
                 dtype=np.float32)])
    for s in (0, 16, 24, 40):
        for v in vals:
            ref = np.rint(np.float64(v) * 2.0 ** s)
            q = O.quantise(float(v), s)
            if abs(ref) >= 2.0 ** 63:
                assert q is None
                assert O.encode(pk, float(v), s) == (0, 1)
                continue
            assert q == int(ref)
            m, st = O.encode(pk, float(v), s)
            assert st == 0 and m == q % pk.n
            q2, val, st2 = O.decode(pk, m, s)
            assert (q2, st2) == (q, 0)
            assert val == float(q) / 2.0 ** s
    # ties go to even
    assert [O.quantise(x, 0) for x in (0.5, 1.5, 2.5, -0.5, -1.5, -2.5)] == [0, 2, 2, 0, -2, -2]
    for bad in (float("inf"), float("-inf"), float("nan")):
        assert O.quantise(bad, 24) is None and O.encode(pk, bad, 24) == (0, 1)


def test_decode_sign_threshold_and_range():
    pk = O.PublicKey(_real_key(512).n)
    n = pk.n
    assert O.decode(pk, n // 2, 0)[2] == 1            # positive but far beyond int64
    assert O.decode(pk, 5, 0) == (5, 5.0, 0)
    assert O.decode(pk, n - 5, 0) == (-5, -5.0, 0)
    assert O.decode(pk, 2 ** 63 - 1, 0)[0::2] == (2 ** 63 - 1, 0)
    assert O.decode(pk, 2 ** 63, 0)[2] == 1
    assert O.decode(pk, n - 2 ** 63, 0)[0::2] == (-(2 ** 63), 0)
    assert O.decode(pk, n - 2 ** 63 - 1, 0)[2] == 1
    # the lift is exactly the centred residue
    tiny = O.PublicKey(77)
    assert [O.decode(tiny, m, 0)[0] for m in (0, 38, 39, 76)] == [0, 38, -38, -1]
    assert O.encode_exponent(0.5, 16) == (32768, 0)
    assert O.encode_exponent(-40000.0, 16) == (0, 1)
    assert O.encode_exponent(32767.99, 16)[1] == 0


def test_limb_helpers_roundtrip():
    rng = random.Random(2)
    for bits in (64, 1024, 2048):
        x = rng.getrandbits(bits)
        limbs = O.to_limbs(x, bits // 32)
        assert all(0 <= w < 2 ** 32 for w in limbs) and O.from_limbs(limbs) == x
    assert O.to_limbs(1 + (2 << 32), 3) == [1, 2, 0]


def test_fore_gradient_plaintext_closed_form():
    """Section 3.4's fore gradient 0.25 (logits_host + logits_guest) - 0.5 label: the decrypted,
    decoded result equals the exact integer combination of the three quantised inputs at scale
    2^(s+2), and lies within the quantisation bound of the real-valued formula. A wrong sign, a
    missing factor 2 on the label or a wrong output scale breaks one of the two."""
    sk = _real_key(512)
    pk = sk.public
    rng = random.Random(99)
    s = 24
    for _ in range(40):
        uh, ug = rng.gauss(0, 2.0), rng.gauss(0, 2.0)
        y = rng.choice([-1.0, 1.0, 0.0])
        uh32, ug32 = float(np.float32(uh)), float(np.float32(ug))
        qh = O.quantise(uh32, s)
        c_host = O.encrypt(pk, qh % pk.n, rng.randrange(1, pk.n))
        c, st = O.fore_gradient(pk, c_host, ug32, y, rng.randrange(1, pk.n), s)
        assert st == 0
        m = O.decrypt(sk, c)
        qd, val, dst = O.decode(pk, m, s + 2)
        assert dst == 0
        assert qd == qh + O.quantise(ug32, s) - 2 * O.quantise(y, s)
        want = 0.25 * (uh32 + ug32) - 0.5 * y
        assert abs(val - want) <= 2.0 ** -(s + 1)
    c, st = O.fore_gradient(pk, 1, float("nan"), 1.0, 5, s)
    assert st == 1 and c == O.encrypt(pk, 0, 5)
    c, st = O.fore_gradient(pk, 1, 1.0, 2.0 ** 38, 5, s)       # 2^62 after scaling
    assert st == 1 and c == O.encrypt(pk, 0, 5)


def test_taylor_loss_plaintext_closed_form():
    """Section 2.1's approximated loss: decrypting the oracle's loss ciphertext and decoding at
    scale 2^(2s+3) gives the exact integer combination and lies within the quantisation bound of
    sum(-y u / 2 + u^2 / 8) evaluated in floating point. A wrong coefficient or sign breaks it."""
    sk = _real_key(512)
    pk = sk.public
    rng = random.Random(5)
    s, count = 20, 24
    uh = [float(np.float32(rng.gauss(0, 1.5))) for _ in range(count)]
    ug = [float(np.float32(rng.gauss(0, 1.5))) for _ in range(count)]
    y = [rng.choice([-1.0, 1.0]) for _ in range(count)]
    m1 = [O.quantise(v, s) for v in uh]
    c_u = [O.encrypt(pk, m % pk.n, rng.randrange(1, pk.n)) for m in m1]
    c_u2 = [O.encrypt(pk, m * m, rng.randrange(1, pk.n)) for m in m1]
    c, st = O.taylor_loss(pk, c_u, c_u2, ug, y, rng.randrange(1, pk.n), s)
    assert st == 0
    q, val, dst = O.decode(pk, O.decrypt(sk, c), 2 * s + 3)
    assert dst == 0
    qg = [O.quantise(v, s) for v in ug]
    qy = [O.quantise(v, s) for v in y]
    assert q == sum((a + b) ** 2 - 4 * t * (a + b) for a, b, t in zip(m1, qg, qy))
    want = sum(-0.5 * t * (a + b) + 0.125 * (a + b) ** 2 for a, b, t in zip(uh, ug, y))
    # each u is off by at most 2^-s (two roundings); d/du of the term is |u/4 - y/2| <= 2 here
    assert abs(val - want) <= count * 2.0 * 2.0 ** -s + count * 2.0 ** (-2 * s)
    c, st = O.taylor_loss(pk, c_u[:2], c_u2[:2], [float("inf"), 0.0], [1.0, 1.0], 7, s)
    assert st == 1
    assert O.decrypt(sk, c) == (m1[0] ** 2 + m1[1] ** 2 - 4 * (1 << s) * m1[1]) % pk.n


def test_obfuscator_encryption_is_the_same_encryption():
    """E(m; r) = g^m * (r^n): with the obfuscator r^n = E(0; r) the split form must reproduce the
    ordinary encryption on every plaintext and unit of a tiny key, and on a real key."""
    for sk in tiny_keys():
        pk = sk.public
        for r in range(1, pk.n):
            if math.gcd(r, pk.n) != 1:
                continue
            obf = O.encrypt(pk, 0, r)
            assert obf == pow(r, pk.n, pk.nsq)
            for m in range(pk.n):
                assert O.encrypt_with_obfuscator(pk, m, obf) == O.encrypt(pk, m, r)
    pk = _real_key(512).public
    rng = random.Random(8)
    m, r = rng.randrange(pk.n), rng.randrange(1, pk.n)
    assert O.encrypt_with_obfuscator(pk, m, O.encrypt(pk, 0, r)) == O.encrypt(pk, m, r)
