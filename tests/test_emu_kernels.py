"""The library's kernel sources, compiled for the CPU against a stand-in for the
HIP runtime (tests/emu), run through the same C entry points and compared with
the oracle. This is a host-side check of indexing, bounds (device buffers end
at a guard page) and lock-step convergence of the cross-lane code; it is not a
parity claim for the GPU build, which tests/test_gpu_parity.py covers.
"""
import ctypes as C
import os
import random

import numpy as np
import pytest

from conftest import oracle_key
from oracle import paillier_oracle as O
from paper_2107_13797_amd import _cabi, synth

BITS = 512


@pytest.fixture(scope="module")
def emu():
    import sys, os
    sys.path.insert(0, os.path.join(os.path.dirname(__file__), "emu"))
    import build_emu
    lib = _cabi.bind(C.CDLL(build_emu.build()))
    lib.hipemu_alloc.restype = C.c_void_p
    lib.hipemu_alloc.argtypes = [C.c_size_t]
    lib.hipemu_free.argtypes = [C.c_void_p]
    return lib


class Dev:
    """A 'device' buffer of the emulated runtime holding a numpy array."""

    def __init__(self, lib, arr):
        arr = np.ascontiguousarray(arr)
        self.lib, self.n, self.dtype, self.shape = lib, arr.nbytes, arr.dtype, arr.shape
        self.p = lib.hipemu_alloc(max(self.n, 1))
        C.memmove(self.p, arr.ctypes.data, self.n)

    def get(self):
        out = np.empty(self.shape, self.dtype)
        C.memmove(out.ctypes.data, self.p, self.n)
        return out

    def __del__(self):
        self.lib.hipemu_free(self.p)


@pytest.fixture(scope="module")
def env(emu):
    p, q = oracle_key(BITS)
    sk = O.PrivateKey(p, q)
    ctx = C.c_void_p()

    def le(x, nbytes):
        return (C.c_uint8 * nbytes).from_buffer_copy(x.to_bytes(nbytes, "little"))

    assert emu.haflo_ctx_create_private(le(p, BITS // 16), le(q, BITS // 16), BITS, C.byref(ctx)) == 0
    cb = C.c_size_t()
    emu.haflo_ctx_info(ctx, None, None, None, C.byref(cb), None)
    yield emu, ctx, sk, cb.value // 4
    emu.haflo_ctx_destroy(ctx)


def words(lib, xs, nl):
    return Dev(lib, synth.ints_to_words(xs, nl))


def zeros(lib, shape, dtype=np.uint32):
    return Dev(lib, np.zeros(shape, dtype))


def export(lib, ctx, d_cipher, count):
    out = zeros(lib, (count, BITS // 16))
    assert lib.haflo_export_cipher(ctx, d_cipher.p, out.p, count, None) == 0
    return synth.words_to_ints(out.get())


def ws(lib, ctx, op, rows, cols=0):
    nb = lib.haflo_workspace_bytes(ctx, op, rows, cols)
    assert nb != 2 ** 64 - 1
    return zeros(lib, (nb // 4 + 1,)), nb


def test_import_export_add_and_montgomery_form(env):
    lib, ctx, sk, nlw = env
    n, nsq = sk.n, sk.n ** 2
    rng = random.Random(1)
    cs = [rng.randrange(nsq) for _ in range(5)] + [0, 1, nsq - 1]
    d_int, st = zeros(lib, (len(cs), nlw)), zeros(lib, (1,))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, BITS // 16).p, d_int.p, st.p, len(cs), None) == 0
    assert export(lib, ctx, d_int, len(cs)) == cs and st.get()[0] == 0
    # the internal form is the Montgomery form in 29-bit limbs (textbook identity x*R mod N)
    R = 1 << (29 * nlw)
    internal = d_int.get()
    assert [sum(int(v) << (29 * i) for i, v in enumerate(row)) for row in internal] == [c * R % nsq for c in cs]
    d_sum = zeros(lib, (len(cs), nlw))
    assert lib.haflo_add(ctx, d_int.p, d_int.p, d_sum.p, len(cs), None) == 0
    assert export(lib, ctx, d_sum, len(cs)) == [c * c % nsq for c in cs]
    bad = [nsq, 3]
    assert lib.haflo_import_cipher(ctx, words(lib, bad, BITS // 16).p, d_int.p, st.p, 2, None) == 0
    assert export(lib, ctx, d_int, 2) == [0, 3] and st.get()[0] == 1


def test_encrypt_decrypt_scalar_mul(env):
    lib, ctx, sk, nlw = env
    pk = sk.public
    n = pk.n
    lp = BITS // 32
    rng = random.Random(2)
    ms = [rng.randrange(n) for _ in range(3)] + [0, 1, n - 1]
    rs = [rng.randrange(1, n) for _ in range(3)] + [1, n - 1, 2]
    d_c = zeros(lib, (len(ms), nlw))
    w, nb = ws(lib, ctx, _cabi.OP_ENCRYPT, len(ms))
    assert lib.haflo_encrypt(ctx, words(lib, ms, lp).p, words(lib, rs, lp).p, d_c.p, len(ms), w.p, nb, None) == 0
    want = [O.encrypt(pk, m, r) for m, r in zip(ms, rs)]
    assert export(lib, ctx, d_c, len(ms)) == want
    d_pl = zeros(lib, (len(ms), lp))
    w, nb = ws(lib, ctx, _cabi.OP_DECRYPT, len(ms))
    assert lib.haflo_decrypt(ctx, d_c.p, d_pl.p, len(ms), w.p, nb, None) == 0
    assert synth.words_to_ints(d_pl.get()) == ms
    # the same through the library's fixed scratch array, twice, the second call on fewer elements
    for count in (len(ms), 2):
        d_ps = zeros(lib, (count, lp))
        assert lib.haflo_decrypt_static(ctx, d_c.p, d_ps.p, count, None) == 0
        assert synth.words_to_ints(d_ps.get()) == ms[:count]
    assert lib.haflo_decrypt_static(ctx, d_c.p, d_pl.p, 10 ** 7, None) == -6
    ks = [rng.getrandbits(64) for _ in range(3)] + [0, 1, 2 ** 64 - 1]
    d_o = zeros(lib, (len(ms), nlw))
    w, nb = ws(lib, ctx, _cabi.OP_SCALAR_MUL, len(ms))
    assert lib.haflo_scalar_mul_u64(ctx, d_c.p, Dev(lib, np.array(ks, dtype=np.uint64)).p, d_o.p, len(ms), w.p, nb,
                                    None) == 0
    assert export(lib, ctx, d_o, len(ms)) == [pow(c, k, n * n) for c, k in zip(want, ks)]
    for k in (0, 1, 5, -1, -7, 2 ** 21, -(2 ** 40) + 3):
        assert lib.haflo_scalar_mul_i64_bcast(ctx, d_c.p, k, d_o.p, len(ms), w.p, nb, None) == 0
        assert export(lib, ctx, d_o, len(ms)) == [O.scalar_mul(pk, c, k) for c in want], k


def test_batch_above_the_wide_lane_threshold(env):
    """Small batches run the exponentiation engine with twice the lanes per integer; 20 elements
    exceed that threshold on the one-unit emulated chip, so this is the regular geometry (both
    encryption paths, decryption, scalar multiplication)."""
    lib, ctx, sk, nlw = env
    pk = sk.public
    n = pk.n
    lp = BITS // 32
    rng = random.Random(23)
    count = 20
    ms = [rng.randrange(n) for _ in range(count)]
    rs = [rng.randrange(1, n) for _ in range(count)]
    want = [O.encrypt(pk, m, r) for m, r in zip(ms, rs)]
    pub = C.c_void_p()
    buf = (C.c_uint8 * (BITS // 8)).from_buffer_copy(n.to_bytes(BITS // 8, "little"))
    assert lib.haflo_ctx_create_public(buf, BITS, C.byref(pub)) == 0
    for handle in (pub, ctx):
        d_c = zeros(lib, (count, nlw))
        w, nb = ws(lib, handle, _cabi.OP_ENCRYPT, count)
        assert lib.haflo_encrypt(handle, words(lib, ms, lp).p, words(lib, rs, lp).p, d_c.p, count, w.p, nb, None) == 0
        assert export(lib, handle, d_c, count) == want
    lib.haflo_ctx_destroy(pub)
    d_pl = zeros(lib, (count, lp))
    w, nb = ws(lib, ctx, _cabi.OP_DECRYPT, count)
    assert lib.haflo_decrypt(ctx, d_c.p, d_pl.p, count, w.p, nb, None) == 0
    assert synth.words_to_ints(d_pl.get()) == ms
    d_o = zeros(lib, (count, nlw))
    w, nb = ws(lib, ctx, _cabi.OP_SCALAR_MUL, count)
    assert lib.haflo_scalar_mul_i64_bcast(ctx, d_c.p, -5, d_o.p, count, w.p, nb, None) == 0
    assert export(lib, ctx, d_o, count) == [O.scalar_mul(pk, c, -5) for c in want]


def test_encrypt_with_obfuscator(env):
    lib, ctx, sk, nlw = env
    pk = sk.public
    lp = BITS // 32
    rng = random.Random(27)
    ms = [rng.randrange(pk.n) for _ in range(5)] + [0, pk.n - 1]
    rs = [rng.randrange(1, pk.n) for _ in range(len(ms))]
    d_obf = zeros(lib, (len(ms), nlw))
    w, nb = ws(lib, ctx, _cabi.OP_ENCRYPT, len(ms))
    zero = zeros(lib, (len(ms), lp))
    assert lib.haflo_encrypt(ctx, zero.p, words(lib, rs, lp).p, d_obf.p, len(ms), w.p, nb, None) == 0
    obf = [pow(r, pk.n, pk.nsq) for r in rs]
    assert export(lib, ctx, d_obf, len(ms)) == obf
    w, nb = ws(lib, ctx, _cabi.OP_ENCRYPT_OBFUSCATOR, len(ms))
    assert lib.haflo_encrypt_with_obfuscator(ctx, words(lib, ms, lp).p, d_obf.p, d_obf.p, len(ms), w.p, nb, None) == 0
    assert export(lib, ctx, d_obf, len(ms)) == [O.encrypt_with_obfuscator(pk, m, o) for m, o in zip(ms, obf)]
    assert export(lib, ctx, d_obf, len(ms)) == [O.encrypt(pk, m, r) for m, r in zip(ms, rs)]
    # with ciphertexts in place of the obfuscators the call adds plaintexts: D(out) = m + b mod n
    bs = [rng.randrange(pk.n) for _ in ms]
    d_sum = zeros(lib, (len(ms), nlw))
    assert lib.haflo_encrypt_with_obfuscator(ctx, words(lib, bs, lp).p, d_obf.p, d_sum.p, len(ms), w.p, nb, None) == 0
    want_sum = [O.add(pk, O.encrypt(pk, m, r), O.encrypt(pk, b, 1)) for m, r, b in zip(ms, rs, bs)]
    assert export(lib, ctx, d_sum, len(ms)) == want_sum
    assert [O.decrypt(sk, c) for c in want_sum] == [(m + b) % pk.n for m, b in zip(ms, bs)]


def test_public_context_encrypts_identically(env):
    """The public-key path (full exponent modulo n^2) and the key owner's path (through p^2 and
    q^2) must produce the same ciphertext bits; a public context cannot decrypt."""
    lib, ctx, sk, nlw = env
    pk = sk.public
    n = pk.n
    lp = BITS // 32
    pub = C.c_void_p()
    buf = (C.c_uint8 * (BITS // 8)).from_buffer_copy(n.to_bytes(BITS // 8, "little"))
    assert lib.haflo_ctx_create_public(buf, BITS, C.byref(pub)) == 0
    rng = random.Random(21)
    ms = [rng.randrange(n) for _ in range(3)] + [0, n - 1]
    rs = [rng.randrange(1, n) for _ in range(3)] + [n - 1, 1]
    want = [O.encrypt(pk, m, r) for m, r in zip(ms, rs)]
    for handle in (pub, ctx):
        d_c = zeros(lib, (len(ms), nlw))
        w, nb = ws(lib, handle, _cabi.OP_ENCRYPT, len(ms))
        assert lib.haflo_encrypt(handle, words(lib, ms, lp).p, words(lib, rs, lp).p, d_c.p, len(ms), w.p, nb,
                                 None) == 0
        assert export(lib, handle, d_c, len(ms)) == want
    mm, limbs = C.c_uint64(), C.c_uint32()
    assert lib.haflo_op_cost(pub, _cabi.OP_ENCRYPT, C.byref(mm), C.byref(limbs)) == 0
    assert 511 < mm.value < 768 and limbs.value == BITS // 16
    d_pl = zeros(lib, (len(ms), lp))
    assert lib.haflo_decrypt(pub, d_c.p, d_pl.p, len(ms), w.p, nb, None) == -3
    assert lib.haflo_workspace_bytes(pub, _cabi.OP_DECRYPT, 4, 0) == 2 ** 64 - 1
    lib.haflo_ctx_destroy(pub)


def test_matvec_sum(env):
    lib, ctx, sk, nlw = env
    pk = sk.public
    n = pk.n
    rng = random.Random(3)
    cs = [O.encrypt(pk, rng.randrange(n), rng.randrange(1, n)) for _ in range(7)]
    d_c = zeros(lib, (len(cs), nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, BITS // 16).p, d_c.p, None, len(cs), None) == 0
    npr = np.random.default_rng(5)
    X = npr.integers(-(1 << 19), 1 << 19, size=(7, 3)).astype(np.int32)
    X[0, 0], X[1, 1], X[2, 2] = 0, -1, -2 ** 31
    w, nb = ws(lib, ctx, _cabi.OP_MATVEC_XT_D, 7, 3)
    d_o = zeros(lib, (3, nlw))
    assert lib.haflo_cipher_matvec(ctx, 0, d_c.p, Dev(lib, X).p, 7, 3, d_o.p, w.p, nb, None) == 0
    assert export(lib, ctx, d_o, 3) == O.matvec(pk, 0, cs, X.tolist())
    Y = npr.integers(-(1 << 16), 1 << 16, size=(5, 7)).astype(np.int32)
    Y[npr.random(Y.shape) < 0.5] = 0
    Y[3, :] = 0
    w, nb = ws(lib, ctx, _cabi.OP_MATVEC_X_W, 5, 7)
    d_o = zeros(lib, (5, nlw))
    assert lib.haflo_cipher_matvec(ctx, 1, d_c.p, Dev(lib, Y).p, 5, 7, d_o.p, w.p, nb, None) == 0
    assert export(lib, ctx, d_o, 5) == O.matvec(pk, 1, cs, Y.tolist())
    w, nb = ws(lib, ctx, _cabi.OP_MATVEC_XT_D, 7, 1)
    d_s = zeros(lib, (1, nlw))
    assert lib.haflo_cipher_sum(ctx, d_c.p, 7, d_s.p, w.p, nb, None) == 0
    assert export(lib, ctx, d_s, 1) == [O.summation(pk, cs)]


@pytest.mark.parametrize("top", [15, 16, 17, 495, 496, 507375, 507376, 2 ** 31 - 1])
def test_matvec_signed_digit_boundaries(env, top):
    """Exponent magnitudes around the points where the signed base-32 recoding of
    orientation 0 needs one more digit position."""
    lib, ctx, sk, nlw = env
    pk = sk.public
    rng = random.Random(top)
    cs = [O.encrypt(pk, rng.randrange(pk.n), rng.randrange(1, pk.n)) for _ in range(4)]
    d_c = zeros(lib, (4, nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, BITS // 16).p, d_c.p, None, 4, None) == 0
    X = np.array([[top, -top], [top - 1, 1], [-(top // 2), top // 3], [16, -17]], dtype=np.int64).astype(np.int32)
    w, nb = ws(lib, ctx, _cabi.OP_MATVEC_XT_D, 4, 2)
    d_o = zeros(lib, (2, nlw))
    assert lib.haflo_cipher_matvec(ctx, 0, d_c.p, Dev(lib, X).p, 4, 2, d_o.p, w.p, nb, None) == 0
    assert export(lib, ctx, d_o, 2) == O.matvec(pk, 0, cs, X.tolist())


@pytest.fixture
def force_buckets(env):
    lib, ctx = env[0], env[1]
    assert lib.haflo_ctx_set_xtd_bucket_min_rows(ctx, 1) == 0
    yield
    assert lib.haflo_ctx_set_xtd_bucket_min_rows(ctx, 0) == 0


def _xtd_case(env, X, seed):
    lib, ctx, sk, nlw = env
    pk = sk.public
    rows, cols = X.shape
    rng = random.Random(seed)
    cs = [O.encrypt(pk, rng.randrange(pk.n), rng.randrange(1, pk.n)) for _ in range(rows)]
    d_c = zeros(lib, (rows, nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, BITS // 16).p, d_c.p, None, rows, None) == 0
    w, nb = ws(lib, ctx, _cabi.OP_MATVEC_XT_D, rows, cols)
    d_o = zeros(lib, (cols, nlw))
    assert lib.haflo_cipher_matvec(ctx, 0, d_c.p, Dev(lib, X).p, rows, cols, d_o.p, w.p, nb, None) == 0
    assert export(lib, ctx, d_o, cols) == O.matvec(pk, 0, cs, X.tolist())


def test_bucket_matvec_random(env, force_buckets):
    """Bucket method on a small matrix: mixed signs, zeros, the most negative exponent."""
    npr = np.random.default_rng(11)
    X = npr.integers(-(1 << 19), 1 << 19, size=(37, 3)).astype(np.int32)
    X[npr.random(X.shape) < 0.2] = 0
    X[1, 1], X[2, 2], X[3, 0] = -1, -2 ** 31, 2 ** 31 - 1
    _xtd_case(env, X, 21)


def test_bucket_matvec_long_chunks(env, force_buckets):
    """A matrix tall enough for the one-unit emulated chip to switch to chunks of 32 items (from 49152
    exponent digits on): few magnitudes, so that buckets hold thousands of rows and three rounds run,
    two of them with their chunks handed out by length. The ciphertexts are random units modulo n^2."""
    lib, ctx, sk, nlw = env
    pk = sk.public
    rows, cols = 12500, 2
    rng = random.Random(5)
    cs = [rng.randrange(2, pk.nsq) for _ in range(rows)]
    npr = np.random.default_rng(12)
    X = npr.choice(np.array([1025, -1025, 3 * 1024 + 7, -(2 * 1024 + 7), 5 * 1024 - 3], dtype=np.int32), size=(rows, cols))
    X[::500, 1] = 0
    d_c = zeros(lib, (rows, nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, BITS // 16).p, d_c.p, None, rows, None) == 0
    w, nb = ws(lib, ctx, _cabi.OP_MATVEC_XT_D, rows, cols)
    d_o = zeros(lib, (cols, nlw))
    assert lib.haflo_cipher_matvec(ctx, 0, d_c.p, Dev(lib, X).p, rows, cols, d_o.p, w.p, nb, None) == 0
    assert export(lib, ctx, d_o, cols) == O.matvec(pk, 0, cs, X.tolist())


def test_bucket_matvec_heavy_buckets(env, force_buckets):
    """Columns of equal entries put every row into one bucket, which then takes several
    reduction rounds (37 rows > 32 items per chunk); a zero column gives the encryption-free one."""
    X = np.zeros((37, 4), dtype=np.int32)
    X[:, 0] = 1 << 16
    X[:, 1] = -3
    X[::2, 3] = 1023
    X[1::2, 3] = -1025
    _xtd_case(env, X, 22)


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("method", [1, 2 ** 64 - 1])
def test_gradient_matvec_random_shapes(env, seed, method):
    """Random shapes and exponent distributions through both gradient-matvec methods (the
    context's row threshold forces either): sparse, dense, one magnitude only, full int32
    range, powers of 1024 and their neighbours."""
    lib, ctx = env[0], env[1]
    assert lib.haflo_ctx_set_xtd_bucket_min_rows(ctx, method) == 0
    try:
        _gradient_matvec_random_shape(env, seed)
    finally:
        assert lib.haflo_ctx_set_xtd_bucket_min_rows(ctx, 0) == 0


def _gradient_matvec_random_shape(env, seed):
    rng = np.random.default_rng(1000 + seed)
    rows, cols = int(rng.integers(1, 45)), int(rng.integers(1, 4))
    kind = seed % 6
    if kind == 0:
        X = rng.integers(-2 ** 31, 2 ** 31, size=(rows, cols), dtype=np.int64)
    elif kind == 1:
        X = rng.integers(-3, 4, size=(rows, cols), dtype=np.int64)
    elif kind == 2:
        X = np.full((rows, cols), -(1 << 20), dtype=np.int64)
    elif kind == 3:
        X = rng.choice(np.array([0, 1, -1, 1023, 1024, 1025, -1024 ** 2, 1024 ** 2 + 511, 1024 ** 3 - 512, -1024 ** 3]),
                       size=(rows, cols))
    elif kind == 4:
        X = rng.integers(-(1 << 19), 1 << 19, size=(rows, cols), dtype=np.int64)
        X[rng.random(X.shape) < 0.8] = 0
    else:
        X = (rng.normal(0, 1, (rows, cols)) * 65536).round().astype(np.int64)
    _xtd_case(env, X.astype(np.int32), 2000 + seed)


@pytest.mark.parametrize("top", [511, 512, 513, 523775, 523776, 535821823, 535821824])
def test_bucket_matvec_digit_boundaries(env, force_buckets, top):
    """Magnitudes around the points where the signed base-1024 recoding needs one more position."""
    X = np.array([[top, -top], [top - 1, 1], [-(top // 2), top // 3], [512, -513]], dtype=np.int64).astype(np.int32)
    _xtd_case(env, X, top)


@pytest.mark.parametrize("bits", [1024, 2048, 4096])
def test_wider_lane_groups(emu, bits):
    """The 4-, 8- and 16-lane geometries (1024/2048/4096-bit keys) on a few elements: Montgomery
    form and addition in the modulus's own lanes; the inverse and a short power, which a batch this
    small runs with one integer per wavefront (single residues at 1024 bits, pairs from 2048 bits on,
    with the accumulators of the 2- and 3-limb lanes held at 8 times their value)."""
    lib = emu
    p, q = oracle_key(bits)
    sk = O.PrivateKey(p, q)
    pk = sk.public
    nsq = pk.nsq
    ctx = C.c_void_p()
    buf = (C.c_uint8 * (bits // 8)).from_buffer_copy(pk.n.to_bytes(bits // 8, "little"))
    assert lib.haflo_ctx_create_public(buf, bits, C.byref(ctx)) == 0
    cb = C.c_size_t()
    lib.haflo_ctx_info(ctx, None, None, None, C.byref(cb), None)
    nlw = cb.value // 4
    assert nlw == bits * 9 // 128
    rng = random.Random(bits)
    cs = [rng.randrange(1, nsq) for _ in range(2)] + [nsq - 1]
    lc = bits // 16

    def exp_(d, count):
        out = zeros(lib, (count, lc))
        assert lib.haflo_export_cipher(ctx, d.p, out.p, count, None) == 0
        return synth.words_to_ints(out.get())

    d_c = zeros(lib, (len(cs), nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, lc).p, d_c.p, None, len(cs), None) == 0
    R = 1 << (29 * nlw)
    assert [sum(int(v) << (29 * i) for i, v in enumerate(row)) for row in d_c.get()] == [c * R % nsq for c in cs]
    assert exp_(d_c, len(cs)) == cs
    d_o = zeros(lib, (len(cs), nlw))
    assert lib.haflo_add(ctx, d_c.p, d_c.p, d_o.p, len(cs), None) == 0
    assert exp_(d_o, len(cs)) == [c * c % nsq for c in cs]
    w, nb = ws(lib, ctx, _cabi.OP_SCALAR_MUL, len(cs))
    assert lib.haflo_scalar_mul_i64_bcast(ctx, d_c.p, -3, d_o.p, len(cs), w.p, nb, None) == 0
    assert exp_(d_o, len(cs)) == [pow(pow(c, -1, nsq), 3, nsq) for c in cs]
    lib.haflo_ctx_destroy(ctx)


@pytest.mark.parametrize("bits,count", [
    (1024, 1),
    # the pair engine with one pair per wavefront (36 lanes, 2 limbs of each half): a minute and a half emulated
    pytest.param(2048, 1, marks=pytest.mark.skipif(not os.environ.get("HAFLO_SLOW_TESTS"),
                                                   reason="slow: set HAFLO_SLOW_TESTS=1")),
])
def test_whole_wavefront_groups_encrypt_decrypt(emu, bits, count):
    """Batches of at most one element per SIMD give every big integer a wavefront to itself (18 to 48
    lanes with 2 or 3 limbs each, neighbour exchange across DPP rows, the quotient digit through a
    scalar register): the full encryption program with the public key, the key owner's two-stage
    route and the decryption through p^2 and q^2, against the oracle."""
    lib = emu
    p, q = oracle_key(bits)
    sk = O.PrivateKey(p, q)
    pk = sk.public
    n = pk.n
    lp, lc = bits // 32, bits // 16

    def le(x, nbytes):
        return (C.c_uint8 * nbytes).from_buffer_copy(x.to_bytes(nbytes, "little"))

    own, pub = C.c_void_p(), C.c_void_p()
    assert lib.haflo_ctx_create_private(le(p, bits // 16), le(q, bits // 16), bits, C.byref(own)) == 0
    assert lib.haflo_ctx_create_public(le(n, bits // 8), bits, C.byref(pub)) == 0
    cb = C.c_size_t()
    lib.haflo_ctx_info(own, None, None, None, C.byref(cb), None)
    nlw = cb.value // 4
    rng = random.Random(bits + 1)
    ms = [rng.randrange(n) for _ in range(count)]
    ms[0] = n - 1
    rs = [rng.randrange(1, n) for _ in range(count)]
    want = [O.encrypt(pk, m, r) for m, r in zip(ms, rs)]
    lc_out = zeros(lib, (count, lc))
    for ctx in (pub, own):
        d_c = zeros(lib, (count, nlw))
        w, nb = ws(lib, ctx, _cabi.OP_ENCRYPT, count)
        assert lib.haflo_encrypt(ctx, words(lib, ms, lp).p, words(lib, rs, lp).p, d_c.p, count, w.p, nb, None) == 0
        assert lib.haflo_export_cipher(ctx, d_c.p, lc_out.p, count, None) == 0
        assert synth.words_to_ints(lc_out.get()) == want
    d_pl = zeros(lib, (count, lp))
    w, nb = ws(lib, own, _cabi.OP_DECRYPT, count)
    assert lib.haflo_decrypt(own, d_c.p, d_pl.p, count, w.p, nb, None) == 0
    assert synth.words_to_ints(d_pl.get()) == ms
    lib.haflo_ctx_destroy(own)
    lib.haflo_ctx_destroy(pub)


def test_pair_arithmetic_on_batches_that_fill_the_chip(env):
    """Batches beyond what the wide geometries take (more than 128 integers of two lanes, or 256 of one
    lane, on the one-unit emulated chip) run the exponentiations on pairs of half-length residues: the
    public-key encryption, the key owner's second stage, both decryption branches and the ciphertext
    powers (with their conversion into and out of the pair form), all against the oracle."""
    lib, ctx, sk, nlw = env
    pk = sk.public
    n, nsq = pk.n, pk.nsq
    lp, lc = BITS // 32, BITS // 16
    rng = random.Random(29)
    count = 270
    ms = [rng.randrange(n) for _ in range(count)]
    ms[:3] = [n - 1, 0, 1]
    rs = [rng.randrange(1, n) for _ in range(count)]
    want = [O.encrypt(pk, m, r) for m, r in zip(ms, rs)]
    pub = C.c_void_p()
    buf = (C.c_uint8 * (BITS // 8)).from_buffer_copy(n.to_bytes(BITS // 8, "little"))
    assert lib.haflo_ctx_create_public(buf, BITS, C.byref(pub)) == 0
    d_m, d_r = words(lib, ms, lp), words(lib, rs, lp)
    # the key owner's route on all 270, the public route on the first 140 (slower in the emulation)
    d_c = zeros(lib, (count, nlw))
    w, nb = ws(lib, ctx, _cabi.OP_ENCRYPT, count)
    assert lib.haflo_encrypt(ctx, d_m.p, d_r.p, d_c.p, count, w.p, nb, None) == 0
    assert export(lib, ctx, d_c, count) == want
    sub = 140
    d_cp = zeros(lib, (sub, nlw))
    w, nb = ws(lib, pub, _cabi.OP_ENCRYPT, sub)
    assert lib.haflo_encrypt(pub, d_m.p, d_r.p, d_cp.p, sub, w.p, nb, None) == 0
    assert export(lib, pub, d_cp, sub) == want[:sub]
    d_pl = zeros(lib, (count, lp))
    w, nb = ws(lib, ctx, _cabi.OP_DECRYPT, count)
    assert lib.haflo_decrypt(ctx, d_c.p, d_pl.p, count, w.p, nb, None) == 0
    assert synth.words_to_ints(d_pl.get()) == ms
    d_o = zeros(lib, (sub, nlw))
    w, nb = ws(lib, pub, _cabi.OP_SCALAR_MUL, sub)
    for k in (-5, 0, 2 ** 21):
        assert lib.haflo_scalar_mul_i64_bcast(pub, d_cp.p, k, d_o.p, sub, w.p, nb, None) == 0
        assert export(lib, pub, d_o, sub) == [O.scalar_mul(pk, c, k) for c in want[:sub]]
    ks = [rng.getrandbits(64) for _ in range(sub)]
    ks[:2] = [0, 2 ** 64 - 1]
    assert lib.haflo_scalar_mul_u64(pub, d_cp.p, Dev(lib, np.array(ks, dtype=np.uint64)).p, d_o.p, sub, w.p, nb, None) == 0
    assert export(lib, pub, d_o, sub) == [pow(c, k, nsq) for c, k in zip(want[:sub], ks)]
    lib.haflo_ctx_destroy(pub)


def test_bucket_matvec_four_lane_groups(emu, force_buckets):
    """The bucket method with 4 lanes per integer (1024-bit key), where several groups share a
    wave and chunks of different length keep them in lock step."""
    lib, bits = emu, 1024
    p, q = oracle_key(bits)
    pk = O.PrivateKey(p, q).public
    ctx = C.c_void_p()
    buf = (C.c_uint8 * (bits // 8)).from_buffer_copy(pk.n.to_bytes(bits // 8, "little"))
    assert lib.haflo_ctx_create_public(buf, bits, C.byref(ctx)) == 0
    nlw, lc = bits * 9 // 128, bits // 16
    rows, cols = 21, 2
    rng = random.Random(77)
    cs = [rng.randrange(1, pk.nsq) for _ in range(rows)]
    npr = np.random.default_rng(78)
    X = npr.integers(-(1 << 18), 1 << 18, size=(rows, cols)).astype(np.int32)
    X[:, 1] = np.where(np.arange(rows) % 3 == 0, 0, 5)
    d_c = zeros(lib, (rows, nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, lc).p, d_c.p, None, rows, None) == 0
    w, nb = ws(lib, ctx, _cabi.OP_MATVEC_XT_D, rows, cols)
    d_o = zeros(lib, (cols, nlw))
    assert lib.haflo_cipher_matvec(ctx, 0, d_c.p, Dev(lib, X).p, rows, cols, d_o.p, w.p, nb, None) == 0
    out = zeros(lib, (cols, lc))
    assert lib.haflo_export_cipher(ctx, d_o.p, out.p, cols, None) == 0
    assert synth.words_to_ints(out.get()) == O.matvec(pk, 0, cs, X.tolist())
    lib.haflo_ctx_destroy(ctx)


def test_fore_gradient(env):
    lib, ctx, sk, nlw = env
    pk = sk.public
    lp = BITS // 32
    rng = random.Random(31)
    ug = np.concatenate([synth.normal_f32(9, 2.0, 32), np.array([np.nan, 1.0, -3.5], dtype=np.float32)])
    y = np.concatenate([np.array([1, -1, 0, 1, 1, -1, 0, 1, -1, 1], dtype=np.float32),
                        np.array([2.0 ** 38, -(2.0 ** 37)], dtype=np.float32)])
    count = len(ug)
    c_host = [O.encrypt(pk, rng.randrange(pk.n), rng.randrange(1, pk.n)) for _ in range(count)]
    rs = [rng.randrange(1, pk.n) for _ in range(count)]
    d_c = zeros(lib, (count, nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, c_host, BITS // 16).p, d_c.p, None, count, None) == 0
    w, nb = ws(lib, ctx, _cabi.OP_FORE_GRADIENT, count)
    d_o, d_st = zeros(lib, (count, nlw)), zeros(lib, (count,))
    assert lib.haflo_fore_gradient(ctx, d_c.p, Dev(lib, ug).p, Dev(lib, y).p, words(lib, rs, lp).p, 24, d_o.p, d_st.p,
                                   count, w.p, nb, None) == 0
    want = [O.fore_gradient(pk, c_host[i], float(ug[i]), float(y[i]), rs[i], 24) for i in range(count)]
    assert export(lib, ctx, d_o, count) == [c for c, _ in want]
    assert d_st.get().tolist() == [st for _, st in want] and sum(st for _, st in want) == 3
    assert lib.haflo_fore_gradient(ctx, d_c.p, Dev(lib, ug).p, Dev(lib, y).p, words(lib, rs, lp).p, 24, d_o.p, None,
                                   count, w.p, nb - 1, None) == -1


def test_taylor_loss(env):
    lib, ctx, sk, nlw = env
    pk = sk.public
    lp = BITS // 32
    rng = random.Random(41)
    s = 20
    for count, bad in ((9, False), (9, True), (0, False)):
        ug = synth.normal_f32(count, 1.5, 42)
        y = np.where(np.arange(count) % 2 == 0, 1.0, -1.0).astype(np.float32)
        if bad:
            ug[3], y[4] = np.nan, 200.0
        m1 = [O.quantise(float(v), s) for v in synth.normal_f32(count, 1.5, 43)]
        c_u = [O.encrypt(pk, m % pk.n, rng.randrange(1, pk.n)) for m in m1]
        c_u2 = [O.encrypt(pk, m * m, rng.randrange(1, pk.n)) for m in m1]
        r = rng.randrange(1, pk.n)
        d_u, d_u2 = zeros(lib, (max(count, 1), nlw)), zeros(lib, (max(count, 1), nlw))
        if count:
            assert lib.haflo_import_cipher(ctx, words(lib, c_u, BITS // 16).p, d_u.p, None, count, None) == 0
            assert lib.haflo_import_cipher(ctx, words(lib, c_u2, BITS // 16).p, d_u2.p, None, count, None) == 0
        w, nb = ws(lib, ctx, _cabi.OP_TAYLOR_LOSS, count)
        d_o, d_st = zeros(lib, (1, nlw)), zeros(lib, (1,))
        assert lib.haflo_taylor_loss(ctx, d_u.p, d_u2.p, Dev(lib, ug).p, Dev(lib, y).p, words(lib, [r], lp).p, s,
                                     d_o.p, d_st.p, count, w.p, nb, None) == 0
        want, st = O.taylor_loss(pk, c_u, c_u2, [float(v) for v in ug], [float(v) for v in y], r, s)
        assert export(lib, ctx, d_o, 1) == [want]
        assert d_st.get().tolist() == [st] and st == (1 if bad else 0)
        # no r: the plaintext part enters as g^P, which is the encryption with r = 1
        assert lib.haflo_taylor_loss(ctx, d_u.p, d_u2.p, Dev(lib, ug).p, Dev(lib, y).p, None, s, d_o.p, None, count,
                                     w.p, nb, None) == 0
        assert export(lib, ctx, d_o, 1) == [O.taylor_loss(pk, c_u, c_u2, [float(v) for v in ug],
                                                          [float(v) for v in y], 1, s)[0]]
    assert lib.haflo_taylor_loss(ctx, d_u.p, d_u2.p, None, None, words(lib, [r], lp).p, 28, d_o.p, None, 0, w.p, nb,
                                 None) == -1


def test_host_staging_roundtrip(env):
    """Chunked staging between host arrays and device arrays: chunk boundaries (count not a multiple
    of the chunk, count below one chunk, zero), reuse of page-locked buffers, the range flag."""
    lib, ctx, sk, nlw = env
    pk = sk.public
    lc, lp = BITS // 16, BITS // 32
    st = C.c_void_p()
    assert lib.haflo_stager_create(ctx, 4, 1 << 20, C.byref(st)) == 0
    rng = random.Random(51)
    for count in (11, 3, 0, 8):
        cs = [rng.randrange(pk.nsq) for _ in range(count)]
        h_in = np.ascontiguousarray(synth.ints_to_words(cs, lc)) if count else np.zeros((0, lc), np.uint32)
        d_c = zeros(lib, (max(count, 1), nlw))
        d_st = zeros(lib, (1,))
        assert lib.haflo_stage_in_cipher(st, h_in.ctypes.data, d_c.p, d_st.p, count, None) == 0
        assert d_st.get().tolist() == [0]
        if count:
            assert export(lib, ctx, d_c, count) == cs
        h_out = np.zeros((max(count, 1), lc), np.uint32)
        assert lib.haflo_stage_out_cipher(st, d_c.p, h_out.ctypes.data, count, None) == 0
        assert synth.words_to_ints(h_out[:count]) == cs
        ms = [rng.randrange(pk.n) for _ in range(count)]
        h_pl = np.ascontiguousarray(synth.ints_to_words(ms, lp)) if count else np.zeros((0, lp), np.uint32)
        d_pl = zeros(lib, (max(count, 1), lp))
        assert lib.haflo_stage_in_plain(st, h_pl.ctypes.data, d_pl.p, count, None) == 0
        h_back = np.zeros((max(count, 1), lp), np.uint32)
        assert lib.haflo_stage_out_plain(st, d_pl.p, h_back.ctypes.data, count, None) == 0
        assert synth.words_to_ints(h_back[:count]) == ms
    bad = np.ascontiguousarray(synth.ints_to_words([5, pk.nsq, 7, 8, 9], lc))
    d_c, d_st = zeros(lib, (5, nlw)), zeros(lib, (1,))
    assert lib.haflo_stage_in_cipher(st, bad.ctypes.data, d_c.p, d_st.p, 5, None) == 0
    assert d_st.get().tolist() == [1] and export(lib, ctx, d_c, 5) == [5, 0, 7, 8, 9]
    pb, pa, pr = C.c_size_t(), C.c_size_t(), C.c_size_t()
    assert lib.haflo_stager_stats(st, C.byref(pb), C.byref(pa), C.byref(pr)) == 0
    assert pa.value <= 4 and pr.value > pa.value and pb.value <= 1 << 20
    assert lib.haflo_stage_in_cipher(st, None, d_c.p, None, 5, None) == -1
    assert lib.haflo_stager_destroy(st) == 0
    assert lib.haflo_stager_create(ctx, 0, 0, C.byref(st)) == -1


def test_summation_levels(env):
    """Enough elements for two first-level blocks on the one-unit emulated chip, so that the
    second (wide-geometry) level runs."""
    lib, ctx, sk, nlw = env
    pk = sk.public
    rng = random.Random(71)
    count = 600
    cs = [rng.randrange(1, pk.nsq) for _ in range(count)]
    d_c = zeros(lib, (count, nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, BITS // 16).p, d_c.p, None, count, None) == 0
    w, nb = ws(lib, ctx, _cabi.OP_MATVEC_XT_D, count, 1)
    d_s = zeros(lib, (1, nlw))
    assert lib.haflo_cipher_sum(ctx, d_c.p, count, d_s.p, w.p, nb, None) == 0
    assert export(lib, ctx, d_s, 1) == [O.summation(pk, cs)]
    assert lib.haflo_cipher_sum(ctx, d_c.p, count, d_s.p, w.p, 64, None) == -1


@pytest.mark.parametrize("offsets", [
    [0, 0, 1, 1, 9, 20, 20, 300, 337],        # empty segments, single elements, three reduction rounds (280 > 16^2)
    [0, 337],                                  # one segment over everything
    [5, 5],                                    # one empty segment
    [3, 20, 36, 37, 337],                      # first element not at 0; lengths 17 (two chunks) and 16 (one)
    list(range(0, 338)),                       # every element its own segment
])
def test_summation_segments(env, offsets):
    lib, ctx, sk, nlw = env
    pk = sk.public
    rng = random.Random(73)
    count = 337
    cs = [rng.randrange(1, pk.nsq) for _ in range(count)]
    d_c = zeros(lib, (count, nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, BITS // 16).p, d_c.p, None, count, None) == 0
    nseg = len(offsets) - 1
    w, nb = ws(lib, ctx, _cabi.OP_SUM_SEGMENTS, count, nseg)
    d_s, st = zeros(lib, (nseg, nlw)), zeros(lib, (1,))
    d_off = Dev(lib, np.array(offsets, dtype=np.uint32))
    assert lib.haflo_cipher_sum_segments(ctx, d_c.p, count, d_off.p, nseg, d_s.p, st.p, w.p, nb, None) == 0
    assert export(lib, ctx, d_s, nseg) == O.summation_segments(pk, cs, offsets)
    assert st.get()[0] == 0


def test_summation_segments_long_chunks(env):
    """An array long enough for the one-unit emulated chip to take chunks of 32 elements (from 49152
    elements on): one slice of 40000 elements (four rounds), a short one, an empty one and the rest."""
    lib, ctx, sk, nlw = env
    pk = sk.public
    rng = random.Random(79)
    count = 49500
    cs = [rng.randrange(1, pk.nsq) for _ in range(count)]
    d_c = zeros(lib, (count, nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, BITS // 16).p, d_c.p, None, count, None) == 0
    offsets = [0, 40000, 40033, 40033, count]
    nseg = len(offsets) - 1
    w, nb = ws(lib, ctx, _cabi.OP_SUM_SEGMENTS, count, nseg)
    d_s, st = zeros(lib, (nseg, nlw)), zeros(lib, (1,))
    d_off = Dev(lib, np.array(offsets, dtype=np.uint32))
    assert lib.haflo_cipher_sum_segments(ctx, d_c.p, count, d_off.p, nseg, d_s.p, st.p, w.p, nb, None) == 0
    assert export(lib, ctx, d_s, nseg) == O.summation_segments(pk, cs, offsets)
    assert st.get()[0] == 0


def test_summation_segments_bad_offsets_and_arguments(env):
    """Offsets that run backwards or past the array are clipped and flagged; nothing outside the
    array is read (the emulated buffers end at a guard page)."""
    lib, ctx, sk, nlw = env
    pk = sk.public
    rng = random.Random(74)
    count = 40
    cs = [rng.randrange(1, pk.nsq) for _ in range(count)]
    d_c = zeros(lib, (count, nlw))
    assert lib.haflo_import_cipher(ctx, words(lib, cs, BITS // 16).p, d_c.p, None, count, None) == 0
    offsets = [0, 10, 5, 30, 2 ** 32 - 1]
    nseg = len(offsets) - 1
    w, nb = ws(lib, ctx, _cabi.OP_SUM_SEGMENTS, count, nseg)
    d_s, st = zeros(lib, (nseg, nlw)), zeros(lib, (1,))
    d_off = Dev(lib, np.array(offsets, dtype=np.uint32))
    assert lib.haflo_cipher_sum_segments(ctx, d_c.p, count, d_off.p, nseg, d_s.p, st.p, w.p, nb, None) == 0
    assert export(lib, ctx, d_s, nseg) == [O.summation(pk, cs[0:10]), 1, O.summation(pk, cs[5:30]), O.summation(pk, cs[30:40])]
    assert st.get()[0] == 1
    assert lib.haflo_cipher_sum_segments(ctx, d_c.p, count, d_off.p, nseg, d_s.p, st.p, w.p, nb - 4, None) == -1
    assert lib.haflo_cipher_sum_segments(ctx, d_c.p, count, None, nseg, d_s.p, st.p, w.p, nb, None) == -1
    assert lib.haflo_cipher_sum_segments(ctx, d_c.p, 2 ** 32, d_off.p, nseg, d_s.p, st.p, w.p, nb, None) == -1
    assert lib.haflo_cipher_sum_segments(ctx, d_c.p, count, d_off.p, 0, None, None, None, 0, None) == 0


def test_encode_decode(env):
    lib, ctx, sk, nlw = env
    pk = sk.public
    n = pk.n
    lp = BITS // 32
    vals = np.concatenate([np.array([0.0, 1.0, -1.0, 0.5, -0.25, np.inf, np.nan, 1e30, -1e30, 1.5 * 2.0 ** -24,
                                     2.5 * 2.0 ** -24, -3.4e38], dtype=np.float32), synth.normal_f32(300, 0.25, 9)])
    d_pl, d_st = zeros(lib, (len(vals), lp)), zeros(lib, (len(vals),))
    assert lib.haflo_encode_f32(ctx, Dev(lib, vals).p, 24, d_pl.p, d_st.p, len(vals), None) == 0
    want = [O.encode(pk, float(v), 24) for v in vals]
    assert list(zip(synth.words_to_ints(d_pl.get()), d_st.get().tolist())) == want
    d_q, d_v = zeros(lib, (len(vals),), np.int64), zeros(lib, (len(vals),), np.float64)
    assert lib.haflo_decode(ctx, d_pl.p, 24, d_q.p, d_v.p, d_st.p, len(vals), None) == 0
    assert list(zip(d_q.get().tolist(), d_v.get().tolist(), d_st.get().tolist())) == [O.decode(pk, m, 24)
                                                                                     for m, _ in want]
    edge = [n // 2, n // 2 + 1, 2 ** 63 - 1, 2 ** 63, n - 2 ** 63, n - 2 ** 63 - 1, n - 1, 0, 1 << 64, n - (1 << 64)]
    d_q, d_v, d_st = zeros(lib, (len(edge),), np.int64), zeros(lib, (len(edge),), np.float64), zeros(lib, (len(edge),))
    assert lib.haflo_decode(ctx, words(lib, edge, lp).p, 40, d_q.p, d_v.p, d_st.p, len(edge), None) == 0
    assert list(zip(d_q.get().tolist(), d_v.get().tolist(), d_st.get().tolist())) == [O.decode(pk, m, 40) for m in edge]
    d_e, d_st = zeros(lib, (len(vals),), np.int32), zeros(lib, (len(vals),))
    assert lib.haflo_encode_exponents_f32(Dev(lib, vals).p, 16, d_e.p, d_st.p, len(vals), None) == 0
    assert list(zip(d_e.get().tolist(), d_st.get().tolist())) == [O.encode_exponent(float(v), 16) for v in vals]


def test_op_cost_and_workspace_queries(env):
    lib, ctx, sk, nlw = env
    mm, limbs = C.c_uint64(), C.c_uint32()
    assert lib.haflo_op_cost(ctx, _cabi.OP_ENCRYPT, C.byref(mm), C.byref(limbs)) == 0
    # key owner: per branch a ~256-bit exponent on the half-size modulus and one on the quarter-size
    # modulus (a product there counts (2*8^2+8)/(2*16^2+16) = 0.258 of a half-size one); each
    # exponent needs at least one squaring per bit and fewer than 1.5 products per bit
    assert 2 * 250 * 1.258 < mm.value < 2 * 384 * 1.258 + 30 and limbs.value == BITS // 32
    assert lib.haflo_op_cost(ctx, 99, None, None) == -1
    assert lib.haflo_workspace_bytes(ctx, 99, 1, 1) == 2 ** 64 - 1
    assert lib.haflo_encrypt(ctx, None, None, None, 4, None, 0, None) == -1
    small = zeros(lib, (4,))
    d = zeros(lib, (1, nlw))
    assert lib.haflo_encrypt(ctx, small.p, small.p, d.p, 1, small.p, 16, None) == -1  # workspace too small
