"""The library's host-side big integers (key generation, per-key constants) against Python
integers, through a small C wrapper compiled with g++ (no GPU, no HIP)."""
import ctypes as C
import os
import random
import subprocess

import pytest

HERE = os.path.dirname(os.path.abspath(__file__))
OPS = {name: i for i, name in enumerate(
    ["add", "sub", "mul", "mod", "gcd", "powmod", "inv_pow2", "shl1", "shr1", "low_bits", "montmul", "div"])}


@pytest.fixture(scope="module")
def shim(tmp_path_factory):
    out = str(tmp_path_factory.mktemp("hostbig") / "libhostbig_shim.so")
    opt = ["-O2"]
    if os.environ.get("HAFLO_EMU_SANITIZE", "") == "1":  # see tests/test_sanitizers.py
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
    subprocess.run(["g++"] + opt + ["-std=c++17", "-shared", "-fPIC", "-o", out, os.path.join(HERE, "hostbig_shim.cpp")],
                   check=True)
    lib = C.CDLL(out)
    lib.hostbig_op.restype = C.c_long
    lib.hostbig_op.argtypes = [C.c_int, C.c_char_p, C.c_size_t, C.c_char_p, C.c_size_t, C.c_char_p, C.c_size_t,
                               C.c_uint64, C.c_char_p, C.c_size_t]
    lib.hostbig_neg_inv32.restype = C.c_uint32
    lib.hostbig_neg_inv32.argtypes = [C.c_uint32]
    lib.hostbig_mod_small.restype = C.c_uint32
    lib.hostbig_mod_small.argtypes = [C.c_char_p, C.c_size_t, C.c_uint32]
    lib.hostbig_cmp.argtypes = [C.c_char_p, C.c_size_t, C.c_char_p, C.c_size_t]
    lib.hostbig_extract.restype = C.c_uint32
    lib.hostbig_extract.argtypes = [C.c_char_p, C.c_size_t, C.c_uint64, C.c_uint]
    return lib


def _b(x):
    return x.to_bytes(max(1, (x.bit_length() + 7) // 8), "little")


def call(lib, op, a=0, b=0, c=0, k=0, nout=1100):
    out = C.create_string_buffer(nout)
    ba, bb, bc = _b(a), _b(b), _b(c)
    bits = lib.hostbig_op(OPS[op], ba, len(ba), bb, len(bb), bc, len(bc), k, out, nout)
    val = int.from_bytes(out.raw, "little")
    assert bits == val.bit_length()
    return val


def operands(rng, bits):
    edge = [0, 1, 2, (1 << 32) - 1, 1 << 32, (1 << 64) - 1, (1 << bits) - 1, 1 << (bits - 1)]
    return edge + [rng.getrandbits(rng.choice((1, 31, 32, 33, 64, 100, bits // 2, bits))) for _ in range(30)]


@pytest.mark.parametrize("bits", [96, 1024, 4096])
def test_ring_operations(shim, bits):
    rng = random.Random(bits)
    xs = operands(rng, bits)
    for _ in range(150):
        a, b = rng.choice(xs), rng.choice(xs)
        assert call(shim, "add", a, b) == a + b
        assert call(shim, "mul", a, b) == a * b
        if b:
            assert call(shim, "div", a, b) == a // b and call(shim, "mod", a, b) == a % b
            assert call(shim, "div", a * b + b - 1, b) == a
        hi, lo = max(a, b), min(a, b)
        assert call(shim, "sub", hi, lo) == hi - lo
        assert shim.hostbig_cmp(_b(a), len(_b(a)), _b(b), len(_b(b))) == (a > b) - (a < b)
        assert call(shim, "shl1", a) == a << 1 and call(shim, "shr1", a) == a >> 1
        k = rng.choice((1, 5, 32, 33, 64, bits // 3 + 1))
        assert call(shim, "low_bits", a, k=k) == a & ((1 << k) - 1)
        if b:
            assert call(shim, "mod", a, b) == a % b
        d = rng.choice((3, 5, 1999, 2 ** 31 - 1, 2 ** 32 - 5))
        assert shim.hostbig_mod_small(_b(a), len(_b(a)), d) == a % d
        pos, ln = rng.randrange(bits), rng.choice((1, 5, 29, 32))
        assert shim.hostbig_extract(_b(a), len(_b(a)), pos, ln) == (a >> pos) & ((1 << ln) - 1)


def test_gcd(shim):
    import math
    rng = random.Random(7)
    for _ in range(60):
        g = rng.getrandbits(rng.choice((1, 20, 64)))
        a, b = g * rng.getrandbits(200), g * rng.getrandbits(150)
        assert call(shim, "gcd", a, b) == math.gcd(a, b)
    assert call(shim, "gcd", 0, 12) == 12 and call(shim, "gcd", 12, 0) == 12 and call(shim, "gcd", 1 << 70, 1 << 40) == 1 << 40


@pytest.mark.parametrize("bits", [64, 521, 2048])
def test_montgomery_and_powers(shim, bits):
    rng = random.Random(bits + 1)
    for _ in range(6):
        m = rng.getrandbits(bits) | (1 << (bits - 1)) | 1
        words = (m.bit_length() + 31) // 32
        rinv = pow(1 << (32 * words), -1, m)
        for _ in range(5):
            a, b = rng.randrange(m), rng.randrange(m)
            assert call(shim, "montmul", a, b, m) == a * b * rinv % m
        a, e = rng.randrange(m), rng.getrandbits(rng.choice((1, 17, bits)))
        assert call(shim, "powmod", a, e, m) == pow(a, e, m)
        assert call(shim, "powmod", a, 0, m) == 1 % m and call(shim, "powmod", 0, 5, m) == 0
        assert shim.hostbig_neg_inv32(m & 0xFFFFFFFF) == (-pow(m, -1, 1 << 32)) % (1 << 32)


def test_inverse_modulo_a_power_of_two(shim):
    rng = random.Random(11)
    for _ in range(40):
        k = rng.choice((1, 2, 29, 32, 33, 261, 522, 1044, 2088))
        x = rng.getrandbits(rng.choice((8, 64, 1024))) | 1
        inv = call(shim, "inv_pow2", x, k=k)
        assert inv < (1 << k) and (inv * x) % (1 << k) == 1
