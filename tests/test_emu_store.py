"""The handle-based store (managed device-resident operands) on the CPU stand-in for the HIP
runtime: allocator bookkeeping, release on last use, and chains of operators over handles
compared with the oracle running the same chain."""
import ctypes as C
import random

import numpy as np

from oracle import paillier_oracle as O
from paper_2107_13797_amd import _cabi, synth
from test_emu_kernels import BITS, Dev, emu, env, words, zeros  # noqa: F401  (fixtures)

K = _cabi
EINVAL, ENOMEM = -1, -5


class EmuStore:
    def __init__(self, lib, ctx, arena_bytes):
        self.lib, self.arena = lib, zeros(lib, (arena_bytes // 4,))
        h = C.c_void_p()
        assert lib.haflo_store_create(ctx, self.arena.p, arena_bytes, None, C.byref(h)) == 0
        self.h = h

    def stats(self):
        v = [C.c_size_t() for _ in range(4)]
        assert self.lib.haflo_store_stats(self.h, *[C.byref(x) for x in v]) == 0
        return dict(zip(("live_bytes", "peak_bytes", "live_objects", "largest_free"), [x.value for x in v]))

    def info(self, handle):
        kind, count, ptr, uses = C.c_int(), C.c_size_t(), C.c_void_p(), C.c_uint32()
        rc = self.lib.haflo_store_info(self.h, handle, C.byref(kind), C.byref(count), C.byref(ptr), C.byref(uses))
        return None if rc != 0 else (kind.value, count.value, ptr.value, uses.value)

    def new(self, kind, count, uses):
        h = C.c_uint64()
        rc = self.lib.haflo_store_new(self.h, kind, count, uses, C.byref(h))
        return rc, h.value

    def up(self, kind, arr, count, uses=1):
        arr = np.ascontiguousarray(arr)
        h = C.c_uint64()
        assert self.lib.haflo_h_upload(self.h, kind, arr.ctypes.data, 1, count, uses, C.byref(h)) == 0
        return h.value

    def down(self, handle, shape, dtype):
        out = np.empty(shape, dtype)
        assert self.lib.haflo_h_download(self.h, handle, out.ctypes.data, 1) == 0
        return out

    def op(self, name, *args, status=None):
        out, st = C.c_uint64(), C.c_uint64()
        fn = getattr(self.lib, name)
        rc = fn(self.h, *args, C.byref(out)) if status is None else fn(self.h, *args, C.byref(out),
                                                                         C.byref(st) if status else None)
        return (rc, out.value, st.value) if status else (rc, out.value)

    def close(self):
        assert self.lib.haflo_store_destroy(self.h) == 0


def test_store_allocator_bookkeeping(env):
    lib, ctx, sk, nlw = env
    bad = C.c_void_p()
    arena = zeros(lib, (1024,))
    assert lib.haflo_store_create(ctx, arena.p + 4, 2048, None, C.byref(bad)) == EINVAL  # misaligned
    assert lib.haflo_store_create(ctx, arena.p, 100, None, C.byref(bad)) == EINVAL       # below one granule
    st = EmuStore(lib, ctx, 16 * 256)
    assert st.stats() == {"live_bytes": 0, "peak_bytes": 0, "live_objects": 0, "largest_free": 4096}
    rc, a = st.new(K.KIND_F32, 64, 0)      # 256 bytes
    rc2, b = st.new(K.KIND_F64, 65, 0)     # 520 -> 768 bytes
    rc3, c = st.new(K.KIND_U32, 1, 0)      # 256
    rc4, z = st.new(K.KIND_I64, 0, 0)      # an empty object still has an address of its own
    assert (rc, rc2, rc3, rc4) == (0, 0, 0, 0) and len({a, b, c, z}) == 4 and 0 not in (a, b, c, z)
    base = st.info(a)[2]
    assert [st.info(h)[2] - base for h in (a, b, c, z)] == [0, 256, 1024, 1280]
    assert st.info(b)[:2] == (K.KIND_F64, 65) and st.info(b)[3] == 0
    assert st.stats() == {"live_bytes": 1536, "peak_bytes": 1536, "live_objects": 4, "largest_free": 2560}
    assert st.new(K.KIND_F32, 641, 0)[0] == ENOMEM and st.new(99, 1, 0)[0] == EINVAL
    assert st.new(K.KIND_F64, 2 ** 62, 0)[0] in (EINVAL, ENOMEM)
    # freeing b leaves a hole of three granules; a request that fits it exactly goes there (best fit)
    assert lib.haflo_store_release(st.h, b) == 0 and st.info(b) is None
    assert lib.haflo_store_release(st.h, b) == EINVAL
    rc, d = st.new(K.KIND_F32, 192, 0)
    assert rc == 0 and st.info(d)[2] - base == 256
    # the slot of b is reused with a new generation: the old handle stays dead
    assert d != b and (d & 0xFFFFFFFF) == (b & 0xFFFFFFFF) and st.info(b) is None
    # neighbours merge on release, in either order
    for h in (a, c, d, z):
        assert lib.haflo_store_release(st.h, h) == 0
    s = st.stats()
    assert s["live_bytes"] == 0 and s["live_objects"] == 0 and s["largest_free"] == 4096 and s["peak_bytes"] == 1536
    assert st.new(K.KIND_F32, 1024, 0)[0] == 0
    assert st.info(0) is None and st.info(12345 << 32 | 1) is None
    st.close()


def test_store_uses_and_failures_consume_nothing(env):
    lib, ctx, sk, nlw = env
    pk, lp = sk.public, BITS // 32
    rng = random.Random(5)
    st = EmuStore(lib, ctx, 1 << 20)
    ms = [rng.randrange(pk.n) for _ in range(3)]
    rs = [rng.randrange(1, pk.n) for _ in range(3)]
    hm, hr = st.up(K.KIND_PLAIN, synth.ints_to_words(ms, lp), 3, 1), st.up(K.KIND_PLAIN, synth.ints_to_words(rs, lp), 3, 2)
    # wrong kinds, mismatched counts and dead handles are refused and leave the operands alone
    hf = st.up(K.KIND_F32, np.zeros(3, np.float32), 3, 1)
    h2 = st.up(K.KIND_PLAIN, synth.ints_to_words(rs[:2], lp), 2, 1)
    assert st.op("haflo_h_encrypt", hm, hf, 1)[0] == EINVAL
    assert st.op("haflo_h_encrypt", hm, h2, 1)[0] == EINVAL
    assert st.op("haflo_h_encrypt", hm, 777, 1)[0] == EINVAL
    assert st.info(hm)[3] == 1 and st.info(hr)[3] == 2
    rc, c = st.op("haflo_h_encrypt", hm, hr, 1)
    assert rc == 0 and st.info(hm) is None and st.info(hr)[3] == 1
    # c + c needs two uses of c
    assert st.op("haflo_h_add", c, c, 1)[0] == EINVAL and st.info(c)[3] == 1
    assert lib.haflo_store_release(st.h, c) == 0
    rc, c = st.op("haflo_h_encrypt", st.up(K.KIND_PLAIN, synth.ints_to_words(ms, lp), 3), hr, 2)
    assert rc == 0 and st.info(hr) is None
    rc, d = st.op("haflo_h_add", c, c, 0)
    assert rc == 0 and st.info(c) is None and st.info(d)[3] == 0
    want = [O.add(pk, x, x) for x in (O.encrypt(pk, m, r) for m, r in zip(ms, rs))]
    out = zeros(lib, (3, BITS // 16))
    assert lib.haflo_export_cipher(ctx, st.info(d)[2], out.p, 3, None) == 0
    assert synth.words_to_ints(out.get()) == want
    # an object kept with uses = 0 survives any number of calls; the result goes to a new block
    rc, e = st.op("haflo_h_scalar_mul", d, -3, 1)
    rc2, f = st.op("haflo_h_scalar_mul", d, 5, 1)
    assert (rc, rc2) == (0, 0) and st.info(d)[3] == 0 and len({st.info(h)[2] for h in (d, e, f)}) == 3
    assert lib.haflo_export_cipher(ctx, st.info(e)[2], out.p, 3, None) == 0
    assert synth.words_to_ints(out.get()) == [O.scalar_mul(pk, x, -3) for x in want]
    # a result at its operand's last use takes over the operand's block
    pe = st.info(e)[2]
    rc, g = st.op("haflo_h_scalar_mul", e, 7, 1)
    assert rc == 0 and st.info(e) is None and st.info(g)[2] == pe
    assert lib.haflo_export_cipher(ctx, st.info(g)[2], out.p, 3, None) == 0
    assert synth.words_to_ints(out.get()) == [O.scalar_mul(pk, x, -21) for x in want]
    st.close()
    # an arena with room for the operands but not for the call: ENOMEM, operands untouched
    small = EmuStore(lib, ctx, 4 * 256)
    hm = small.up(K.KIND_PLAIN, synth.ints_to_words(ms, lp), 3, 1)
    hr = small.up(K.KIND_PLAIN, synth.ints_to_words(rs, lp), 3, 1)
    before = small.stats()
    assert small.op("haflo_h_encrypt", hm, hr, 1)[0] == ENOMEM
    after = small.stats()
    assert small.info(hm)[3] == 1 and small.info(hr)[3] == 1
    assert {k: after[k] for k in ("live_bytes", "live_objects")} == {k: before[k] for k in ("live_bytes", "live_objects")}
    small.close()


def test_store_fore_gradient_chain_matches_oracle(env):
    """The fore gradient as the framework's chain of basic operators over handles:
    [[q_host]] + E(q_guest) + (-2) * E(q_label), every intermediate freed by its last use."""
    lib, ctx, sk, nlw = env
    pk, lp, s = sk.public, BITS // 32, 20
    rng = random.Random(9)
    count = 7
    uh, ug = synth.normal_f32(count, 2.0, 91), synth.normal_f32(count, 2.0, 92)
    y = np.where(np.arange(count) % 3 == 0, 1.0, -1.0).astype(np.float32)
    r = [[rng.randrange(1, pk.n) for _ in range(count)] for _ in range(3)]
    st = EmuStore(lib, ctx, 1 << 20)
    enc = []
    for vals, rr in zip((uh, ug, y), r):
        rc, hp, hs = st.op("haflo_h_encode", st.up(K.KIND_F32, vals, count), s, 1, status=True)
        assert rc == 0 and st.down(hs, (count,), np.uint32).tolist() == [0] * count
        rc, hc = st.op("haflo_h_encrypt", hp, st.up(K.KIND_PLAIN, synth.ints_to_words(rr, lp), count), 1)
        assert rc == 0
        enc.append(hc)
    p_host = st.info(enc[0])[2]
    rc, t = st.op("haflo_h_add", enc[0], enc[1], 1)
    rc2, l2 = st.op("haflo_h_scalar_mul", enc[2], -2, 1)
    rc3, d = st.op("haflo_h_add", t, l2, 0)
    assert (rc, rc2, rc3) == (0, 0, 0)
    # only the result is left, and it sits where the host's ciphertexts were
    assert st.stats()["live_objects"] == 1 and st.info(d)[2] == p_host
    q = [[O.quantise(float(v), s) for v in vals] for vals in (uh, ug, y)]
    c = [[O.encrypt(pk, m % pk.n, rr) for m, rr in zip(qs, rs)] for qs, rs in zip(q, r)]
    want = [O.add(pk, O.add(pk, a, b), O.scalar_mul(pk, l, -2)) for a, b, l in zip(*c)]
    out = zeros(lib, (count, BITS // 16))
    assert lib.haflo_export_cipher(ctx, st.info(d)[2], out.p, count, None) == 0
    assert synth.words_to_ints(out.get()) == want
    # the key owner reads q_host + q_guest - 2 q_label
    rc, hp = st.op("haflo_h_decrypt", d, 1)
    rc2, hv, hs = st.op("haflo_h_decode", hp, s + 2, 1, status=True)
    assert (rc, rc2) == (0, 0) and st.info(d)[3] == 0
    vals = st.down(hv, (count,), np.float64)
    assert st.down(hs, (count,), np.uint32).tolist() == [0] * count
    assert vals.tolist() == [(a + b - 2 * l) / 2.0 ** (s + 2) for a, b, l in zip(*q)]
    assert lib.haflo_store_release(st.h, d) == 0 and st.stats()["live_bytes"] == 0
    st.close()
    # a store over a public-only context refuses to decrypt and keeps the operand
    pub = C.c_void_p()
    nb = pk.n.to_bytes(BITS // 8, "little")
    assert lib.haflo_ctx_create_public((C.c_uint8 * len(nb)).from_buffer_copy(nb), BITS, C.byref(pub)) == 0
    ps = EmuStore(lib, pub, 1 << 20)
    rc, hc = ps.new(K.KIND_CIPHER, 2, 1)
    assert rc == 0 and ps.op("haflo_h_decrypt", hc, 1)[0] == -3 and ps.info(hc)[3] == 1
    ps.close()
    assert lib.haflo_ctx_destroy(pub) == 0


def test_store_matvec_sum_and_scalars_match_oracle(env):
    lib, ctx, sk, nlw = env
    pk, lp = sk.public, BITS // 32
    rng = random.Random(13)
    rows, cols = 6, 3
    cs = [O.encrypt(pk, rng.randrange(pk.n), rng.randrange(1, pk.n)) for _ in range(rows)]
    Xf = synth.normal_f32((rows, cols), 1.0, 14)
    Xf[2, 1] = 0.0
    st = EmuStore(lib, ctx, 8 << 20)
    rc, hc = st.new(K.KIND_CIPHER, rows, 0)
    assert rc == 0 and lib.haflo_import_cipher(ctx, words(lib, cs, BITS // 16).p, st.info(hc)[2], None, rows, None) == 0
    rc, hx, hs = st.op("haflo_h_encode_exponents", st.up(K.KIND_F32, Xf, rows * cols), 8, 0, status=True)
    assert rc == 0 and not st.down(hs, (rows * cols,), np.uint32).any()
    X = [[O.encode_exponent(float(v), 8)[0] for v in row] for row in Xf]
    assert st.op("haflo_h_matvec", 0, hc, hx, rows + 1, cols, 1)[0] == EINVAL
    assert st.op("haflo_h_matvec", 2, hc, hx, rows, cols, 1)[0] == EINVAL
    out = zeros(lib, (rows, BITS // 16))
    rc, g = st.op("haflo_h_matvec", 0, hc, hx, rows, cols, 2)
    assert rc == 0 and lib.haflo_export_cipher(ctx, st.info(g)[2], out.p, cols, None) == 0
    want_g = O.matvec(pk, 0, cs, X)
    assert synth.words_to_ints(out.get())[:cols] == want_g
    rc, f = st.op("haflo_h_matvec", 1, g, hx, rows, cols, 1)
    assert rc == 0 and st.info(g)[3] == 1
    assert lib.haflo_export_cipher(ctx, st.info(f)[2], out.p, rows, None) == 0
    assert synth.words_to_ints(out.get()) == O.matvec(pk, 1, want_g, X)
    rc, t = st.op("haflo_h_sum", g, 1)
    assert rc == 0 and st.info(g) is None and st.info(t)[1] == 1
    assert lib.haflo_export_cipher(ctx, st.info(t)[2], out.p, 1, None) == 0
    assert synth.words_to_ints(out.get())[0] == O.summation(pk, want_g)
    ks = [rng.randrange(2 ** 64) for _ in range(rows)]
    rc, e = st.op("haflo_h_scalar_mul_each", hc, st.up(K.KIND_U64, np.array(ks, dtype=np.uint64), rows), 1)
    assert rc == 0 and lib.haflo_export_cipher(ctx, st.info(e)[2], out.p, rows, None) == 0
    assert synth.words_to_ints(out.get()) == [O.scalar_mul(pk, c, k) for c, k in zip(cs, ks)]
    # temporaries are gone: what is live is hc, hx, f, t, e
    assert st.stats()["live_objects"] == 5 and st.stats()["peak_bytes"] > st.stats()["live_bytes"]
    st.close()


def test_store_allocator_random_sequences(env):
    """Random allocate / release traffic against a model: blocks never overlap, stay inside the
    arena, the accounting matches, and everything merges back into one free block."""
    lib, ctx, sk, nlw = env
    arena_bytes = 64 * 1024
    sizes = {K.KIND_F32: 4, K.KIND_F64: 8, K.KIND_CIPHER: nlw * 4, K.KIND_PLAIN: BITS // 8}
    for seed in range(4):
        rng = random.Random(seed)
        st = EmuStore(lib, ctx, arena_bytes)
        base, live = None, {}
        for _ in range(400):
            if live and (rng.random() < 0.45 or len(live) > 40):
                h = rng.choice(sorted(live))
                assert lib.haflo_store_release(st.h, h) == 0
                del live[h]
            else:
                kind = rng.choice(sorted(sizes))
                count = rng.choice((0, 1, 3, 17, 64, 200, 1000))
                rc, h = st.new(kind, count, rng.choice((0, 1, 2)))
                need = max(1, -(-sizes[kind] * count // 256)) * 256
                if rc == ENOMEM:
                    assert st.stats()["largest_free"] < need
                    continue
                assert rc == 0 and h not in live
                ptr = st.info(h)[2]
                base = ptr if base is None else min(base, ptr)
                live[h] = (ptr, need)
            spans = sorted(live.values())
            assert all(a + n <= b for (a, n), (b, _) in zip(spans, spans[1:]))
            s = st.stats()
            assert s["live_bytes"] == sum(n for _, n in spans) and s["live_objects"] == len(live)
            assert all(st.arena.p <= a and a + n <= st.arena.p + arena_bytes for a, n in spans)
        for h in sorted(live):
            assert lib.haflo_store_release(st.h, h) == 0
        s = st.stats()
        assert s["live_bytes"] == 0 and s["largest_free"] == arena_bytes
        st.close()
