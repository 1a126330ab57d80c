#!/usr/bin/env python3
"""Benchmark of the Paillier operator path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--batch B] [--features F] [--bits 2048]

One step is one pass of the whole hot path over one batch of synthetic
federated-LR-shaped input, with everything resident in HBM before timing:

    encode residuals -> encrypt -> add another party's ciphertexts ->
    scalar multiply -> X^T [[d]] -> X [[w]] -> decrypt -> decode

at a 2048-bit key (the key size the headline metric is quoted on). The
headline value is full-length modular exponentiations (2048-bit exponent,
4096-bit modulus: the r^n of every encryption) per second over the whole step
time. The JSON line also carries the rate of the encrypted-gradient product,
the roofline of the dominant kernel (encryption) against the chip's 32-bit
integer multiply-add issue rate, and the CPU oracle timed on the host cores
on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X: 256 compute units x 64 lanes x one instruction per lane and clock at 2.4 GHz, the nominal vector
# rate. The 32x32+64 integer multiply-add itself reaches 0.66 - 0.74 of it (bench_peak.py measures that,
# profiles/peak_microbench.md holds the figures); the nominal figure stays the denominator.
PEAK_MAD32_PER_S = 256 * 64 * 2.4e9

# HBM bytes of the encryption launch at the profiled shape (2048-bit key, 65536 elements): rocprofv3 --pmc
# FETCH_SIZE / WRITE_SIZE, each scaled by what the counter reads for a 1 GiB device copy. The figure is
# transcribed from the profile named here, not measured by this run, and is reported for that shape only.
TRAFFIC_PROFILE = "profiles/k_engine_pairs_encrypt_2048bit_b65536_pmc.md"
TRAFFIC_BYTES_PROFILED = {(2048, 65536): (11180151 + 2579578) * 1024}


def montmul_mul32(limbs):
    """32x32->64 multiply-adds of one word-serial Montgomery product on `limbs` 32-bit limbs."""
    return 2 * limbs * limbs + limbs


def _oracle_encrypt_chunk(args):
    from oracle import paillier_oracle as O
    n, ms, rs = args
    pk = O.PublicKey(n)
    t0 = time.perf_counter()
    out = [O.encrypt(pk, m, r) for m, r in zip(ms, rs)]
    return time.perf_counter() - t0, out


def _oracle_operators_one_core(p, q, seed):
    """The oracle's operators one by one on one core (the paper's Table 2 has a one-core CPU column):
    -> {operator: {"per_s": rate, "sample": count}}; a few seconds in total."""
    import random

    from oracle import paillier_oracle as O
    sk = O.PrivateKey(p, q)
    pk = sk.public
    n = pk.n
    rng = random.Random(seed)
    res = {}

    def rate(name, count, fn):
        t0 = time.perf_counter()
        out = fn()
        res[name] = {"per_s": count / (time.perf_counter() - t0), "sample": count}
        return out
    vals = [rng.gauss(0.0, 0.25) for _ in range(20000)]
    enc = rate("encode", len(vals), lambda: [O.encode(pk, v, 24)[0] for v in vals])
    rate("decode", len(enc), lambda: [O.decode(pk, m, 24) for m in enc])
    ms = enc[:12]
    rs = [rng.randrange(1, n) for _ in ms]
    cs = rate("encrypt", len(ms), lambda: [O.encrypt(pk, m, r) for m, r in zip(ms, rs)])
    rate("decrypt (lambda, mu)", 6, lambda: [O.decrypt(sk, c) for c in cs[:6]])
    rate("decrypt (through p^2, q^2)", len(cs), lambda: [O.decrypt_crt(sk, c) for c in cs])
    many = [cs[i % len(cs)] for i in range(4000)]
    rate("add", len(many), lambda: [O.add(pk, a, b) for a, b in zip(many, many[1:] + many[:1])])
    ks = [rng.getrandbits(64) for _ in range(60)]
    rate("scalar_mul (64-bit)", len(ks), lambda: [O.scalar_mul(pk, cs[i % len(cs)], k) for i, k in enumerate(ks)])
    X = [[rng.randrange(-(1 << 18), 1 << 18)] for _ in range(240)]
    rate("matvec X^T[[d]] entries", len(X), lambda: O.matvec(pk, 0, [cs[i % len(cs)] for i in range(len(X))], X))
    rate("summation", len(many), lambda: O.summation(pk, many))
    return res


def _gmp_powm_one_core(n, rs, want_rn):
    """Secondary CPU figure, never the checker: the same r^n mod n^2 with mpz_powm of the system's libgmp
    through ctypes on one core (the paper's CPU column used gmpy2, which wraps the same routine).
    -> dict, or None where the library is not there."""
    import ctypes as C
    try:
        g = C.CDLL("libgmp.so.10")
    except OSError:
        return None

    class Mpz(C.Structure):
        _fields_ = [("alloc", C.c_int), ("size", C.c_int), ("d", C.c_void_p)]
    for name in ("__gmpz_init", "__gmpz_clear", "__gmpz_set_str", "__gmpz_powm", "__gmpz_get_str"):
        if not hasattr(g, name):
            return None
    g.__gmpz_set_str.argtypes = [C.POINTER(Mpz), C.c_char_p, C.c_int]
    g.__gmpz_get_str.argtypes = [C.c_char_p, C.c_int, C.POINTER(Mpz)]
    g.__gmpz_get_str.restype = C.c_char_p
    base, exp, mod, out = Mpz(), Mpz(), Mpz(), Mpz()
    for z in (base, exp, mod, out):
        g.__gmpz_init(C.byref(z))
    g.__gmpz_set_str(C.byref(exp), b"%x" % n, 16)
    g.__gmpz_set_str(C.byref(mod), b"%x" % (n * n), 16)
    buf = C.create_string_buffer((n * n).bit_length() // 4 + 8)
    got, spent = [], 0.0
    for r in rs:
        g.__gmpz_set_str(C.byref(base), b"%x" % r, 16)
        t0 = time.perf_counter()
        g.__gmpz_powm(C.byref(out), C.byref(base), C.byref(exp), C.byref(mod))
        spent += time.perf_counter() - t0
        got.append(int(g.__gmpz_get_str(buf, 16, C.byref(out)), 16))
    for z in (base, exp, mod, out):
        g.__gmpz_clear(C.byref(z))
    assert got == want_rn, "libgmp disagrees with python's pow"
    return {"value": len(rs) / spent, "unit": "modexp/s", "cores": 1, "kind": "libgmp mpz_powm through ctypes; "
            "a secondary figure, not the oracle and never the checker",
            "sample": "%d of the same r^n mod n^2, %.1f s" % (len(rs), spent)}


def cpu_baseline(p, q, ms, rs, want):
    """The oracle's encryption (the same r^n modexp the GPU headline counts) on all host cores and on
    one core, and the other operators on one core."""
    import multiprocessing as mp
    n = p * q
    cores = max(1, min(16, os.cpu_count() or 1))
    per = max(1, len(ms) // cores)
    chunks = [(n, ms[i * per:(i + 1) * per], rs[i * per:(i + 1) * per]) for i in range(cores)]
    chunks = [c for c in chunks if c[1]]
    with mp.get_context("spawn").Pool(len(chunks)) as pool:
        t0 = time.perf_counter()
        res = pool.map(_oracle_encrypt_chunk, chunks)
        wall = time.perf_counter() - t0
    done = sum(len(c[1]) for c in chunks)
    got = [c for _, part in res for c in part]
    assert got == want[:done], "GPU encryption disagrees with the oracle on the timed sample"
    k1 = min(24, len(ms))
    t1, one = _oracle_encrypt_chunk((n, ms[:k1], rs[:k1]))
    assert one == want[:k1], "GPU encryption disagrees with the oracle on the one-core sample"
    return {"value": done / wall, "unit": "modexp/s", "cores": len(chunks), "kind": "oracle",
            "sample": "%d encryptions (2048-bit r^n mod n^2) of the step's first elements, python int pow, "
                      "%.1f core-seconds" % (done, sum(t for t, _ in res)),
            "one_core": {"value": k1 / t1, "unit": "modexp/s", "cores": 1,
                         "sample": "the first %d of the same encryptions, %.1f s" % (k1, t1)},
            "gmp_one_core": _gmp_powm_one_core(n, rs[:96], [pow(r, n, n * n) for r in rs[:96]]),
            "operators_one_core": _oracle_operators_one_core(p, q, 99),
            "operators_note": "python int oracle at the benchmark's key size, one core, instances per second "
                              "(the shape of the paper's one-core CPU column in its Table 2)"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--batch", type=int, default=65536)
    ap.add_argument("--features", type=int, default=32)
    ap.add_argument("--bits", type=int, default=2048)
    ap.add_argument("--cpu-sample", type=int, default=192)
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-configs", action="store_true",
                    help="skip the per-operator timing of the five benchmark configurations (about 40 s)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device-to-device copy: the known-size kernel that scales "
                         "rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path; run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2107_13797_amd import _cabi, api, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    bits, B, F = args.bits, args.batch, args.features
    seed = synth.BASE_SEED + bits
    p, q = api.haflo_keygen(bits, seed)
    n = p * q
    ctx = api.haflo_ctx_create_private(p, q, bits)  # the key owner: decrypts
    pub = api.haflo_ctx_create_public(n, bits)       # everyone else: encrypts and computes on ciphertexts
    lp = bits // 32

    def dev(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint32:
            a = a.view(np.int32)
        return torch.from_numpy(a).cuda()

    # synthetic inputs (hetero-LR shapes: residuals ~N(0, 0.25) at 2^24, features ~N(0,1) at 2^16,
    # a sparse forward-pass matrix with 70% zeros at 2^16), all resident before timing
    rng = np.random.default_rng(seed)
    d = dev(synth.normal_f32(B, 0.25, seed + 1))
    r_words = rng.integers(0, 2 ** 32, size=(B, lp), dtype=np.uint32)
    r_words[:, -1] &= 0x7FFFFFFF
    r = dev(r_words)
    Xg = api.haflo_encode_exponents_f32(dev(synth.normal_f32((B, F), 1.0, seed + 2)), 16)
    Xw = api.haflo_encode_exponents_f32(dev(synth.sparse_uniform_f32((B, F), 0.7, seed + 3)), 16)
    other = api.haflo_encrypt(ctx, api.haflo_encode_f32(ctx, dev(synth.normal_f32(B, 0.25, seed + 4)), 24),
                              dev(np.roll(r_words, 1, axis=0)))
    wc = api.haflo_encrypt(ctx, api.haflo_encode_f32(ctx, dev(synth.normal_f32(F, 0.1, seed + 5)), 24),
                           dev(r_words[:F].copy()))
    k_quarter = 1 << 6  # the fore-gradient's factor 0.25 at 2^8, keeps decoded sums inside int64
    torch.cuda.synchronize()
    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.int32, device="cuda").fill_(7)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)  # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    stages = ("encode", "encrypt", "add", "scalar_mul", "matvec_xt_d", "matvec_x_w", "decrypt", "decode")
    # HIP events on torch's current stream, which is the stream every kernel is launched on
    events = [{name: (torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for name in stages}
              for _ in range(args.steps)]
    stage_ms = {name: 0.0 for name in stages}
    keep = {}

    def step(ev):
        record = ev is not None

        def timed(name, fn):
            if record:
                ev[name][0].record()
            out = fn()
            if record:
                ev[name][1].record()
            return out
        # the public-key path everywhere except decryption: every encryption is one full-length
        # exponentiation r^n modulo n^2 (4096-bit modulus, 2048-bit exponent)
        plain = timed("encode", lambda: api.haflo_encode_f32(pub, d, 24))
        c = timed("encrypt", lambda: api.haflo_encrypt(pub, plain, r))
        s = timed("add", lambda: api.haflo_add(pub, c, other))
        fg = timed("scalar_mul", lambda: api.haflo_scalar_mul_i64_bcast(pub, s, k_quarter))
        grad = timed("matvec_xt_d", lambda: api.haflo_cipher_matvec(pub, 0, fg, Xg))
        fwd = timed("matvec_x_w", lambda: api.haflo_cipher_matvec(pub, 1, wc, Xw))
        both = torch.cat([fwd[:4096], grad], dim=0)
        pl = timed("decrypt", lambda: api.haflo_decrypt(ctx, both))
        qv = timed("decode", lambda: (api.haflo_decode(ctx, pl[:4096], 40), api.haflo_decode(ctx, pl[4096:], 48)))
        keep["c"], keep["q"], keep["plain"] = c, qv, plain

    for _ in range(args.warmup):
        step(None)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(events[i])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    for ev in events:
        for name in stages:
            stage_ms[name] += ev[name][0].elapsed_time(ev[name][1])

    ms_per_step = wall * 1e3 / args.steps
    modexp_per_s = B * args.steps / wall
    enc_ms = stage_ms["encrypt"] / args.steps
    mm, limbs = api.haflo_op_cost(pub, _cabi.OP_ENCRYPT)
    algo_mad = B * mm * montmul_mul32(limbs)
    achieved = algo_mad / (enc_ms * 1e-3)
    executed = B * api.haflo_op_work(pub, _cabi.OP_ENCRYPT) / (enc_ms * 1e-3)

    # outside the timed steps: the key owner's encryption of the same batch (r^n through p^2 and
    # q^2, bit-identical ciphertexts), reported next to the headline, never inside it
    own = api.haflo_encrypt(ctx, keep["plain"], r)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(3):
        own = api.haflo_encrypt(ctx, keep["plain"], r, own)
    e1.record()
    torch.cuda.synchronize()
    own_ms = e0.elapsed_time(e1) / 3
    assert torch.equal(own, keep["c"]), "key-owner and public-key encryption disagree"
    mm_o, limbs_o = api.haflo_op_cost(ctx, _cabi.OP_ENCRYPT)
    achieved_o = B * mm_o * montmul_mul32(limbs_o) / (own_ms * 1e-3)
    out = {
        "metric": "Paillier modexp/s at 2048-bit n; encrypted X^T[[d]] entries/s",
        "value": modexp_per_s,
        "unit": "modexp/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "u32",
        "dtype_note": "29-bit limbs in u32 words, 32x32+64-bit integer multiply-add, exact integer arithmetic",
        "data": "synthetic",
        "config": {"workload": "hetero-LR step at a %d-bit key: encode, encrypt, add, scalar_mul, X^T[[d]], "
                               "X[[w]], decrypt, decode" % bits,
                   "n_bits": bits, "batch": B, "features": F},
        "xt_d_entries_per_s": B * F / (stage_ms["matvec_xt_d"] / args.steps * 1e-3),
        "encrypt_per_s": B / (enc_ms * 1e-3),
        "encrypt_key_owner_per_s": B / (own_ms * 1e-3),
        "roofline_key_owner_encrypt": {"bound": "alu", "kernel": "k_engine_pair (r^n mod p^2, q^2) + recombination",
                                       "achieved": achieved_o / 1e12, "peak": PEAK_MAD32_PER_S / 1e12,
                                       "unit": "TOP/s", "op": "32x32+64-bit integer multiply-add", "frac": achieved_o / PEAK_MAD32_PER_S,
                                       "algorithmic": "%d Montgomery-product equivalents x (2*%d^2+%d) mul32 per "
                                                      "encryption" % (mm_o, limbs_o, limbs_o)},
        "stage_ms": {k: v / args.steps for k, v in stage_ms.items()},
        "roofline": {"bound": "alu", "kernel": "k_engine_pairs (encryption program on pairs of residues modulo n)", "achieved": achieved / 1e12,
                     "peak": PEAK_MAD32_PER_S / 1e12, "unit": "TOP/s", "op": "32x32+64-bit integer multiply-add",
                     "frac": achieved / PEAK_MAD32_PER_S,
                     "traffic": TRAFFIC_BYTES_PROFILED.get((bits, B)),
                     "traffic_unit": "bytes per launch",
                     "traffic_source": "%s (rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE on this launch shape); "
                                       "not measured in this run" % TRAFFIC_PROFILE,
                     "accounting": "achieved counts every product of the exponentiation schedule as a word-serial "
                                   "Montgomery product on 32-bit limbs, 2 L^2 + L multiply-adds, squarings included; the "
                                   "kernel needs fewer: it works modulo n^2 on pairs of half-length residues (5/8 of the "
                                   "limb products of a product, 0.57 of a squaring's) in 29-bit limbs",
                     "executed": executed / 1e12,
                     "frac_executed": executed / PEAK_MAD32_PER_S,
                     "executed_note": "v_mad_u64_u32 the kernel really issues per second, in 10^12, and their share of "
                                      "the same peak; a stream of nothing but this instruction sustains 0.66 of that "
                                      "peak at the kernel's four wavefronts per SIMD (profiles/peak_microbench.md)",
                     "algorithmic": "%d Montgomery products x (2*%d^2+%d) mul32 per encryption" % (mm, limbs, limbs)},
    }
    if not args.no_cpu:
        k = min(args.cpu_sample, B)
        from paper_2107_13797_amd import synth as _s
        ms = _s.words_to_ints(api.haflo_encode_f32(pub, d[:k].contiguous(), 24).cpu().numpy())
        rs = _s.words_to_ints(r_words[:k])
        want = _s.words_to_ints(api.haflo_export_cipher(pub, keep["c"][:k].contiguous()).cpu().numpy())
        out["cpu_baseline"] = cpu_baseline(p, q, ms, rs, want)
    if not args.no_configs:
        # the five benchmark configurations, operator by operator (bench_configs.py), outside the timed steps
        ctx.close()
        pub.close()
        del other, wc, Xg, Xw, d, r, own, keep
        torch.cuda.empty_cache()
        import bench_configs
        rep = bench_configs.run_configs((1, 2, 3, 4, 5), reps=1, verbose=False)
        out["configs"] = {"cfg%d" % k: rows for k, rows in rep.items()}
        for k in (2, 5):
            row = [x for x in rep[k] if x["op"].startswith("matvec")][0]
            out["xt_d_entries_per_s_cfg%d" % k] = row["rate"]
        out["configs_note"] = ("per operator: units, ms (one run after a warm-up, HIP events), units per second, "
                               "fraction of the bounding roofline (alu: 39.3e12 mul32/s, hbm: 8 TB/s); frac counts every "
                               "product of the schedule as a full-length Montgomery product (it can pass 1 where the "
                               "kernels work on pairs of half-length residues), frac_executed the multiply-adds "
                               "really issued")
    print(json.dumps(out))


if __name__ == "__main__":
    main()
