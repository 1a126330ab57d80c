#!/usr/bin/env python3
"""Wall time of the five benchmark configurations, operator by operator.

    python bench_configs.py [--configs 1,2,3,4,5] [--reps 3] [--json out.json]

Each configuration of `paper_2107_13797_amd.synth.CONFIGS` is generated with its seeded inputs,
made resident in HBM, and its operators are timed with HIP events on the launch stream (median of
`--reps` runs after one warm-up). `bench.py` remains the contract benchmark; the parity of the same
configurations with the oracle is what `tests/test_gpu_parity.py` checks.
"""
import argparse
import json
import os
import statistics
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="1,2,3,4,5")
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--json", default=None)
    args = ap.parse_args()

    import numpy as np
    import torch

    from paper_2107_13797_amd import api, synth

    assert torch.cuda.is_available(), "needs a GPU"

    def dev(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint32:
            a = a.view(np.int32)
        elif a.dtype == np.uint64:
            a = a.view(np.int64)
        return torch.from_numpy(a).cuda()

    def timed(fn):
        out = fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(args.reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            out = fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return statistics.median(ts), out

    def rand_words(count, lp, seed, top_mask=0x7FFFFFFF):
        r = np.random.default_rng(seed).integers(0, 2 ** 32, size=(count, lp), dtype=np.uint32)
        r[:, -1] &= top_mask
        return dev(r)

    report = {}
    for k in [int(x) for x in args.configs.split(",")]:
        cfg = synth.CONFIGS[k]
        bits = cfg["n_bits"]
        lp = bits // 32
        p, q = api.haflo_keygen(bits, synth.BASE_SEED + bits)
        own = api.haflo_ctx_create_private(p, q, bits)
        pub = api.haflo_ctx_create_public(p * q, bits)
        rows = []

        def add(name, units, ms, unit):
            rows.append((name, units, ms, unit))

        if k == 1:
            n = cfg["count"]
            m, r = rand_words(n, lp, synth.seed_for(1, 0), 0x3FFFFFFF), rand_words(n, lp, synth.seed_for(1, 1))
            ks = dev(np.random.default_rng(synth.seed_for(1, 2)).integers(0, 2 ** 63, size=n, dtype=np.uint64))
            ms, c = timed(lambda: api.haflo_encrypt(pub, m, r))
            add("encrypt", n, ms, "encryptions")
            ms, s = timed(lambda: api.haflo_add(pub, c, torch.roll(c, -1, 0).contiguous()))
            add("add", n, ms, "additions")
            ms, pr = timed(lambda: api.haflo_scalar_mul_u64(pub, c, ks))
            add("scalar_mul (64-bit)", n, ms, "products")
            allc = torch.cat([c, s, pr], 0)
            ms, _ = timed(lambda: api.haflo_decrypt(own, allc))
            add("decrypt", 3 * n, ms, "decryptions")
        elif k in (2, 5):
            R, F = cfg["rows"], cfg["cols"]
            d = dev(synth.normal_f32(R, cfg["d_sigma"], synth.seed_for(k, 0)))
            Xf = dev(synth.normal_f32((R, F), 1.0, synth.seed_for(k, 1)))
            r = rand_words(R, lp, synth.seed_for(k, 2))
            ms, plain = timed(lambda: api.haflo_encode_f32(pub, d, cfg["scale_d"]))
            add("encode", R, ms, "values")
            ms, c = timed(lambda: api.haflo_encrypt(pub, plain, r))
            add("encrypt", R, ms, "encryptions")
            X = api.haflo_encode_exponents_f32(Xf, cfg["scale_x"])
            ms, out = timed(lambda: api.haflo_cipher_matvec(pub, 0, c, X))
            add("matvec X^T[[d]]", R * F, ms, "entries")
            ms, pl = timed(lambda: api.haflo_decrypt(own, out))
            add("decrypt", F, ms, "decryptions")
            ms, _ = timed(lambda: api.haflo_decode(own, pl, cfg["scale_d"] + cfg["scale_x"]))
            add("decode", F, ms, "values")
        elif k == 3:
            R, F = cfg["rows"], cfg["cols"]
            w = dev(synth.normal_f32(F, cfg["w_sigma"], synth.seed_for(3, 0)))
            Xf = synth.sparse_uniform_f32((R, F), cfg["zero_frac"], synth.seed_for(3, 1))
            r = rand_words(F, lp, synth.seed_for(3, 2))
            ms, c = timed(lambda: api.haflo_encrypt(pub, api.haflo_encode_f32(pub, w, cfg["scale_w"]), r))
            add("encode + encrypt weights", F, ms, "encryptions")
            X = api.haflo_encode_exponents_f32(dev(Xf), cfg["scale_x"])
            nnz = int((X != 0).sum().item())
            ms, out = timed(lambda: api.haflo_cipher_matvec(pub, 1, c, X))
            add("matvec X[[w]] (non-zero terms)", nnz, ms, "terms")
            ms, _ = timed(lambda: api.haflo_decrypt(own, out))
            add("decrypt", R, ms, "decryptions")
        elif k == 4:
            P, n = cfg["parties"], cfg["count"]
            vec = dev(synth.normal_f32(n, cfg["w_sigma"], synth.seed_for(4, 0)))
            r = rand_words(n, lp, synth.seed_for(4, 1))
            # the eight parties' vectors are the same size: one is encrypted and timed, the other
            # seven encryptions would take the same time each
            ms, c = timed(lambda: api.haflo_encrypt(pub, api.haflo_encode_f32(pub, vec, cfg["scale_w"]), r))
            add("encode + encrypt, one party's vector", n, ms, "encryptions")
            ms, c_own = timed(lambda: api.haflo_encrypt(own, api.haflo_encode_f32(own, vec, cfg["scale_w"]), r))
            add("the same by a key owner", n, ms, "encryptions")
            assert torch.equal(c, c_own)
            del c_own
            acc = c.clone()

            def fold():
                for _ in range(P - 1):
                    api.haflo_add(pub, acc, c, out=acc)
                return acc
            ms, s = timed(fold)
            add("add (7 folds)", (P - 1) * n, ms, "additions")
            ms, avg = timed(lambda: api.haflo_scalar_mul_i64_bcast(pub, s, 1 << (cfg["inv_parties_scale"] - 3)))
            add("scalar_mul by 2^21", n, ms, "products")
            ms, _ = timed(lambda: api.haflo_decrypt(own, avg))
            add("decrypt", n, ms, "decryptions")
        print("%s (%d-bit key)" % (cfg["name"], bits))
        for name, units, ms, unit in rows:
            print("  %-38s %12.3f ms  %14.4g %s/s" % (name, ms, units / (ms * 1e-3), unit))
        sys.stdout.flush()
        report[k] = [dict(op=n_, units=u, ms=ms, unit=un) for n_, u, ms, un in rows]
        own.close()
        pub.close()
        torch.cuda.empty_cache()
    if args.json:
        with open(args.json, "w") as fh:
            json.dump(report, fh, indent=1)


if __name__ == "__main__":
    main()
