#!/usr/bin/env python3
"""Wall time of the five benchmark configurations, operator by operator, with the fraction of the
roofline that bounds each operator.

    python bench_configs.py [--configs 1,2,3,4,5] [--reps 3] [--json out.json]

Each configuration of `paper_2107_13797_amd.synth.CONFIGS` is generated with its seeded inputs,
made resident in HBM, and its operators are timed with HIP events on the launch stream (median of
`--reps` runs after one warm-up). `bench.py` calls `run_configs` with one repetition for the
`configs` object of its JSON line; the parity of the same configurations with the oracle is what
`tests/test_gpu_parity.py` checks.

Roofline fractions. Operators built on Montgomery products are bound by the issue rate of the
32x32+64-bit integer multiply-add, 256 compute units x 64 lanes x 2.4 GHz = 39.3e12 per second;
their algorithmic work is (Montgomery products of the library's schedule) x (2 L^2 + L), L the
32-bit limbs of the modulus, squarings counted like general products. For the matrix products the
schedule's products are one per non-zero digit of every entry (signed base-1024 digits for
X^T [[d]] with buckets, signed base-32 digits with tables, base-256 digits for X [[w]]), counted
from the matrix itself. Encode and decode are bound by HBM (8 TB/s) and move 4 + 4 Lp + 4 and
4 Lp + 20 bytes per element. That is the conventional accounting. The exponentiation kernels execute
fewer multiply-adds than it counts (squarings without the symmetric half, arithmetic modulo n^2 on pairs
of half-length residues: 0.57 - 0.63 of them), so `frac` can exceed what the instruction stream itself can
reach (0.66 of the peak at four wavefronts per SIMD) and even 1.0 at a 4096-bit key; rows of a chip-filling
encryption or decryption therefore also carry `frac_executed`, the multiply-adds really issued per second
against the same peak (`haflo_op_work`).
"""
import argparse
import json
import os
import statistics
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_MAD32_PER_S = 256 * 64 * 2.4e9
PEAK_HBM_BYTES_PER_S = 8.0e12


def montmul_mul32(limbs):
    """32x32->64 multiply-adds of one word-serial Montgomery product on `limbs` 32-bit limbs."""
    return 2 * limbs * limbs + limbs


def nonzero_digits_signed(X, torch, digit_bits, positions):
    """Non-zero digits of |x| + c written in base 2^digit_bits with each digit minus half the base
    (the signed-digit form both X^T [[d]] methods use), summed over the matrix."""
    base = 1 << digit_bits
    offset = 0
    for _ in range(positions):
        offset = offset * base + base // 2
    mag = X.to(torch.int64).abs()
    shifted = mag + offset
    total = 0
    for s in range(positions):
        d = ((shifted >> (digit_bits * s)) & (base - 1)) - base // 2
        total += int(((d != 0) & (mag != 0)).sum().item())
    return total


def positions_needed(maxmag, digit_bits, max_positions):
    base = 1 << digit_bits
    offset = 0
    for s in range(1, max_positions):
        offset = offset * base + base // 2
        if maxmag + offset < base ** s:
            return s
    return max_positions


def run_configs(which=(1, 2, 3, 4, 5), reps=3, verbose=True):
    """-> {cfg: [ {op, units, unit, ms, rate, bound, frac, note}, ... ]}"""
    import numpy as np
    import torch

    from paper_2107_13797_amd import _cabi, api, synth

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
        for _ in range(reps):
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
    for k in which:
        cfg = synth.CONFIGS[k]
        bits = cfg["n_bits"]
        lp, lc = bits // 32, bits // 16
        p, q = api.haflo_keygen(bits, synth.BASE_SEED + bits)
        own = api.haflo_ctx_create_private(p, q, bits)
        pub = api.haflo_ctx_create_public(p * q, bits)
        enc_mm, enc_limbs = api.haflo_op_cost(pub, _cabi.OP_ENCRYPT)
        own_mm, own_limbs = api.haflo_op_cost(own, _cabi.OP_ENCRYPT)
        dec_mm, dec_limbs = api.haflo_op_cost(own, _cabi.OP_DECRYPT)
        enc_work, own_work = api.haflo_op_work(pub, _cabi.OP_ENCRYPT), None  # defined for the public route
        dec_work = api.haflo_op_work(own, _cabi.OP_DECRYPT)
        rows = []

        def alu(name, units, ms, unit, products_per_unit, limbs, note="", executed_per_unit=None):
            mad = units * products_per_unit * montmul_mul32(limbs)
            row = dict(op=name, units=units, unit=unit, ms=ms, rate=units / (ms * 1e-3), bound="alu",
                       frac=mad / (ms * 1e-3) / PEAK_MAD32_PER_S,
                       note=note or "%g Montgomery products of %d limbs per unit" % (products_per_unit, limbs))
            if executed_per_unit is not None:
                row["frac_executed"] = units * executed_per_unit / (ms * 1e-3) / PEAK_MAD32_PER_S
            rows.append(row)

        def hbm(name, units, ms, unit, bytes_per_unit):
            rows.append(dict(op=name, units=units, unit=unit, ms=ms, rate=units / (ms * 1e-3), bound="hbm",
                             frac=units * bytes_per_unit / (ms * 1e-3) / PEAK_HBM_BYTES_PER_S,
                             note="%d bytes per unit" % bytes_per_unit))

        if k == 1:
            n = cfg["count"]
            m, r = rand_words(n, lp, synth.seed_for(1, 0), 0x3FFFFFFF), rand_words(n, lp, synth.seed_for(1, 1))
            ks = dev(np.random.default_rng(synth.seed_for(1, 2)).integers(0, 2 ** 63, size=n, dtype=np.uint64))
            ms, c = timed(lambda: api.haflo_encrypt(pub, m, r))
            alu("encrypt", n, ms, "encryptions", enc_mm, enc_limbs)
            ms, s = timed(lambda: api.haflo_add(pub, c, torch.roll(c, -1, 0).contiguous()))
            alu("add", n, ms, "additions", 1, lc)
            ms, pr = timed(lambda: api.haflo_scalar_mul_u64(pub, c, ks))
            # table c^2..c^15 (14 products), 15 windows of four squarings and one product
            alu("scalar_mul (64-bit)", n, ms, "products", 14 + 15 * 5, lc)
            allc = torch.cat([c, s, pr], 0)
            ms, _ = timed(lambda: api.haflo_decrypt(own, allc))
            alu("decrypt", 3 * n, ms, "decryptions", dec_mm, dec_limbs)
        elif k in (2, 5):
            R, F = cfg["rows"], cfg["cols"]
            d = dev(synth.normal_f32(R, cfg["d_sigma"], synth.seed_for(k, 0)))
            Xf = dev(synth.normal_f32((R, F), 1.0, synth.seed_for(k, 1)))
            r = rand_words(R, lp, synth.seed_for(k, 2))
            ms, plain = timed(lambda: api.haflo_encode_f32(pub, d, cfg["scale_d"]))
            hbm("encode", R, ms, "values", 4 + 4 * lp + 4)
            ms, c = timed(lambda: api.haflo_encrypt(pub, plain, r))
            big = k == 5  # a chip-filling batch: the kernels of haflo_op_work
            alu("encrypt", R, ms, "encryptions", enc_mm, enc_limbs, executed_per_unit=enc_work if big else None)
            ms, c_own = timed(lambda: api.haflo_encrypt(own, plain, r))
            alu("encrypt (key owner)", R, ms, "encryptions", own_mm, own_limbs,
                executed_per_unit=own_work)
            assert torch.equal(c, c_own)
            del c_own
            X = api.haflo_encode_exponents_f32(Xf, cfg["scale_x"])
            maxmag = int(X.to(torch.int64).abs().max().item())
            buckets = R >= 4096
            if buckets:
                digits = nonzero_digits_signed(X, torch, 10, 4)
            else:
                digits = nonzero_digits_signed(X, torch, 5, positions_needed(maxmag, 5, 7))
            ms, out = timed(lambda: api.haflo_cipher_matvec(pub, 0, c, X))
            alu("matvec X^T[[d]]", R * F, ms, "entries", digits / (R * F), lc,
                "%s method, %.2f non-zero digits (one product each) per entry" % ("bucket" if buckets else "table", digits / (R * F)))
            ms, pl = timed(lambda: api.haflo_decrypt(own, out))
            alu("decrypt", F, ms, "decryptions", dec_mm, dec_limbs)
            ms, _ = timed(lambda: api.haflo_decode(own, pl, cfg["scale_d"] + cfg["scale_x"]))
            hbm("decode", F, ms, "values", 4 * lp + 20)
        elif k == 3:
            R, F = cfg["rows"], cfg["cols"]
            w = dev(synth.normal_f32(F, cfg["w_sigma"], synth.seed_for(3, 0)))
            Xf = synth.sparse_uniform_f32((R, F), cfg["zero_frac"], synth.seed_for(3, 1))
            r = rand_words(F, lp, synth.seed_for(3, 2))
            ms, c = timed(lambda: api.haflo_encrypt(pub, api.haflo_encode_f32(pub, w, cfg["scale_w"]), r))
            alu("encode + encrypt weights", F, ms, "encryptions", enc_mm, enc_limbs)
            X = api.haflo_encode_exponents_f32(dev(Xf), cfg["scale_x"])
            nnz = int((X != 0).sum().item())
            mag = X.to(torch.int64).abs()
            digits = sum(int((((mag >> (8 * s)) & 255) != 0).sum().item()) for s in range(4))
            ms, out = timed(lambda: api.haflo_cipher_matvec(pub, 1, c, X))
            alu("matvec X[[w]] (non-zero terms)", nnz, ms, "terms", digits / max(nnz, 1), lc,
                "%.2f non-zero base-256 digits (one product each) per non-zero entry" % (digits / max(nnz, 1)))
            ms, _ = timed(lambda: api.haflo_decrypt(own, out))
            alu("decrypt", R, ms, "decryptions", dec_mm, dec_limbs, executed_per_unit=dec_work)
        elif k == 4:
            P, n = cfg["parties"], cfg["count"]
            vec = dev(synth.normal_f32(n, cfg["w_sigma"], synth.seed_for(4, 0)))
            r = rand_words(n, lp, synth.seed_for(4, 1))
            # the eight parties' vectors are the same size: one is encrypted and timed, the other
            # seven encryptions would take the same time each
            ms, c = timed(lambda: api.haflo_encrypt(pub, api.haflo_encode_f32(pub, vec, cfg["scale_w"]), r))
            alu("encode + encrypt, one party's vector", n, ms, "encryptions", enc_mm, enc_limbs, executed_per_unit=enc_work)
            ms, c_own = timed(lambda: api.haflo_encrypt(own, api.haflo_encode_f32(own, vec, cfg["scale_w"]), r))
            alu("the same by a key owner", n, ms, "encryptions", own_mm, own_limbs, executed_per_unit=own_work)
            assert torch.equal(c, c_own)
            del c_own
            acc = c.clone()

            def fold():
                for _ in range(P - 1):
                    api.haflo_add(pub, acc, c, out=acc)
                return acc
            ms, s = timed(fold)
            alu("add (7 folds)", (P - 1) * n, ms, "additions", 1, lc)
            ms, avg = timed(lambda: api.haflo_scalar_mul_i64_bcast(pub, s, 1 << (cfg["inv_parties_scale"] - 3)))
            alu("scalar_mul by 2^21", n, ms, "products", cfg["inv_parties_scale"] - 3, lc,
                "21 squarings of %d limbs per unit" % lc)
            ms, _ = timed(lambda: api.haflo_decrypt(own, avg))
            alu("decrypt", n, ms, "decryptions", dec_mm, dec_limbs, executed_per_unit=dec_work)
        if verbose:
            print("%s (%d-bit key)" % (cfg["name"], bits))
            for row in rows:
                print("  %-38s %12.3f ms  %14.4g %s/s  %5.1f %% of the %s roofline%s" %
                      (row["op"], row["ms"], row["rate"], row["unit"], 100 * row["frac"], row["bound"],
                       " (%.1f %% in executed multiply-adds)" % (100 * row["frac_executed"])
                       if "frac_executed" in row else ""))
            sys.stdout.flush()
        report[k] = rows
        own.close()
        pub.close()
        del own, pub
        torch.cuda.empty_cache()
    return report


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="1,2,3,4,5")
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--json", default=None)
    args = ap.parse_args()
    report = run_configs([int(x) for x in args.configs.split(",")], args.reps)
    if args.json:
        with open(args.json, "w") as fh:
            json.dump(report, fh, indent=1)


if __name__ == "__main__":
    main()
