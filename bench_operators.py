#!/usr/bin/env python3
"""Per-operator throughput table in the shape of the paper's Table 2.

    python bench_operators.py [--bits 1024] [--instances 100000] [--json out.json]

For each operator of the paper's Table 2 (encoding, decoding, encryption,
decryption, multiplication, addition, matrix multiplication, summation) this
times `instances` elements at the given key size on one MI355X, inputs resident
in HBM, and prints instances per second next to the V100 figures the paper
reports for a 1024-bit key (context only: other hardware, unknown whether host
transfers were inside the paper's timings). `bench.py` remains the contract
benchmark; this is the operator-level view.
"""
import argparse
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# paper Table 2, GPU column (V100, 1024-bit key, 10^5 instances), instances per second
PAPER_V100_1024 = {
    "encoding": 15108620, "decoding": 22343405, "encryption": 83909, "decryption": 287273,
    "multiplication": 991946, "addition": 1226803, "matrix multiplication": 931942, "summation": 19575768,
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--bits", type=int, default=1024)
    ap.add_argument("--instances", type=int, default=100000)
    ap.add_argument("--features", type=int, default=32)
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--tall", action="store_true", help="also time X^T[[d]] on an instances x features matrix")
    ap.add_argument("--memory-side", action="store_true",
                    help="time only the operators with little arithmetic per byte (encode, decode, import, export, "
                         "add) and print bytes and multiply-adds per second against both rooflines")
    ap.add_argument("--json", default=None)
    args = ap.parse_args()

    import numpy as np
    import torch

    from paper_2107_13797_amd import api, synth

    assert torch.cuda.is_available(), "needs a GPU"
    bits, N, F = args.bits, args.instances, args.features
    seed = synth.BASE_SEED + bits
    p, q = api.haflo_keygen(bits, seed)
    own = api.haflo_ctx_create_private(p, q, bits)
    pub = api.haflo_ctx_create_public(p * q, bits)
    lp = bits // 32

    def dev(a):
        a = np.ascontiguousarray(a)
        if a.dtype == np.uint32:
            a = a.view(np.int32)
        elif a.dtype == np.uint64:
            a = a.view(np.int64)
        return torch.from_numpy(a).cuda()

    if args.memory_side:
        return memory_side(args, api, synth, torch, np, own, dev)
    rng = np.random.default_rng(seed)
    v = dev(synth.normal_f32(N, 0.25, seed + 1))
    r_words = rng.integers(0, 2 ** 32, size=(N, lp), dtype=np.uint32)
    r_words[:, -1] &= 0x7FFFFFFF
    r = dev(r_words)
    k64 = dev(rng.integers(0, 2 ** 63, size=N, dtype=np.uint64) * 2 + 1)
    rows = max(1, N // F)
    X = api.haflo_encode_exponents_f32(dev(synth.normal_f32((rows, F), 1.0, seed + 2)), 16)

    def timed(fn):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.reps):
            out = fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / args.reps * 1e-3, out

    res = {}
    t, plain = timed(lambda: api.haflo_encode_f32(pub, v, 24))
    res["encoding"] = N / t
    t, c = timed(lambda: api.haflo_encrypt(pub, plain, r))
    res["encryption"] = N / t
    t, _ = timed(lambda: api.haflo_encrypt(own, plain, r))
    res["encryption (key owner)"] = N / t
    t, _ = timed(lambda: api.haflo_encrypt_with_obfuscator(pub, plain, c))
    res["encryption (precomputed r^n)"] = N / t
    t, pl = timed(lambda: api.haflo_decrypt(own, c))
    res["decryption"] = N / t
    t, _ = timed(lambda: api.haflo_decode(own, pl, 24))
    res["decoding"] = N / t
    t, _ = timed(lambda: api.haflo_scalar_mul_u64(pub, c, k64))
    res["multiplication"] = N / t
    t, _ = timed(lambda: api.haflo_add(pub, c, c))
    res["addition"] = N / t
    t, _ = timed(lambda: api.haflo_cipher_matvec(pub, 0, c[:rows].contiguous(), X))
    res["matrix multiplication"] = rows * F / t
    if args.tall:
        # a tall matrix (the shape of the encrypted gradient of a large mini-batch): the bucket method
        tall = api.haflo_encode_exponents_f32(dev(synth.normal_f32((N, F), 1.0, seed + 3)), 16)
        t, _ = timed(lambda: api.haflo_cipher_matvec(pub, 0, c, tall))
        res["matrix multiplication (%d x %d)" % (N, F)] = N * F / t
    label = dev(np.where(rng.random(N) < 0.5, -1.0, 1.0).astype(np.float32))
    t, _ = timed(lambda: api.haflo_fore_gradient(pub, c, v, label, r, 24))
    res["fore gradient (fused)"] = N / t
    t, _ = timed(lambda: api.haflo_cipher_sum(pub, c))
    res["summation"] = N / t

    print("%-26s %16s %16s %8s" % ("operator (%d-bit key)" % bits, "MI355X inst/s", "paper V100 inst/s", "ratio"))
    for name, rate in res.items():
        ref = PAPER_V100_1024.get(name) if bits == 1024 else None
        print("%-26s %16.0f %16s %8s" % (name, rate, ref if ref else "-", ("%.1f" % (rate / ref)) if ref else "-"))
    if args.json:
        with open(args.json, "w") as fh:
            json.dump({"n_bits": bits, "instances": N, "features": F, "instances_per_s": res}, fh, indent=1)


def memory_side(args, api, synth, torch, np, ctx, dev):
    """encode / decode (HBM-bound) and import / export / add (one Montgomery product per element) on
    `--instances` resident elements: milliseconds (median of --reps launches after a warm-up),
    algorithmic bytes per second against 8 TB/s, multiply-adds per second against 39.3e12."""
    import statistics
    bits, N = args.bits, args.instances
    lp, lc = bits // 32, bits // 16
    internal = ctx.cipher_words * 4
    seed = synth.BASE_SEED + bits
    rng = np.random.default_rng(seed)
    v = dev(synth.normal_f32(N, 0.25, seed + 1))
    canon = torch.from_numpy(rng.integers(0, 2 ** 32, size=(N, lc), dtype=np.uint32).view(np.int32)).cuda()
    canon[:, -1] &= 0x3FFFFFFF  # below 2^(2 bits - 2) < n^2

    def timed(fn):
        out = fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(max(3, args.reps)):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            out = fn()
            e1.record()
            torch.cuda.synchronize()
            ts.append(e0.elapsed_time(e1))
        return statistics.median(ts) * 1e-3, out

    mad = 2 * lc * lc + lc
    rows = []
    st = torch.zeros(N, dtype=torch.int32, device="cuda")
    t, plain = timed(lambda: api.haflo_encode_f32(ctx, v, 24, st))
    rows.append(("k_encode", t, 4 + 4 * lp + 4, 0))
    t, _ = timed(lambda: api.haflo_decode(ctx, plain, 24, st))
    rows.append(("k_decode", t, 4 * lp + 20, 0))
    t, c = timed(lambda: api.haflo_import_cipher(ctx, canon))
    rows.append(("k_import", t, 4 * lc + internal, mad))
    t, _ = timed(lambda: api.haflo_export_cipher(ctx, c))
    rows.append(("k_export", t, 4 * lc + internal, mad))
    dst = torch.empty_like(c)
    t, _ = timed(lambda: api.haflo_add(ctx, c, c, out=dst))
    rows.append(("k_add", t, 3 * internal, mad))
    print("%d-bit key, %d elements" % (bits, N))
    print("| kernel | ms | bytes/element | TB/s | of 8 TB/s | 10^12 mul32/s | of 39.3 |")
    print("|---|---:|---:|---:|---:|---:|---:|")
    for name, t, nbytes, m in rows:
        print("| %s | %.3f | %d | %.2f | %.3f | %s | %s |" % (
            name, t * 1e3, nbytes, N * nbytes / t / 1e12, N * nbytes / t / 8e12,
            ("%.1f" % (N * m / t / 1e12)) if m else "-", ("%.3f" % (N * m / t / 39.3216e12)) if m else "-"))
    if args.json:
        with open(args.json, "w") as fh:
            json.dump({"n_bits": bits, "elements": N,
                       "kernels": {name: {"ms": t * 1e3, "bytes_per_element": nbytes, "mul32_per_element": m}
                                   for name, t, nbytes, m in rows}}, fh, indent=1)


if __name__ == "__main__":
    main()
