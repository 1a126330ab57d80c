#!/usr/bin/env python3
"""Alternative limb widths for the Montgomery product, timed against the shipped core
(libhaflo_peak.so, include/haflo_peak.h: haflo_peak_montmul_chain).

    python bench_limbs.py [--lanes-per-simd 256] [--iters 64] [--markdown]

One big integer per lane, a 510-bit modulus, `iters` dependent products per lane; every variant's
results are first checked against Python integers (x y^iters / R^iters mod n), then timed with HIP
events (median of five launches). Reported per variant: nanoseconds per product and lane slot,
products per second over the chip, and the same normalised by modulus bits squared, which is what
a longer modulus would scale by.
"""
import argparse
import ctypes as C
import json
import os
import random
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

MOD_BITS = 510


def pack(values, limbs, bits, as_double):
    import numpy as np
    out = np.zeros((len(values), limbs), dtype=np.float64 if as_double else np.uint32)
    mask = (1 << bits) - 1
    for i, v in enumerate(values):
        for j in range(limbs):
            out[i, j] = (v >> (bits * j)) & mask
    return out


def unpack(arr, bits):
    return [sum(int(w) << (bits * j) for j, w in enumerate(row)) for row in arr]


def variants(cabi):
    return [("29-bit limbs, v_mad_u64_u32 (shipped core)", cabi.LIMBS_29_MAD64, False),
            ("29-bit limbs, squaring without the symmetric half (shipped)", cabi.LIMBS_29_MAD64_SQUARE, True),
            ("24-bit limbs, v_mul_u32_u24 + v_mul_hi_u32_u24", cabi.LIMBS_24_MUL24, False),
            ("23-bit limbs in doubles, v_fma_f64", cabi.LIMBS_23_FMA64, False)]


def run(lib, torch, np, cabi, kind, square, n, xs, ys, iters, reps=5):
    """-> (results as integers modulo n, median ms)"""
    limbs, bits = C.c_uint32(), C.c_uint32()
    assert lib.haflo_peak_limbs(kind, C.byref(limbs), C.byref(bits)) == 0
    L, b = limbs.value, bits.value
    dbl = kind == cabi.LIMBS_23_FMA64
    dx = torch.from_numpy(pack(xs, L, b, dbl)).cuda()
    dy = torch.from_numpy(pack(ys, L, b, dbl)).cuda()
    dn = torch.from_numpy(pack([n], L, b, dbl)).cuda()
    if not dbl:
        dx, dy, dn = dx.view(torch.int32), dy.view(torch.int32), dn.view(torch.int32)
    out = torch.empty_like(dx)
    n0inv = (-pow(n, -1, 1 << b)) % (1 << b)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def launch():
        return lib.haflo_peak_montmul_chain(kind, C.c_void_p(dx.data_ptr()), C.c_void_p(dy.data_ptr()),
                                            C.c_void_p(dn.data_ptr()), n0inv, iters, C.c_void_p(out.data_ptr()),
                                            len(xs), stream)
    assert launch() == 0
    torch.cuda.synchronize()
    times = []
    for _ in range(reps):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        assert launch() == 0
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1))
    host = out.cpu().numpy()
    if not dbl:
        host = host.view(np.uint32)
    return [v % n for v in unpack(host, b)], sorted(times)[len(times) // 2], L * b


def expected(n, xs, ys, iters, rbits, square):
    rinv = pow(1 << rbits, -1, n)
    want = []
    for x, y in zip(xs, ys):
        v = x
        for _ in range(iters):
            v = v * (v if square else y) * rinv % n
        want.append(v)
    return want


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--lanes-per-simd", type=int, default=256, help="integers per SIMD (64 = one wavefront)")
    ap.add_argument("--iters", type=int, default=64)
    ap.add_argument("--markdown", action="store_true")
    args = ap.parse_args()

    import numpy as np
    import torch

    from paper_2107_13797_amd import _cabi

    assert torch.cuda.is_available(), "bench_limbs.py needs a GPU"
    path = os.path.join(ROOT, "paper_2107_13797_amd", "libhaflo_peak.so")
    if not os.path.exists(path):
        raise SystemExit("libhaflo_peak.so is missing: build it with `python -m paper_2107_13797_amd.build`")
    lib = _cabi.bind(C.CDLL(path), prototypes=_cabi.PEAK_PROTOTYPES)
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    count = cus * 4 * args.lanes_per_simd
    rng = random.Random(2107)
    n = rng.getrandbits(MOD_BITS) | (1 << (MOD_BITS - 1)) | 1
    check = 64
    xs = [rng.randrange(n) for _ in range(check)] + [0] * (count - check)
    ys = [rng.randrange(n) for _ in range(check)] + [0] * (count - check)
    for i in range(check, count):  # cheap distinct fillers for the lanes that are only timed
        xs[i] = (xs[i % check] + i) % n
        ys[i] = (ys[i % check] ^ i) % n
    rows = []
    for name, kind, square in variants(_cabi):
        got, ms, rbits = run(lib, torch, np, _cabi, kind, square, n, xs, ys, args.iters)
        want = expected(n, xs[:check], ys[:check], args.iters, rbits, square)
        assert got[:check] == want, "variant %r disagrees with Python integers" % name
        per_s = count * args.iters / (ms * 1e-3)
        rows.append({"variant": name, "limbs_x_bits": rbits, "ms": ms, "products_per_s": per_s,
                     "ns_per_product_per_lane": ms * 1e6 / args.iters / args.lanes_per_simd * 64 / 64,
                     "modulus_bits2_per_ns": per_s * MOD_BITS * MOD_BITS / 1e9})
    base = rows[0]["products_per_s"]
    for r in rows:
        r["relative_to_shipped_product"] = r["products_per_s"] / base
    if not args.markdown:
        print(json.dumps({"modulus_bits": MOD_BITS, "integers": count, "iters": args.iters, "variants": rows}))
        return
    print("%d-bit modulus, %d integers (one per lane, %d per SIMD), %d dependent products each; all variants agree "
          "with Python integers on %d sampled lanes" % (MOD_BITS, count, args.lanes_per_simd, args.iters, check))
    print()
    print("| variant | radix bits | ms | 10^9 products/s | relative |")
    print("|---|---:|---:|---:|---:|")
    for r in rows:
        print("| %s | %d | %.3f | %.2f | %.2f |" % (r["variant"], r["limbs_x_bits"], r["ms"], r["products_per_s"] / 1e9,
                                                 r["relative_to_shipped_product"]))


if __name__ == "__main__":
    main()
