#!/usr/bin/env python3
"""Roofline denominators measured on the GPU itself (libhaflo_peak.so, include/haflo_peak.h).

    python bench_peak.py [--iters 4096] [--gib 2] [--markdown]

Instruction streams (no memory traffic, 16 independent chains per lane) for the candidate limb
products - v_mad_u64_u32, v_mul_lo_u32 + v_mul_hi_u32, v_mul_u32_u24, FP64 FMA - and a plain 32-bit
add for reference, at 1, 2, 4 and 8 wavefronts per SIMD; then device fill, copy and read over a
buffer far larger than the caches. Every launch is timed with HIP events on the launch stream
(median of five after a warm-up). Prints one JSON line, or with --markdown the table that
profiles/peak_microbench.md holds.
"""
import argparse
import ctypes as C
import json
import os
import sys

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

NOMINAL_CLOCK_HZ = 2.4e9
NOMINAL_HBM_BYTES_PER_S = 8.0e12


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--iters", type=int, default=4096)
    ap.add_argument("--gib", type=float, default=2.0)
    ap.add_argument("--markdown", action="store_true")
    args = ap.parse_args()

    import torch

    from paper_2107_13797_amd import _cabi

    assert torch.cuda.is_available(), "bench_peak.py needs a GPU"
    path = os.path.join(ROOT, "paper_2107_13797_amd", "libhaflo_peak.so")
    if not os.path.exists(path):
        raise SystemExit("libhaflo_peak.so is missing: build it with `python -m paper_2107_13797_amd.build`")
    lib = _cabi.bind(C.CDLL(path), prototypes=_cabi.PEAK_PROTOTYPES)
    torch.cuda.set_device(0)
    props = torch.cuda.get_device_properties(0)
    cus = props.multi_processor_count
    streams = lib.haflo_peak_streams()
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)

    def timed(launch, reps=5):
        launch()
        torch.cuda.synchronize()
        times = []
        for _ in range(reps):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            rc = launch()
            e1.record()
            torch.cuda.synchronize()
            assert rc == 0
            times.append(e0.elapsed_time(e1))
        return sorted(times)[len(times) // 2]

    # (name, kind, VALU instructions per chain and iteration, all of them counted as operations)
    alu_kinds = [
        ("v_mad_u64_u32", _cabi.PEAK_MAD_U64_U32, 1, 1),
        ("v_mul_lo_u32, v_mul_hi_u32, v_add_u32", _cabi.PEAK_MUL_LO_HI, 3, 3),
        ("v_mad_u32_u24", _cabi.PEAK_MUL_U24, 1, 1),
        ("v_fma_f64", _cabi.PEAK_FMA_F64, 1, 1),
        ("v_add_u32", _cabi.PEAK_ADD_U32, 1, 1),
    ]
    full_rate = cus * 64 * NOMINAL_CLOCK_HZ  # lane-instructions per second at one per lane and clock
    out = {"device": props.name, "compute_units": cus, "streams_per_lane": streams, "iters": args.iters,
           "nominal_lane_ops_per_s": full_rate, "alu": [], "hbm": []}
    for name, kind, per_iter, valu_per_iter in alu_kinds:
        for wps in (1, 2, 4, 8):
            blocks = cus * wps  # a 256-lane workgroup is one wavefront on each of a compute unit's four SIMDs
            buf = torch.empty(blocks * 256, dtype=torch.int32, device="cuda")
            ms = timed(lambda: lib.haflo_peak_alu(kind, blocks, args.iters, C.c_void_p(buf.data_ptr()), stream))
            ops = blocks * 256 * args.iters * streams * per_iter
            rate = ops / (ms * 1e-3)
            out["alu"].append({"instruction": name, "waves_per_simd": wps, "ms": ms, "ops_per_s": rate,
                               "frac_of_nominal_full_rate": rate / full_rate,
                               "valu_instructions_per_op": valu_per_iter / per_iter})
    nbytes = int(args.gib * (1 << 30)) & ~15
    src = torch.empty(nbytes, dtype=torch.uint8, device="cuda").fill_(7)
    dst = torch.empty(nbytes, dtype=torch.uint8, device="cuda")
    for name, kind, moved in (("fill", _cabi.PEAK_FILL, 1), ("copy", _cabi.PEAK_COPY, 2), ("read", _cabi.PEAK_READ, 1)):
        best = None
        for per_cu in (1, 2, 4, 8, 16, 32):
            blocks = cus * per_cu
            ms = timed(lambda: lib.haflo_peak_hbm(kind, blocks, C.c_void_p(dst.data_ptr()), C.c_void_p(src.data_ptr()),
                                                  nbytes, stream))
            rate = moved * nbytes / (ms * 1e-3)
            if best is None or rate > best["bytes_per_s"]:
                best = {"kernel": name, "blocks_per_cu": per_cu, "ms": ms, "bytes_per_s": rate,
                        "frac_of_nominal": rate / NOMINAL_HBM_BYTES_PER_S, "buffer_gib": args.gib}
        out["hbm"].append(best)
    if not args.markdown:
        print(json.dumps(out))
        return
    print("device: %s, %d compute units; %d chains per lane, %d iterations" % (props.name, cus, streams, args.iters))
    print()
    print("| instruction stream | waves/SIMD | ms | 10^12 instructions/s | of 256 CU x 64 lanes x 2.4 GHz |")
    print("|---|---:|---:|---:|---:|")
    for r in out["alu"]:
        print("| %s | %d | %.3f | %.2f | %.3f |" % (r["instruction"], r["waves_per_simd"], r["ms"], r["ops_per_s"] / 1e12,
                                                   r["frac_of_nominal_full_rate"]))
    print()
    print("| HBM kernel (%.1f GiB) | blocks/CU | ms | TB/s | of 8 TB/s |" % args.gib)
    print("|---|---:|---:|---:|---:|")
    for r in out["hbm"]:
        print("| %s | %d | %.3f | %.2f | %.3f |" % (r["kernel"], r["blocks_per_cu"], r["ms"], r["bytes_per_s"] / 1e12,
                                                   r["frac_of_nominal"]))


if __name__ == "__main__":
    main()
