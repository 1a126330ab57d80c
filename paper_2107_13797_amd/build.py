"""Compile the HIP sources under csrc/ into libhaflo.so (gfx950) next to this file.

    python -m paper_2107_13797_amd.build

hipcc cross-compiles without a GPU. Objects go to paper_2107_13797_amd/_build/.
"""
import os
import subprocess
import sys
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "csrc")
OBJ = os.path.join(HERE, "_build")
LIB = os.path.join(HERE, "libhaflo.so")
PEAK_LIB = os.path.join(HERE, "libhaflo_peak.so")  # the roofline microbenchmarks, a library of their own
SOURCES = ["ctx.cpp", "staging.cpp", "store.cpp", "kernels_basic.hip", "kernels_modexp.hip", "kernels_matvec.hip", "kernels_buckets.hip", "kernels_loss.hip"]
PEAK_SOURCES = ["peak_microbench.hip", "limb_variants.hip"]
HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
FLAGS = [
    "-O3", "-std=c++17", "--offload-arch=gfx950", "-fPIC", "-x", "hip",
    # keep the compiler from forming packed FP32 instructions
    "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
]


def _compile(src):
    obj = os.path.join(OBJ, os.path.splitext(src)[0] + ".o")
    cmd = [HIPCC] + FLAGS + ["-c", os.path.join(CSRC, src), "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc failed on %s:\n%s" % (src, res.stderr[-4000:]))
    return obj


def build_library(verbose=True):
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(4, os.cpu_count() or 1)) as pool:
        objs = list(pool.map(_compile, SOURCES + PEAK_SOURCES))
    for lib, parts in ((LIB, objs[:len(SOURCES)]), (PEAK_LIB, objs[len(SOURCES):])):
        cmd = [HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", lib] + parts
        res = subprocess.run(cmd, capture_output=True, text=True)
        if res.returncode != 0:
            raise RuntimeError("link failed:\n%s" % res.stderr[-4000:])
        if verbose:
            print("built", lib)
    return LIB


if __name__ == "__main__":
    build_library()
    sys.exit(0)
