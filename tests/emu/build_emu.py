"""Build the CPU-emulated test library: the library's own sources compiled by
g++ against tests/emu/include (which shadows <hip/hip_runtime.h>)."""
import glob
import os
import subprocess

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_2107_13797_amd", "csrc")
OUT = os.path.join(HERE, "libhaflo_emu.so")


def build():
    srcs = [os.path.join(CSRC, "ctx.cpp"), os.path.join(CSRC, "staging.cpp"), os.path.join(CSRC, "store.cpp")] + sorted(glob.glob(os.path.join(CSRC, "kernels_*.hip")))
    srcs.append(os.path.join(HERE, "hipemu.cpp"))
    newest = max(os.path.getmtime(p) for p in srcs + glob.glob(os.path.join(CSRC, "*.hpp")) +
                 [os.path.join(HERE, "include", "hip", "hip_runtime.h")])
    if os.path.exists(OUT) and os.path.getmtime(OUT) >= newest:
        return OUT
    cmd = ["g++", "-O2", "-std=c++17", "-fPIC", "-shared", "-Wno-unknown-pragmas", "-x", "c++",
           "-I", os.path.join(HERE, "include"), "-I", os.path.join(ROOT, "include")] + srcs + ["-o", OUT]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("emulation build failed:\n" + res.stderr[-4000:])
    return OUT


if __name__ == "__main__":
    print(build())
