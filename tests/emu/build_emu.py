"""Build the CPU-emulated test library: the library's own sources compiled by
g++ against tests/emu/include (which shadows <hip/hip_runtime.h>).

HAFLO_EMU_SANITIZE=1 selects a second build with AddressSanitizer and
UndefinedBehaviorSanitizer (libhaflo_emu_san.so); the process that loads it
must have the sanitizer runtime preloaded, which tests/test_sanitizers.py does."""
import glob
import os
import subprocess
from concurrent.futures import ThreadPoolExecutor

HERE = os.path.dirname(os.path.abspath(__file__))
ROOT = os.path.dirname(os.path.dirname(HERE))
CSRC = os.path.join(ROOT, "paper_2107_13797_amd", "csrc")
SANITIZE = os.environ.get("HAFLO_EMU_SANITIZE", "") == "1"
OUT = os.path.join(HERE, "libhaflo_emu_san.so" if SANITIZE else "libhaflo_emu.so")
OBJ = os.path.join(HERE, "_build", "san" if SANITIZE else "plain")
SAN_FLAGS = ["-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer"]
OPT = ["-O1", "-g1"] + SAN_FLAGS if SANITIZE else ["-O2"]


def _compile(src):
    obj = os.path.join(OBJ, os.path.basename(src) + ".o")
    cmd = ["g++"] + OPT + ["-std=c++17", "-fPIC", "-Wno-unknown-pragmas", "-x", "c++", "-c",
                           "-I", os.path.join(HERE, "include"), "-I", os.path.join(ROOT, "include"), src, "-o", obj]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("emulation build failed on %s:\n%s" % (src, res.stderr[-4000:]))
    return obj


def build():
    srcs = [os.path.join(CSRC, "ctx.cpp"), os.path.join(CSRC, "staging.cpp"), os.path.join(CSRC, "store.cpp")] + sorted(glob.glob(os.path.join(CSRC, "kernels_*.hip")))
    srcs.append(os.path.join(HERE, "hipemu.cpp"))
    newest = max(os.path.getmtime(p) for p in srcs + glob.glob(os.path.join(CSRC, "*.hpp")) +
                 [os.path.join(HERE, "include", "hip", "hip_runtime.h"), os.path.join(ROOT, "include", "haflo.h"),
                  os.path.abspath(__file__)])
    if os.path.exists(OUT) and os.path.getmtime(OUT) >= newest:
        return OUT
    os.makedirs(OBJ, exist_ok=True)
    with ThreadPoolExecutor(max_workers=min(8, os.cpu_count() or 1)) as pool:
        objs = list(pool.map(_compile, srcs))
    cmd = ["g++", "-shared", "-fPIC"] + (SAN_FLAGS if SANITIZE else []) + objs + ["-o", OUT]
    res = subprocess.run(cmd, capture_output=True, text=True)
    if res.returncode != 0:
        raise RuntimeError("emulation link failed:\n" + res.stderr[-4000:])
    return OUT


if __name__ == "__main__":
    print(build())
