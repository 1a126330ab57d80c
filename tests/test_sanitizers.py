"""Sanitizer leg of the CPU build: the library's own sources (host code and the kernels stepped by
the CPU stand-in for the HIP runtime) compiled with AddressSanitizer and
UndefinedBehaviorSanitizer, running the store, host big-integer and a subset of the emulated
kernel tests in a child process that has the sanitizer runtime preloaded. Nothing of this runs
on a GPU.

The same by hand, over every emulated test:

    HAFLO_EMU_SANITIZE=1 LD_PRELOAD=$(gcc -print-file-name=libasan.so) ASAN_OPTIONS=detect_leaks=0 \
        python -m pytest tests/test_emu_kernels.py tests/test_emu_store.py tests/test_hostbig.py -q
"""
import os
import subprocess
import sys

import pytest

from conftest import ROOT

# the emulated kernel tests that touch the most pointer arithmetic for the least time
KERNEL_SUBSET = ("import_export_add or encrypt_decrypt_scalar or summation_segments or bucket_matvec_random "
                 "or host_staging or encode_decode")


def _asan_runtime():
    try:
        path = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True, check=True).stdout.strip()
    except (OSError, subprocess.CalledProcessError):
        return None
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_emulated_library_under_asan_and_ubsan():
    asan = _asan_runtime()
    if asan is None:
        pytest.skip("no AddressSanitizer runtime next to gcc")
    env = dict(os.environ)
    env.update({
        "HAFLO_EMU_SANITIZE": "1",
        "LD_PRELOAD": asan,
        # Python itself leaks by design; the fibers of the emulated runtime switch stacks
        "ASAN_OPTIONS": "detect_leaks=0:detect_stack_use_after_return=0:abort_on_error=1",
        "UBSAN_OPTIONS": "print_stacktrace=1:halt_on_error=1",
    })
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider",
           os.path.join(ROOT, "tests", "test_hostbig.py"), os.path.join(ROOT, "tests", "test_emu_store.py"),
           os.path.join(ROOT, "tests", "test_emu_kernels.py"), "-k",
           "(hostbig or store or ring or " + KERNEL_SUBSET + ") and not long_chunks"]
    res = subprocess.run(cmd, capture_output=True, text=True, cwd=ROOT, env=env)
    tail = (res.stdout + res.stderr)[-6000:]
    assert res.returncode == 0, tail
    assert "AddressSanitizer" not in tail and "runtime error" not in tail, tail
