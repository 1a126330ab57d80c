"""The limb-width variants of the Montgomery product in the measurement library (29-bit limbs in
64-bit columns: the shipped core; 24-bit limbs; 23-bit limbs in doubles) must all compute
x y^k / R^k mod n: compared with Python integers, through the C boundary of libhaflo_peak.so."""
import ctypes as C
import os
import random

import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from conftest import ROOT  # noqa: E402
from paper_2107_13797_amd import _cabi  # noqa: E402


def test_limb_variants_agree_with_python_integers():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    import numpy as np

    import bench_limbs
    lib = _cabi.bind(C.CDLL(os.path.join(ROOT, "paper_2107_13797_amd", "libhaflo_peak.so")), prototypes=_cabi.PEAK_PROTOTYPES)
    rng = random.Random(77)
    for bits in (510, 505):
        n = rng.getrandbits(bits) | (1 << (bits - 1)) | 1
        xs = [0, 1, n - 1] + [rng.randrange(n) for _ in range(300)]
        ys = [n - 1, n - 1, n - 1] + [rng.randrange(n) for _ in range(300)]
        for iters in (1, 5):
            for name, kind, square in bench_limbs.variants(_cabi):
                got, _, rbits = bench_limbs.run(lib, torch, np, _cabi, kind, square, n, xs, ys, iters, reps=1)
                assert got == bench_limbs.expected(n, xs, ys, iters, rbits, square), (name, bits, iters)
