"""Seeded synthetic inputs shaped like the benchmark configurations.

Shared by the tests, the smoke check and the benchmark, for both the HIP path
and the CPU oracle. It holds no Paillier arithmetic: only random draws, the
workload shapes, and conversions between Python integers and the little-endian
32-bit-limb interchange format.

The paper evaluates on a public credit-card dataset that is not available
here; these generators stand in for it with the shapes the benchmark
configurations prescribe (feature matrices of tens to hundreds of columns,
mini-batch residual vectors, weight vectors). "N(0, s)" is read with s the
standard deviation.
"""
import math
import random

import numpy as np

BASE_SEED = 210713797

# The five benchmark configurations. scale_* are fixed-point fraction bits.
CONFIGS = {
    1: dict(name="cfg1: operator mix", n_bits=1024, count=1024),
    2: dict(name="cfg2: hetero-LR encrypted gradient X^T[[d]]", n_bits=1024, rows=4096, cols=32,
            d_sigma=0.25, scale_d=24, scale_x=16),
    3: dict(name="cfg3: encrypted forward pass X[[w]]", n_bits=2048, rows=16384, cols=256,
            w_sigma=0.1, zero_frac=0.7, scale_w=24, scale_x=16),
    4: dict(name="cfg4: homo-LR aggregation", n_bits=2048, parties=8, count=1000000,
            w_sigma=0.05, scale_w=24, inv_parties_scale=24),
    5: dict(name="cfg5: large-key hetero-LR gradient", n_bits=4096, rows=65536, cols=64,
            d_sigma=0.25, scale_d=24, scale_x=16),
}


def seed_for(cfg, stream=0):
    return BASE_SEED + 1000 * cfg + stream


def uniform_below(n, count, seed):
    """count integers uniform in [0, n)."""
    rng = random.Random(seed)
    return [rng.randrange(0, n) for _ in range(count)]


def units_below(n, count, seed):
    """count integers uniform in [1, n) that are coprime to n (encryption randomness)."""
    rng = random.Random(seed)
    out = []
    while len(out) < count:
        r = rng.randrange(1, n)
        if math.gcd(r, n) == 1:
            out.append(r)
    return out


def uniform_u64(count, seed):
    rng = random.Random(seed)
    return [rng.getrandbits(64) for _ in range(count)]


def normal_f32(shape, sigma, seed):
    return np.random.default_rng(seed).normal(0.0, sigma, size=shape).astype(np.float32)


def sparse_uniform_f32(shape, zero_frac, seed):
    """Entries zero with probability zero_frac, else uniform in (-1, 1)."""
    rng = np.random.default_rng(seed)
    vals = rng.uniform(-1.0, 1.0, size=shape).astype(np.float32)
    mask = rng.random(size=shape) < zero_frac
    vals[mask] = 0.0
    return vals


def ints_to_words(xs, nlimbs):
    """Python integers -> uint32 array [len(xs), nlimbs], little-endian limbs."""
    buf = b"".join(int(x).to_bytes(4 * nlimbs, "little") for x in xs)
    return np.frombuffer(buf, dtype="<u4").reshape(len(xs), nlimbs).copy()


def words_to_ints(arr):
    """uint32 (or raw int32) array [count, nlimbs] -> Python integers."""
    a = np.ascontiguousarray(arr).view(np.uint32) if arr.dtype != np.uint32 else np.ascontiguousarray(arr)
    a = a.astype("<u4", copy=False)
    nbytes = a.shape[1] * 4
    raw = a.tobytes()
    return [int.from_bytes(raw[i * nbytes:(i + 1) * nbytes], "little") for i in range(a.shape[0])]
