"""Glue for the GPU parity tests: host integers <-> device tensors."""
import numpy as np
import torch

from paper_2107_13797_amd import synth


def to_dev(arr):
    a = np.ascontiguousarray(arr)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    elif a.dtype == np.uint64:
        a = a.view(np.int64)
    return torch.from_numpy(a).cuda()


def ints_to_dev(xs, nlimbs):
    return to_dev(synth.ints_to_words(xs, nlimbs))


def dev_to_ints(t):
    return synth.words_to_ints(t.cpu().numpy())


def random_units_words(count, n_bits, seed):
    """count random integers in [0, 2^(n_bits-1)) as uint32 words [count, n_bits/32]: below any
    n of n_bits bits, and coprime to it except with negligible probability. For full-size
    batches where drawing Python integers one by one would dominate the test."""
    rng = np.random.default_rng(seed)
    w = rng.integers(0, 2 ** 32, size=(count, n_bits // 32), dtype=np.uint32)
    w[:, -1] &= 0x7FFFFFFF
    return w
