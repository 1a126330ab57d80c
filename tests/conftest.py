import os
import sys


ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def pytest_configure(config):
    config.addinivalue_line("markers", "gpu: needs a real MI355X (runs through the C boundary of libhaflo)")


_KEYS = {}


def oracle_key(n_bits, seed=None):
    """(p, q) from the oracle's deterministic key generation, cached per process."""
    from oracle import paillier_oracle as O
    from paper_2107_13797_amd import synth
    if seed is None:
        seed = synth.BASE_SEED + n_bits
    k = (n_bits, seed)
    if k not in _KEYS:
        _KEYS[k] = O.keygen(n_bits, seed)
    return _KEYS[k]
