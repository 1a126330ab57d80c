"""Run oracle calls on several host cores (spawned workers that import only
the oracle, never torch or the HIP library)."""
import multiprocessing as mp
import os

from oracle import paillier_oracle as O


def workers():
    return max(1, min(16, os.cpu_count() or 1))


def _enc(args):
    n, m, r = args
    return O.encrypt(O.PublicKey(n), m, r)


def _dec(args):
    p, q, c = args
    return O.decrypt_crt(O.PrivateKey(p, q), c)


def _pow(args):
    n, c, k = args
    return O.scalar_mul(O.PublicKey(n), c, k)


def _matvec_cols(args):
    n, cs, cols = args
    pk = O.PublicKey(n)
    return [O.matvec(pk, 0, cs, [[x] for x in col])[0] for col in cols]


def _matvec_rows(args):
    n, cs, rows = args
    return O.matvec(O.PublicKey(n), 1, cs, rows)


_POOL = None


def pool():
    global _POOL
    if _POOL is None:
        _POOL = mp.get_context("spawn").Pool(workers())
    return _POOL


def pmap(fn, items, chunk=None):
    items = list(items)
    if len(items) < 4 or workers() == 1:
        return [fn(x) for x in items]
    if chunk is None:
        chunk = max(1, len(items) // (workers() * 4))
    return pool().map(fn, items, chunksize=chunk)


def encrypt_many(n, ms, rs):
    return pmap(_enc, [(n, m, r) for m, r in zip(ms, rs)])


def decrypt_many(p, q, cs):
    return pmap(_dec, [(p, q, c) for c in cs])


def pow_many(n, cs, ks):
    return pmap(_pow, [(n, c, k) for c, k in zip(cs, ks)])


def _split(items, parts):
    parts = max(1, min(parts, len(items)))
    size = (len(items) + parts - 1) // parts
    return [items[i:i + size] for i in range(0, len(items), size)]


def matvec_cols(n, cs, columns):
    """orientation 0 outputs, one per given column (each a list of len(cs) exponents)."""
    columns = list(columns)
    if not columns:
        return []
    chunks = _split(columns, workers())
    res = pmap(_matvec_cols, [(n, cs, ch) for ch in chunks], chunk=1)
    return [y for part in res for y in part]


def matvec_rows(n, cs, rows):
    """orientation 1 outputs, one per given row (each a list of len(cs) exponents)."""
    rows = list(rows)
    if not rows:
        return []
    chunks = _split(rows, workers() * 2)
    res = pmap(_matvec_rows, [(n, cs, ch) for ch in chunks], chunk=1)
    return [y for part in res for y in part]
