"""Thin binding over the C boundary of libhaflo (include/haflo.h).

Same names as the C entry points, argument marshalling only: tensors are
allocated with torch on the current CUDA(HIP) device, their data pointers and
the current torch stream are passed through, and every step runs in the
library's kernels. Big-integer arrays travel as int32 tensors holding the raw
32-bit words (little-endian limbs, item-major).
"""
import ctypes as C
import os

import torch

from . import _cabi

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libhaflo.so")
_lib = None


class HafloError(RuntimeError):
    pass


def lib():
    """The loaded library; raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise HafloError(
                "libhaflo.so is missing: build it with `python -m paper_2107_13797_amd.build` "
                "(there is no CPU fallback)")
        _lib = _cabi.bind(C.CDLL(_LIB_PATH))
    return _lib


def _check(rc):
    if rc != 0:
        raise HafloError("libhaflo: %s (code %d)" % (lib().haflo_strerror(rc).decode(), rc))


def _stream():
    return C.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise HafloError("expected a contiguous CUDA tensor")
    return C.c_void_p(t.data_ptr())


def _le(x, nbytes):
    return (C.c_uint8 * nbytes).from_buffer_copy(int(x).to_bytes(nbytes, "little"))


class Context:
    """Owner of a haflo_ctx plus a growable workspace tensor."""

    def __init__(self, handle):
        self.handle = handle
        nb, lc, lp = C.c_uint32(), C.c_uint32(), C.c_uint32()
        cb, pb = C.c_size_t(), C.c_size_t()
        _check(lib().haflo_ctx_info(handle, C.byref(nb), C.byref(lc), C.byref(lp), C.byref(cb), C.byref(pb)))
        self.n_bits, self.cipher_limbs, self.plain_limbs = nb.value, lc.value, lp.value
        self.cipher_words = cb.value // 4  # int32 words of one internal ciphertext
        self._ws = None

    def workspace(self, nbytes):
        if nbytes == 2 ** 64 - 1:
            raise HafloError("bad workspace query")
        need = max(nbytes, 256)
        if self._ws is None or self._ws.numel() < need:
            self._ws = None
            self._ws = torch.empty(need, dtype=torch.uint8, device="cuda")
        return self._ws

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize()
            lib().haflo_ctx_destroy(self.handle)
            self.handle = None
            self._ws = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def haflo_keygen(n_bits, seed):
    p = (C.c_uint8 * (n_bits // 16))()
    q = (C.c_uint8 * (n_bits // 16))()
    _check(lib().haflo_keygen(n_bits, seed, p, q))
    return int.from_bytes(bytes(p), "little"), int.from_bytes(bytes(q), "little")


def haflo_ctx_create_private(p, q, n_bits):
    h = C.c_void_p()
    _check(lib().haflo_ctx_create_private(_le(p, n_bits // 16), _le(q, n_bits // 16), n_bits, C.byref(h)))
    return Context(h)


def haflo_ctx_create_public(n, n_bits):
    h = C.c_void_p()
    _check(lib().haflo_ctx_create_public(_le(n, n_bits // 8), n_bits, C.byref(h)))
    return Context(h)


def haflo_ctx_destroy(ctx):
    ctx.close()


def haflo_workspace_bytes(ctx, op, rows, cols=0):
    return lib().haflo_workspace_bytes(ctx.handle, op, rows, cols)


def haflo_op_cost(ctx, op):
    """(Montgomery products per element, 32-bit limbs of their modulus)."""
    mm, limbs = C.c_uint64(), C.c_uint32()
    _check(lib().haflo_op_cost(ctx.handle, op, C.byref(mm), C.byref(limbs)))
    return mm.value, limbs.value


def _new_cipher(ctx, count):
    return torch.empty((count, ctx.cipher_words), dtype=torch.int32, device="cuda")


def haflo_import_cipher(ctx, canon, status=None):
    count = canon.shape[0]
    out = _new_cipher(ctx, count)
    _check(lib().haflo_import_cipher(ctx.handle, _ptr(canon), _ptr(out), _ptr(status), count, _stream()))
    return out


def haflo_export_cipher(ctx, cipher):
    count = cipher.shape[0]
    out = torch.empty((count, ctx.cipher_limbs), dtype=torch.int32, device="cuda")
    _check(lib().haflo_export_cipher(ctx.handle, _ptr(cipher), _ptr(out), count, _stream()))
    return out


def haflo_encode_f32(ctx, v, scale_bits, status=None):
    count = v.numel()
    out = torch.empty((count, ctx.plain_limbs), dtype=torch.int32, device="cuda")
    _check(lib().haflo_encode_f32(ctx.handle, _ptr(v), scale_bits, _ptr(out), _ptr(status), count, _stream()))
    return out


def haflo_encode_exponents_f32(x, scale_bits, status=None):
    out = torch.empty(x.shape, dtype=torch.int32, device="cuda")
    _check(lib().haflo_encode_exponents_f32(_ptr(x), scale_bits, _ptr(out), _ptr(status), x.numel(), _stream()))
    return out


def haflo_decode(ctx, plain, scale_bits, status=None):
    count = plain.shape[0]
    q = torch.empty(count, dtype=torch.int64, device="cuda")
    v = torch.empty(count, dtype=torch.float64, device="cuda")
    _check(lib().haflo_decode(ctx.handle, _ptr(plain), scale_bits, _ptr(q), _ptr(v), _ptr(status), count, _stream()))
    return q, v


def haflo_encrypt(ctx, plain, r, out=None):
    count = plain.shape[0]
    if out is None:
        out = _new_cipher(ctx, count)
    nb = haflo_workspace_bytes(ctx, _cabi.OP_ENCRYPT, count)
    ws = ctx.workspace(nb)
    _check(lib().haflo_encrypt(ctx.handle, _ptr(plain), _ptr(r), _ptr(out), count, _ptr(ws), ws.numel(), _stream()))
    return out


def haflo_fore_gradient(ctx, c_host, logits_guest, label, r, scale_bits, out=None, status=None):
    count = c_host.shape[0]
    if out is None:
        out = _new_cipher(ctx, count)
    ws = ctx.workspace(haflo_workspace_bytes(ctx, _cabi.OP_FORE_GRADIENT, count))
    _check(lib().haflo_fore_gradient(ctx.handle, _ptr(c_host), _ptr(logits_guest), _ptr(label), _ptr(r), scale_bits,
                                     _ptr(out), _ptr(status) if status is not None else None, count, _ptr(ws),
                                     ws.numel(), _stream()))
    return out


def haflo_encrypt_with_obfuscator(ctx, plain, obfuscator, out=None):
    count = plain.shape[0]
    if out is None:
        out = _new_cipher(ctx, count)
    ws = ctx.workspace(haflo_workspace_bytes(ctx, _cabi.OP_ENCRYPT_OBFUSCATOR, count))
    _check(lib().haflo_encrypt_with_obfuscator(ctx.handle, _ptr(plain), _ptr(obfuscator), _ptr(out), count, _ptr(ws),
                                               ws.numel(), _stream()))
    return out


def haflo_taylor_loss(ctx, c_u, c_u2, u_guest, label, r, scale_bits, status=None):
    count = c_u.shape[0]
    out = _new_cipher(ctx, 1)
    ws = ctx.workspace(haflo_workspace_bytes(ctx, _cabi.OP_TAYLOR_LOSS, count))
    _check(lib().haflo_taylor_loss(ctx.handle, _ptr(c_u), _ptr(c_u2), _ptr(u_guest), _ptr(label),
                                   _ptr(r) if r is not None else None, scale_bits,
                                   _ptr(out), _ptr(status) if status is not None else None, count, _ptr(ws),
                                   ws.numel(), _stream()))
    return out


def haflo_decrypt(ctx, cipher, out=None):
    count = cipher.shape[0]
    if out is None:
        out = torch.empty((count, ctx.plain_limbs), dtype=torch.int32, device="cuda")
    nb = haflo_workspace_bytes(ctx, _cabi.OP_DECRYPT, count)
    ws = ctx.workspace(nb)
    _check(lib().haflo_decrypt(ctx.handle, _ptr(cipher), _ptr(out), count, _ptr(ws), ws.numel(), _stream()))
    return out


def haflo_add(ctx, c1, c2, out=None):
    count = c1.shape[0]
    if out is None:
        out = _new_cipher(ctx, count)
    _check(lib().haflo_add(ctx.handle, _ptr(c1), _ptr(c2), _ptr(out), count, _stream()))
    return out


def haflo_scalar_mul_u64(ctx, c, k, out=None):
    count = c.shape[0]
    if out is None:
        out = _new_cipher(ctx, count)
    ws = ctx.workspace(haflo_workspace_bytes(ctx, _cabi.OP_SCALAR_MUL, count))
    _check(lib().haflo_scalar_mul_u64(ctx.handle, _ptr(c), _ptr(k), _ptr(out), count, _ptr(ws), ws.numel(), _stream()))
    return out


def haflo_scalar_mul_i64_bcast(ctx, c, k, out=None):
    count = c.shape[0]
    if out is None:
        out = _new_cipher(ctx, count)
    ws = ctx.workspace(haflo_workspace_bytes(ctx, _cabi.OP_SCALAR_MUL, count))
    _check(lib().haflo_scalar_mul_i64_bcast(ctx.handle, _ptr(c), int(k), _ptr(out), count, _ptr(ws), ws.numel(),
                                            _stream()))
    return out


def haflo_cipher_matvec(ctx, orientation, c, X, out=None):
    rows, cols = X.shape
    nout = cols if orientation == 0 else rows
    if out is None:
        out = _new_cipher(ctx, nout)
    op = _cabi.OP_MATVEC_XT_D if orientation == 0 else _cabi.OP_MATVEC_X_W
    ws = ctx.workspace(haflo_workspace_bytes(ctx, op, rows, cols))
    _check(lib().haflo_cipher_matvec(ctx.handle, orientation, _ptr(c), _ptr(X), rows, cols, _ptr(out), _ptr(ws),
                                     ws.numel(), _stream()))
    return out


def haflo_cipher_sum(ctx, c):
    count = c.shape[0]
    out = _new_cipher(ctx, 1)
    ws = ctx.workspace(haflo_workspace_bytes(ctx, _cabi.OP_MATVEC_XT_D, count, 1))
    _check(lib().haflo_cipher_sum(ctx.handle, _ptr(c), count, _ptr(out), _ptr(ws), ws.numel(), _stream()))
    return out


class Stager:
    """Owner of a haflo_stager: host numpy arrays in the interchange format <-> device arrays."""

    def __init__(self, ctx, chunk_elems=8192, pool_cap_bytes=256 << 20):
        self.ctx = ctx
        h = C.c_void_p()
        _check(lib().haflo_stager_create(ctx.handle, chunk_elems, pool_cap_bytes, C.byref(h)))
        self.handle = h

    def stats(self):
        a, b, c = C.c_size_t(), C.c_size_t(), C.c_size_t()
        _check(lib().haflo_stager_stats(self.handle, C.byref(a), C.byref(b), C.byref(c)))
        return {"pinned_bytes": a.value, "pinned_allocs": b.value, "pinned_reuses": c.value}

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize()
            lib().haflo_stager_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def _host_words(arr, words):
    import numpy as np
    arr = np.ascontiguousarray(arr, dtype=np.uint32)
    if arr.ndim != 2 or arr.shape[1] != words:
        raise HafloError("expected a [count, %d] uint32 array" % words)
    return arr


def haflo_stage_in_cipher(stager, h_canon, status=None):
    h = _host_words(h_canon, stager.ctx.cipher_limbs)
    out = _new_cipher(stager.ctx, h.shape[0])
    _check(lib().haflo_stage_in_cipher(stager.handle, h.ctypes.data, _ptr(out),
                                       _ptr(status) if status is not None else None, h.shape[0], _stream()))
    return out


def haflo_stage_in_plain(stager, h_plain):
    h = _host_words(h_plain, stager.ctx.plain_limbs)
    out = torch.empty((h.shape[0], stager.ctx.plain_limbs), dtype=torch.int32, device="cuda")
    _check(lib().haflo_stage_in_plain(stager.handle, h.ctypes.data, _ptr(out), h.shape[0], _stream()))
    return out


def haflo_stage_out_cipher(stager, cipher):
    import numpy as np
    h = np.empty((cipher.shape[0], stager.ctx.cipher_limbs), dtype=np.uint32)
    _check(lib().haflo_stage_out_cipher(stager.handle, _ptr(cipher), h.ctypes.data, cipher.shape[0], _stream()))
    return h


def haflo_stage_out_plain(stager, plain):
    import numpy as np
    h = np.empty((plain.shape[0], stager.ctx.plain_limbs), dtype=np.uint32)
    _check(lib().haflo_stage_out_plain(stager.handle, _ptr(plain), h.ctypes.data, plain.shape[0], _stream()))
    return h
