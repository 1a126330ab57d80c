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
    """Owner of a haflo_ctx plus a growable workspace tensor.

    Every wrapper below that needs temporaries uses this one workspace, so calls through one
    Context must be ordered on one stream (torch's current stream); use a second Context, or the
    C entry points with workspaces of your own, to run operators concurrently.
    """

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


def haflo_ctx_set_xtd_bucket_min_rows(ctx, min_rows):
    _check(lib().haflo_ctx_set_xtd_bucket_min_rows(ctx.handle, min_rows))


def haflo_workspace_bytes(ctx, op, rows, cols=0):
    return lib().haflo_workspace_bytes(ctx.handle, op, rows, cols)


def haflo_op_work(ctx, op):
    """32x32+64-bit multiply-adds the kernels execute per element of the operator (chip-filling batches)."""
    w = C.c_uint64()
    _check(lib().haflo_op_work(ctx.handle, op, C.byref(w)))
    return w.value


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


def haflo_decrypt_static(ctx, cipher, out=None):
    """haflo_decrypt through the library's fixed scratch array: no workspace, nothing allocated by the call."""
    count = cipher.shape[0]
    if out is None:
        out = torch.empty((count, ctx.plain_limbs), dtype=torch.int32, device="cuda")
    _check(lib().haflo_decrypt_static(ctx.handle, _ptr(cipher), _ptr(out), count, _stream()))
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


def haflo_cipher_sum_segments(ctx, c, offsets, status=None):
    """offsets: int32 CUDA tensor of nseg + 1 non-decreasing element indices (read as uint32)."""
    count, nseg = c.shape[0], offsets.numel() - 1
    if offsets.dtype != torch.int32 or nseg < 0:
        raise HafloError("offsets: int32 tensor of nseg + 1 entries")
    out = _new_cipher(ctx, nseg)
    ws = ctx.workspace(haflo_workspace_bytes(ctx, _cabi.OP_SUM_SEGMENTS, count, nseg))
    _check(lib().haflo_cipher_sum_segments(ctx.handle, _ptr(c) if count else None, count, _ptr(offsets), nseg,
                                           _ptr(out) if nseg else None, _ptr(status), _ptr(ws), ws.numel(), _stream()))
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


class Store:
    """Owner of a haflo_store over an arena tensor: operands and results named by integer handles.

    Methods mirror the haflo_h_* entry points; `uses` is the number of operator calls that will
    consume the result (0 = until release()). The store enqueues everything on the torch stream
    that is current when it is created: call it with that stream current, so that tensors handed
    to upload() and returned by download() are ordered with its work.
    """

    def __init__(self, ctx, arena_bytes):
        self.ctx = ctx
        self.arena = torch.empty(arena_bytes, dtype=torch.uint8, device="cuda")
        h = C.c_void_p()
        _check(lib().haflo_store_create(ctx.handle, _ptr(self.arena), arena_bytes, _stream(), C.byref(h)))
        self.handle = h

    def stats(self):
        a, b, c, d = C.c_size_t(), C.c_size_t(), C.c_size_t(), C.c_size_t()
        _check(lib().haflo_store_stats(self.handle, C.byref(a), C.byref(b), C.byref(c), C.byref(d)))
        return {"live_bytes": a.value, "peak_bytes": b.value, "live_objects": c.value, "largest_free": d.value}

    def info(self, h):
        kind, count, ptr, uses = C.c_int(), C.c_size_t(), C.c_void_p(), C.c_uint32()
        _check(lib().haflo_store_info(self.handle, h, C.byref(kind), C.byref(count), C.byref(ptr), C.byref(uses)))
        return {"kind": kind.value, "count": count.value, "ptr": ptr.value, "uses": uses.value}

    def release(self, h):
        _check(lib().haflo_store_release(self.handle, h))

    def upload(self, kind, tensor, uses=1):
        """A device tensor's elements as a new object; `kind` says how its words are read."""
        t = tensor.contiguous()
        words = {_cabi.KIND_CIPHER: self.ctx.cipher_words, _cabi.KIND_PLAIN: self.ctx.plain_limbs}.get(kind)
        count = t.numel() // words if words else t.numel()
        h = C.c_uint64()
        _check(lib().haflo_h_upload(self.handle, kind, _ptr(t), 0, count, uses, C.byref(h)))
        return h.value

    def download(self, h):
        """The object's contents as a new device tensor (consumes one use)."""
        i = self.info(h)
        shapes = {_cabi.KIND_CIPHER: ((i["count"], self.ctx.cipher_words), torch.int32),
                  _cabi.KIND_PLAIN: ((i["count"], self.ctx.plain_limbs), torch.int32),
                  _cabi.KIND_F32: ((i["count"],), torch.float32), _cabi.KIND_F64: ((i["count"],), torch.float64),
                  _cabi.KIND_I32: ((i["count"],), torch.int32), _cabi.KIND_U32: ((i["count"],), torch.int32),
                  _cabi.KIND_I64: ((i["count"],), torch.int64), _cabi.KIND_U64: ((i["count"],), torch.int64)}
        shape, dtype = shapes[i["kind"]]
        out = torch.empty(shape, dtype=dtype, device="cuda")
        _check(lib().haflo_h_download(self.handle, h, _ptr(out), 0))
        return out

    def _call(self, fn, *args, status=False):
        out, st = C.c_uint64(), C.c_uint64()
        if status is None:
            _check(fn(self.handle, *args, C.byref(out)))
            return out.value
        _check(fn(self.handle, *args, C.byref(out), C.byref(st) if status else None))
        return (out.value, st.value) if status else out.value

    def encode(self, values, scale_bits, uses=1, status=False):
        return self._call(lib().haflo_h_encode, values, scale_bits, uses, status=status)

    def encode_exponents(self, values, scale_bits, uses=1, status=False):
        return self._call(lib().haflo_h_encode_exponents, values, scale_bits, uses, status=status)

    def decode(self, plain, scale_bits, uses=1, status=False):
        return self._call(lib().haflo_h_decode, plain, scale_bits, uses, status=status)

    def encrypt(self, plain, r, uses=1):
        return self._call(lib().haflo_h_encrypt, plain, r, uses, status=None)

    def decrypt(self, cipher, uses=1):
        return self._call(lib().haflo_h_decrypt, cipher, uses, status=None)

    def add(self, a, b, uses=1):
        return self._call(lib().haflo_h_add, a, b, uses, status=None)

    def scalar_mul(self, cipher, k, uses=1):
        return self._call(lib().haflo_h_scalar_mul, cipher, int(k), uses, status=None)

    def scalar_mul_each(self, cipher, scalars, uses=1):
        return self._call(lib().haflo_h_scalar_mul_each, cipher, scalars, uses, status=None)

    def matvec(self, orientation, cipher, exponents, rows, cols, uses=1):
        return self._call(lib().haflo_h_matvec, orientation, cipher, exponents, rows, cols, uses, status=None)

    def sum(self, cipher, uses=1):
        return self._call(lib().haflo_h_sum, cipher, uses, status=None)

    def close(self):
        if self.handle is not None:
            torch.cuda.synchronize()
            lib().haflo_store_destroy(self.handle)
            self.handle = None
            self.arena = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
