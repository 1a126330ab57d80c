"""The allocation-free entry point (haflo_decrypt_static: temporaries in a fixed array inside the
library's device image) against haflo_decrypt, through the C boundary: two calls in a row, the
second with a smaller batch, plus the size limit. Collected last so that a failure here hides no
other test."""
import ctypes as C
import random

import pytest

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

from conftest import oracle_key  # noqa: E402
from oracle import paillier_oracle as O  # noqa: E402
from paper_2107_13797_amd import _cabi  # noqa: E402

from helpers import dev_to_ints, ints_to_dev  # noqa: E402


@pytest.mark.parametrize("bits,counts", [(1024, (700, 37)), (2048, (300, 300, 5)), (4096, (64, 1))])
def test_decrypt_static_matches_decrypt(bits, counts):
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2107_13797_amd import api
    lib = api.lib()
    p, q = oracle_key(bits)
    sk = O.PrivateKey(p, q)
    n = sk.public.n
    ctx = api.haflo_ctx_create_private(p, q, bits)
    stream = C.c_void_p(torch.cuda.current_stream().cuda_stream)
    rng = random.Random(bits)
    for call, count in enumerate(counts):
        print("decrypt_static", bits, "call", call, "count", count, flush=True)
        cs = [rng.randrange(1, n * n) for _ in range(count)]
        ms = [rng.randrange(n) for _ in range(min(count, 3))]
        cs[:len(ms)] = [O.encrypt(sk.public, m, rng.randrange(1, n)) for m in ms]
        cipher = api.haflo_import_cipher(ctx, ints_to_dev(cs, bits // 16))
        want = api.haflo_decrypt(ctx, cipher)
        got = torch.full((count, ctx.plain_limbs), -1, dtype=torch.int32, device="cuda")
        rc = lib.haflo_decrypt_static(ctx.handle, C.c_void_p(cipher.data_ptr()), C.c_void_p(got.data_ptr()), count, stream)
        assert rc == 0
        torch.cuda.synchronize()
        assert torch.equal(got, want)
        assert dev_to_ints(got)[:len(ms)] == ms
        assert dev_to_ints(got[-2:].contiguous()) == [O.decrypt_crt(sk, c) for c in cs[-2:]]
    # a batch whose temporaries do not fit the fixed array is refused, and nothing is written
    big = 200000
    assert lib.haflo_workspace_bytes(ctx.handle, _cabi.OP_DECRYPT, big, 0) > (16 << 20)
    dummy = torch.zeros(4, dtype=torch.int32, device="cuda")
    rc = lib.haflo_decrypt_static(ctx.handle, C.c_void_p(dummy.data_ptr()), C.c_void_p(dummy.data_ptr()), big, stream)
    assert rc == -6 and lib.haflo_strerror(rc)
    assert lib.haflo_decrypt_static(ctx.handle, None, None, 0, stream) == 0
    assert lib.haflo_decrypt_static(None, None, None, 1, stream) == -1
    pub = api.haflo_ctx_create_public(n, bits)
    assert lib.haflo_decrypt_static(pub.handle, C.c_void_p(cipher.data_ptr()), C.c_void_p(got.data_ptr()), 1, stream) == -3
    pub.close()
    ctx.close()
