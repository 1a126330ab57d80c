"""One training iteration of two-party heterogeneous logistic regression on synthetic data, built
from the library's operators (paper sections 2.1 and 3.4).

Parties: the host holds features X_h and weights w_h; the guest holds features X_g, weights w_g and
the labels y in {-1, +1}; an arbiter holds the private key. Every array stays on the device.

    host    u_h = X_h w_h                     -> [[u_h]], [[u_h^2]]          (encode, encrypt)
    guest   [[d]] = [[1/4 (u_h + u_g) - 1/2 y]]                              (fused fore gradient)
    guest   [[g_g]] = X_g^T [[d]],  host  [[g_h]] = X_h^T [[d]]              (gradient matvec)
    guest   [[loss]] = [[sum(-1/2 y u + 1/8 u^2)]]                           (Taylor loss)
    arbiter decrypts and decodes the gradients and the loss

`run_iteration` returns what the arbiter decodes together with the same quantities computed with
exact integers on the host from the quantised inputs, so that a caller can check them for equality.

    python -m paper_2107_13797_amd.examples.hetero_lr [--bits 2048] [--instances 65536] [--features 16]
"""
import argparse
import time

import numpy as np
import torch

SCALE_U = 20   # logits and labels
SCALE_X = 16   # feature matrices, as exponents


def _dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def _quant(v, s):
    return np.rint(np.asarray(v, dtype=np.float64) * 2.0 ** s).astype(np.int64)


def run_iteration(api, pub, own, instances, features, seed=0, timings=None):
    """pub: public context (both parties), own: private context (the arbiter)."""
    rng = np.random.default_rng(seed)
    lp = pub.plain_limbs
    X_h = rng.normal(0, 1, (instances, features)).astype(np.float32)
    X_g = rng.normal(0, 1, (instances, features)).astype(np.float32)
    w_h = rng.normal(0, 0.3, features).astype(np.float32)
    w_g = rng.normal(0, 0.3, features).astype(np.float32)
    y = np.where(rng.random(instances) < 0.5, -1.0, 1.0).astype(np.float32)
    u_h = (X_h @ w_h).astype(np.float32)
    u_g = (X_g @ w_g).astype(np.float32)

    def rand_r(count):
        r = rng.integers(0, 2 ** 32, size=(count, lp), dtype=np.uint32)
        r[:, -1] &= 0x7FFFFFFF
        return _dev(r)

    def timed(name, fn):
        if timings is None:
            return fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = fn()
        torch.cuda.synchronize()
        timings[name] = timings.get(name, 0.0) + (time.perf_counter() - t0) * 1e3
        return out

    # host: encrypted logits and their squares (the squares of the quantised logits, exactly)
    q_h = _quant(u_h, SCALE_U)
    sq_words = np.zeros((instances, lp), dtype=np.uint32)
    sq = q_h.astype(object) ** 2
    sq_words[:, 0] = np.array([int(v) & 0xFFFFFFFF for v in sq], dtype=np.uint32)
    sq_words[:, 1] = np.array([(int(v) >> 32) & 0xFFFFFFFF for v in sq], dtype=np.uint32)
    sq_words[:, 2] = np.array([(int(v) >> 64) & 0xFFFFFFFF for v in sq], dtype=np.uint32)
    c_u = timed("host: encrypt logits", lambda: api.haflo_encrypt(
        pub, api.haflo_encode_f32(pub, _dev(u_h), SCALE_U), rand_r(instances)))
    c_u2 = timed("host: encrypt squared logits", lambda: api.haflo_encrypt(pub, _dev(sq_words), rand_r(instances)))

    # guest: fore gradient, its gradient share and the loss; host: its gradient share
    d = timed("guest: fore gradient", lambda: api.haflo_fore_gradient(
        pub, c_u, _dev(u_g), _dev(y), rand_r(instances), SCALE_U))
    E_g = api.haflo_encode_exponents_f32(_dev(X_g), SCALE_X)
    E_h = api.haflo_encode_exponents_f32(_dev(X_h), SCALE_X)
    g_g = timed("guest: X_g^T [[d]]", lambda: api.haflo_cipher_matvec(pub, 0, d, E_g))
    g_h = timed("host: X_h^T [[d]]", lambda: api.haflo_cipher_matvec(pub, 0, d, E_h))
    loss = timed("guest: Taylor loss", lambda: api.haflo_taylor_loss(
        pub, c_u, c_u2, _dev(u_g), _dev(y), None, SCALE_U))  # goes to the arbiter only: no fresh r needed

    # arbiter
    both = torch.cat([g_g, g_h, loss], dim=0)
    plain = timed("arbiter: decrypt", lambda: api.haflo_decrypt(own, both))
    q_grad, v_grad = api.haflo_decode(own, plain[:2 * features], SCALE_U + 2 + SCALE_X)
    q_loss, v_loss = api.haflo_decode(own, plain[2 * features:], 2 * SCALE_U + 3)

    # the same from the quantised inputs with exact integers
    q_g, q_y = _quant(u_g, SCALE_U), _quant(y, SCALE_U)
    fore = (q_h + q_g - 2 * q_y).astype(object)
    want_grad = [int(np.dot(_quant(X, SCALE_X)[:, j].astype(object), fore)) for X in (X_g, X_h)
                 for j in range(features)]
    u = (q_h + q_g).astype(object)
    want_loss = int(np.sum(u * u - 4 * q_y.astype(object) * u))
    return {
        "gradient_q": q_grad.cpu().tolist(), "gradient": v_grad.cpu().tolist(), "want_gradient_q": want_grad,
        "loss_q": q_loss.cpu().tolist()[0], "loss_sum": v_loss.cpu().tolist()[0], "want_loss_q": want_loss,
        "float_gradient": [float(np.dot(X[:, j].astype(np.float64), 0.25 * (u_h + u_g).astype(np.float64) - 0.5 * y))
                           for X in (X_g, X_h) for j in range(features)],
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--bits", type=int, default=2048)
    ap.add_argument("--instances", type=int, default=65536)
    ap.add_argument("--features", type=int, default=16)
    args = ap.parse_args()
    from paper_2107_13797_amd import api
    p, q = api.haflo_keygen(args.bits, 7)
    own = api.haflo_ctx_create_private(p, q, args.bits)
    pub = api.haflo_ctx_create_public(p * q, args.bits)
    run_iteration(api, pub, own, min(args.instances, 4096), args.features, seed=1)  # warm-up
    timings = {}
    res = run_iteration(api, pub, own, args.instances, args.features, seed=2, timings=timings)
    assert res["gradient_q"] == res["want_gradient_q"] and res["loss_q"] == res["want_loss_q"]
    print("%d-bit key, %d instances, %d + %d features: decoded gradient and loss equal the exact fixed-point values"
          % (args.bits, args.instances, args.features, args.features))
    for name, ms in timings.items():
        print("  %-32s %9.2f ms" % (name, ms))
    err = max(abs(a - b) for a, b in zip(res["gradient"], res["float_gradient"]))
    print("  largest gradient deviation from the float64 formula: %.3g" % err)


if __name__ == "__main__":
    main()
