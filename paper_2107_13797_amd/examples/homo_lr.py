"""One aggregation round of homogeneous federated logistic regression on synthetic data, built
from the library's operators over handles (paper section 2.1, the iteration workflow: local
computation, encrypted intermediates sent to a coordinator, aggregation on ciphertexts, decryption
by the parties).

Every party holds the key pair, its own instances and the common model; the coordinator sees
ciphertexts only and holds the public key.

    party k      w_k = w - lr * grad_k(w)      local step on its n_k instances (plain arithmetic)
    party k      [[w_k]]                       (encode, encrypt as the key owner)
    coordinator  [[S]] = sum_k n_k [[w_k]]     (scalar_mul by the instance count, add)
    party        w' = D([[S]]) / sum_k n_k     (decrypt, decode)

Operands and results live in a `Store` on each side; a ciphertext array crosses from a party to the
coordinator as a device copy. `run_round` returns the decoded sum together with the same sum in
exact integers on the quantised local models.

    python -m paper_2107_13797_amd.examples.homo_lr [--bits 2048] [--parties 8] [--weights 65536]
"""
import argparse
import time

import numpy as np
import torch

SCALE_W = 24


def _dev(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.uint32:
        a = a.view(np.int32)
    return torch.from_numpy(a).cuda()


def run_round(api, pub, own, parties, weights, seed=0, timings=None):
    """pub: public context (the coordinator), own: private context (the parties)."""
    from paper_2107_13797_amd import _cabi as K
    rng = np.random.default_rng(seed)
    lp = pub.plain_limbs
    w = rng.normal(0, 0.5, weights).astype(np.float32)
    counts = [int(c) for c in rng.integers(500, 5000, parties)]
    # the local step is plain arithmetic on each party's own data; here its result is synthetic:
    # the common model moved by a party-specific gradient
    local = [(w - 0.1 * rng.normal(0, 1, weights)).astype(np.float32) for _ in range(parties)]

    cipher_bytes = weights * pub.cipher_words * 4
    slack = 64 << 20
    party = api.Store(own, 3 * cipher_bytes + 4 * api.haflo_workspace_bytes(own, K.OP_ENCRYPT, weights) + slack)
    coord = api.Store(pub, 4 * cipher_bytes + 2 * api.haflo_workspace_bytes(pub, K.OP_SCALAR_MUL, weights) + slack)

    def timed(name, fn):
        if timings is None:
            return fn()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        out = fn()
        torch.cuda.synchronize()
        timings[name] = timings.get(name, 0.0) + (time.perf_counter() - t0) * 1e3
        return out

    total = None
    for k in range(parties):
        r = rng.integers(0, 2 ** 32, size=(weights, lp), dtype=np.uint32)
        r[:, -1] &= 0x7FFFFFFF
        hv, hr = party.upload(K.KIND_F32, _dev(local[k])), party.upload(K.KIND_PLAIN, _dev(r))
        hc = timed("parties: encode + encrypt", lambda: party.encrypt(party.encode(hv, SCALE_W), hr))
        sent = coord.upload(K.KIND_CIPHER, party.download(hc))
        scaled = timed("coordinator: scalar_mul by n_k", lambda: coord.scalar_mul(sent, counts[k]))
        total = scaled if total is None else timed("coordinator: add", lambda: coord.add(total, scaled))
    back = party.upload(K.KIND_CIPHER, coord.download(total))
    hq = timed("party: decrypt + decode", lambda: party.decode(party.decrypt(back), SCALE_W))
    summed = party.download(hq).cpu().numpy()
    assert party.stats()["live_objects"] == 0 and coord.stats()["live_objects"] == 0
    peak = {"party": party.stats()["peak_bytes"], "coordinator": coord.stats()["peak_bytes"]}
    party.close()
    coord.close()

    q = [np.rint(v.astype(np.float64) * 2.0 ** SCALE_W).astype(np.int64) for v in local]
    want_q = sum(n * qk for n, qk in zip(counts, q))
    return {
        "sum_q": (summed * 2.0 ** SCALE_W).tolist(),
        "want_sum_q": want_q.astype(np.float64).tolist(),
        "model": (summed / sum(counts)).tolist(),
        "float_model": (sum(n * v.astype(np.float64) for n, v in zip(counts, local)) / sum(counts)).tolist(),
        "peak_bytes": peak,
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--bits", type=int, default=2048)
    ap.add_argument("--parties", type=int, default=8)
    ap.add_argument("--weights", type=int, default=65536)
    args = ap.parse_args()
    from paper_2107_13797_amd import api
    p, q = api.haflo_keygen(args.bits, 7)
    own = api.haflo_ctx_create_private(p, q, args.bits)
    pub = api.haflo_ctx_create_public(p * q, args.bits)
    run_round(api, pub, own, 2, min(args.weights, 4096), seed=1)  # warm-up
    timings = {}
    res = run_round(api, pub, own, args.parties, args.weights, seed=2, timings=timings)
    assert res["sum_q"] == res["want_sum_q"]
    print("%d-bit key, %d parties, %d weights each: the decoded aggregate equals the exact fixed-point sum"
          % (args.bits, args.parties, args.weights))
    for name, ms in timings.items():
        print("  %-32s %9.2f ms" % (name, ms))
    print("  peak arena use: party %.1f MB, coordinator %.1f MB"
          % (res["peak_bytes"]["party"] / 1e6, res["peak_bytes"]["coordinator"] / 1e6))
    err = max(abs(a - b) for a, b in zip(res["model"], res["float_model"]))
    print("  largest deviation of the averaged model from the float64 average: %.3g" % err)


if __name__ == "__main__":
    main()
