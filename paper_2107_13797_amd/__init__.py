"""MI355X-native Paillier operator path for federated logistic regression.

The arithmetic lives in libhaflo.so (hand-written HIP for gfx950, see csrc/ and
include/haflo.h). `api` is the thin binding over its C boundary; PyTorch only
supplies device memory and streams. There is no CPU fallback: using `api`
without the built library raises.
"""
__all__ = ["api", "build"]
