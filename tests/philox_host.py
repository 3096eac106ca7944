"""Philox4x32-10 (Salmon, Moraes, Dror and Shaw, "Parallel random numbers: as easy as 1, 2, 3", 2011) written out
on the host with numpy, from the published description: the reference the seeded sampling test regenerates the
library's uniforms with.  Pinned by the known-answer vectors published with the generator (test_abi_host.py)."""
import numpy as np

_M0, _M1 = np.uint64(0xD2511F53), np.uint64(0xCD9E8D57)
_W0, _W1 = np.uint64(0x9E3779B9), np.uint64(0xBB67AE85)
_MASK, _S32 = np.uint64(0xffffffff), np.uint64(32)


def philox4x32_10(counter, key):
    """counter: four uint64 arrays (values below 2^32), key: two; returns the four output words."""
    c = [np.asarray(x, dtype=np.uint64) for x in counter]
    k0, k1 = np.uint64(key[0]), np.uint64(key[1])
    for _ in range(10):
        p0, p1 = _M0 * c[0], _M1 * c[2]            # 32 x 32 -> 64 bit products
        c = [(p1 >> _S32) ^ c[1] ^ k0, p1 & _MASK, (p0 >> _S32) ^ c[3] ^ k1, p0 & _MASK]
        k0, k1 = (k0 + _W0) & _MASK, (k1 + _W1) & _MASK
    return c


def uniforms(seed, B, N):
    """float32 [B, N]: key = the two halves of the seed, counter = (k mod 2^32, k / 2^32, 0, 0) for k = b N + i,
    the upper 24 bits of the first output word times 2^-24."""
    k = np.arange(B * N, dtype=np.uint64)
    zero = np.zeros_like(k)
    out = philox4x32_10([k & _MASK, k >> _S32, zero, zero], [seed & 0xffffffff, (seed >> 32) & 0xffffffff])
    return ((out[0] >> np.uint64(8)).astype(np.float64) * 2.0 ** -24).astype(np.float32).reshape(B, N)
