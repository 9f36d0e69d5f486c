"""TEST INFRASTRUCTURE ONLY: CPU oracle, never imported by the product path.

Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, "Parallel
random numbers: as easy as 1, 2, 3", SC'11, Sec. 3.2: the Philox S-box built
from a 32x32->64 multiply, the Feistel-like word permutation, and the Weyl key
schedule).  The paper only says that clients and the edge server draw the
local perturbation from a shared random seed (Sec. 3.1 workflow step 5,
Algorithm 1 "shared random seed s" and the edge server's "regenerate identical
z_h via seed s"); a counter-based generator is what makes that regeneration
a pure function of (seed, step, tensor, element).

Plain numpy, vectorised over the leading axes, one round at a time in the
order the definition states.  Pinned by the published known-answer vectors in
tests/golden/philox_kat.txt.
"""
import numpy as np

PHILOX_M0 = np.uint64(0xD2511F53)
PHILOX_M1 = np.uint64(0xCD9E8D57)
PHILOX_W0 = np.uint64(0x9E3779B9)   # golden ratio
PHILOX_W1 = np.uint64(0xBB67AE85)   # sqrt(3) - 1
_MASK32 = np.uint64(0xFFFFFFFF)
_SH32 = np.uint64(32)


def philox4x32(ctr, key, rounds: int = 10):
    """ctr: uint array [..., 4]; key: uint array [..., 2] (broadcastable).
    Returns uint32 array [..., 4]."""
    ctr = np.asarray(ctr, dtype=np.uint64)
    key = np.asarray(key, dtype=np.uint64)
    c0, c1, c2, c3 = (ctr[..., i] & _MASK32 for i in range(4))
    k0 = key[..., 0] & _MASK32
    k1 = key[..., 1] & _MASK32
    for r in range(rounds):
        if r > 0:                         # Weyl sequence: bump the key between rounds
            k0 = (k0 + PHILOX_W0) & _MASK32
            k1 = (k1 + PHILOX_W1) & _MASK32
        p0 = PHILOX_M0 * c0               # 64-bit products of 32-bit words
        p1 = PHILOX_M1 * c2
        hi0, lo0 = p0 >> _SH32, p0 & _MASK32
        hi1, lo1 = p1 >> _SH32, p1 & _MASK32
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    out = np.stack(np.broadcast_arrays(c0, c1, c2, c3), axis=-1)
    return out.astype(np.uint32)
