"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11).

TEST INFRASTRUCTURE ONLY (see oracle/__init__.py).

The paper's Alg. 2 draws r ~ U(0,1) per drafted token and samples one token
from a final distribution; it does not say where the random numbers come from.
Reading taken: every draw is one Philox4x32-10 block addressed by
    key     = (seed low 32 bits, seed high 32 bits)
    counter = (slot, call, level, 0)
where `level` is the hierarchy level doing the draw, `call` counts that
level's Verify calls (or draft steps for the lowest level) and `slot` is
i-1 for the accept test of draft token i and t for the final sample.
Word 0 of the block feeds accept tests, word 1 feeds sampling.

Pinned by the published known-answer vectors of the Random123 distribution
(tests/golden/philox_kat.txt).
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_SH = np.uint64(32)


def philox4x32_10(counter, key):
    """Ten Philox rounds.  counter: (..., 4) uint32-valued, key: (2,) ints.
    Returns an array of the same leading shape with 4 uint32 words."""
    c = np.asarray(counter, dtype=np.uint64)
    c0, c1, c2, c3 = (c[..., 0].copy(), c[..., 1].copy(), c[..., 2].copy(), c[..., 3].copy())
    k0 = int(key[0]) & 0xFFFFFFFF
    k1 = int(key[1]) & 0xFFFFFFFF
    for _ in range(10):
        p0 = _M0 * c0            # 64-bit products of 32-bit values
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _SH, p0 & _MASK
        hi1, lo1 = p1 >> _SH, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + _W0) & 0xFFFFFFFF
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return np.stack([c0, c1, c2, c3], axis=-1).astype(np.uint32)


def draw(seed, level, call, slot):
    """The 4 words of the block addressed by (seed, level, call, slot)."""
    key = (seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    ctr = np.array([slot & 0xFFFFFFFF, call & 0xFFFFFFFF, level & 0xFFFFFFFF, 0], dtype=np.uint64)
    return philox4x32_10(ctr, key)


def uniform24(word):
    """u in [0,1) on a 2^-24 grid from the top 24 bits of a 32-bit word (exact in fp32)."""
    return np.float32(int(word) >> 8) * np.float32(2.0 ** -24)
