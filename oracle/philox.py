"""Oracle Philox4x32-10 (test infrastructure).

Philox4x32-10 is the public counter-based generator of Salmon et al. (SC'11): ten rounds, each of
which multiplies two of the four 32-bit counter words by fixed odd constants, keeps both halves
of the 64-bit products, and mixes them with the other words and a 2x32-bit key that is bumped by
Weyl constants between rounds.  Written here with 64-bit integer arithmetic on NumPy arrays.

The CD-1 sampler (see rbm.py) draws the uniform of flat element index e as
    block = philox(counter = (e >> 2, step, layer, phase), key = (seed_lo, seed_hi))
    u     = (block[e & 3] >> 8) * 2^-24          in [0, 1)
which is exactly representable in float32 and float64 alike.
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint64(0x9E3779B9)
_W1 = np.uint64(0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0, k1):
    """Vectorised over the counter words (array-likes of equal shape or scalars).

    Returns four uint32 arrays (the output block)."""
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & _MASK for c in np.broadcast_arrays(c0, c1, c2, c3))
    k0 = np.uint64(int(k0) & 0xFFFFFFFF)
    k1 = np.uint64(int(k1) & 0xFFFFFFFF)
    for r in range(10):
        if r > 0:
            k0 = (k0 + _W0) & _MASK
            k1 = (k1 + _W1) & _MASK
        p0 = _M0 * c0          # < 2^64: both factors < 2^32
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return tuple(c.astype(np.uint32) for c in (c0, c1, c2, c3))


def uniforms(count: int, seed: int, step: int, layer: int, phase: int) -> np.ndarray:
    """float64 array u[e], e = 0..count-1, of the sampler's uniforms (24-bit, in [0,1))."""
    e = np.arange(count, dtype=np.uint64)
    blk = philox4x32_10(e >> np.uint64(2), step, layer, phase, seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    words = np.stack(blk, axis=1)                       # count x 4
    w = words[np.arange(count), (e & np.uint64(3)).astype(np.int64)]
    return (w >> np.uint32(8)).astype(np.float64) * (1.0 / 16777216.0)
