"""Philox4x32-10 counter-based generator (Salmon et al., "Parallel random numbers:
as easy as 1, 2, 3", SC'11) and the uniform map used by the round.

Test infrastructure only (see oracle/__init__.py).

Algorithm 2 only says r_i ~ Unif[0,1]; the reading taken here makes every
uniform a pure function of (seed, slot i, round index, sequence id, stream):

    key     = (seed & 0xffffffff, seed >> 32)
    counter = (slot, round, seq, stream)
    u       = (first output word >> 8) * 2**-24          in [0, 1)

stream 0 = draft sample y_i, stream 1 = accept test r_i, stream 2 = the
residual / bonus sample y'.  u has 24 significant bits, so fp32 and fp64 hold
the same real number.

Pins: the generator's published known-answer vectors (tests/golden/philox_kat.txt)
and a uniformity chi-square.
"""
from __future__ import annotations

import numpy as np

_M0 = 0xD2511F53
_M1 = 0xCD9E8D57
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = 0xFFFFFFFF

STREAM_DRAFT = 0
STREAM_ACCEPT = 1
STREAM_RESAMPLE = 2


def philox4x32_10(counter, key):
    """One Philox4x32 block with 10 rounds on python ints.

    counter: 4 words, key: 2 words (each 0..2**32-1).  Returns 4 output words.
    """
    c0, c1, c2, c3 = (int(c) & _MASK for c in counter)
    k0, k1 = (int(k) & _MASK for k in key)
    for rnd in range(10):
        if rnd > 0:                      # key schedule: bump before rounds 2..10
            k0 = (k0 + _W0) & _MASK
            k1 = (k1 + _W1) & _MASK
        p0 = _M0 * c0                    # 64-bit products
        p1 = _M1 * c2
        hi0, lo0 = p0 >> 32, p0 & _MASK
        hi1, lo1 = p1 >> 32, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ k0) & _MASK, lo1, (hi0 ^ c3 ^ k1) & _MASK, lo0
    return c0, c1, c2, c3


def philox4x32_10_np(c0, c1, c2, c3, k0, k1):
    """Vectorised Philox4x32-10: every argument broadcasts; returns word 0..3 arrays
    (uint64 holding 32-bit values)."""
    c0, c1, c2, c3, k0, k1 = np.broadcast_arrays(
        *(np.asarray(a, dtype=np.uint64) & np.uint64(_MASK) for a in (c0, c1, c2, c3, k0, k1)))
    m0, m1 = np.uint64(_M0), np.uint64(_M1)
    mask, s32 = np.uint64(_MASK), np.uint64(32)
    for rnd in range(10):
        if rnd > 0:
            k0 = (k0 + np.uint64(_W0)) & mask
            k1 = (k1 + np.uint64(_W1)) & mask
        p0 = m0 * c0
        p1 = m1 * c2
        hi0, lo0 = p0 >> s32, p0 & mask
        hi1, lo1 = p1 >> s32, p1 & mask
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return c0, c1, c2, c3


def uniform(seed: int, slot: int, rnd: int, seq: int, stream: int) -> float:
    """The uniform for (seed, slot, round, sequence, stream); a float64 in [0,1)
    that is exactly representable in float32."""
    w0 = philox4x32_10((slot, rnd, seq, stream), (seed & _MASK, (seed >> 32) & _MASK))[0]
    return (w0 >> 8) * 2.0 ** -24


def uniform_np(seed, slot, rnd, seq, stream):
    """Vectorised `uniform` (arguments broadcast)."""
    seed = np.asarray(seed, dtype=np.uint64)
    w0 = philox4x32_10_np(slot, rnd, seq, stream, seed & np.uint64(_MASK), seed >> np.uint64(32))[0]
    return (w0 >> np.uint64(8)).astype(np.float64) * 2.0 ** -24
