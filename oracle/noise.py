"""TEST INFRASTRUCTURE ONLY — counter-based Gaussian gradient noise, fp64.

The additive noise of the stochastic gradient oracle ("oracle class"
assumption: unbiased, variance bounded by sigma^2) is too large to pass in as
an array at the big sizes, so both sides regenerate it from a counter.  The
generator is Philox-4x32 with 10 rounds as published by Salmon, Moraes, Dror
and Shaw ("Parallel random numbers: as easy as 1, 2, 3", SC'11), followed by
the Box-Muller transform.  This file implements it from that definition with
numpy integers; it is pinned to the authors' known-answer vectors.

Counter layout for the noise of (step t, worker i, columns 4q..4q+3):
    counter = (q mod 2^32, q div 2^32, i, t),  key = (seed mod 2^32, seed div 2^32)
The four output words r0..r3 give four normals:
    u(r)  = ((r >> 9) + 1/2) * 2^-23           (23 bits + 1/2: exact in fp32, never 0 or 1)
    z0,z1 = sqrt(-2 ln u(r0)) * (cos, sin)(2 pi u(r1))
    z2,z3 = sqrt(-2 ln u(r2)) * (cos, sin)(2 pi u(r3))
"""
from __future__ import annotations

import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = np.uint64(0x9E3779B9)
_W1 = np.uint64(0xBB67AE85)
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(ctr, key):
    """ctr: four uint32 arrays (or scalars), key: two.  Returns four uint32
    arrays: ten rounds of the Philox S-P network, the key bumped by the Weyl
    constants between rounds."""
    c0, c1, c2, c3 = (np.asarray(c, dtype=np.uint64) & _MASK for c in ctr)
    k0, k1 = (np.asarray(k, dtype=np.uint64) & _MASK for k in key)
    for rnd in range(10):
        if rnd:
            k0 = (k0 + _W0) & _MASK
            k1 = (k1 + _W1) & _MASK
        p0 = _M0 * c0           # 32x32 -> 64 bit products, exact in uint64
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = hi1 ^ c1 ^ k0, lo1, hi0 ^ c3 ^ k1, lo0
    return tuple(np.asarray(c, dtype=np.uint64).astype(np.uint32) for c in (c0, c1, c2, c3))


def _unit(r: np.ndarray) -> np.ndarray:
    return ((r >> np.uint32(9)).astype(np.float64) + 0.5) * (2.0 ** -23)


def normal_noise(seed: int, step: int, n: int, cols) -> np.ndarray:
    """Standard-normal noise for workers 0..n-1 at the given column indices
    (any subset, any order), shape (n, len(cols)), fp64."""
    cols = np.asarray(cols, dtype=np.int64)
    q = (cols // 4).astype(np.uint64)
    lane = cols % 4
    out = np.empty((n, len(cols)), dtype=np.float64)
    key = (np.uint64(seed) & _MASK, (np.uint64(seed) >> _S32) & _MASK)
    for i in range(n):
        r = philox4x32_10((q & _MASK, q >> _S32, np.full_like(q, i), np.full_like(q, step)), key)
        rad_a = np.sqrt(-2.0 * np.log(_unit(r[0])))
        ang_a = 2.0 * np.pi * _unit(r[1])
        rad_b = np.sqrt(-2.0 * np.log(_unit(r[2])))
        ang_b = 2.0 * np.pi * _unit(r[3])
        z = np.stack([rad_a * np.cos(ang_a), rad_a * np.sin(ang_a),
                      rad_b * np.cos(ang_b), rad_b * np.sin(ang_b)])
        out[i] = z[lane, np.arange(len(cols))]
    return out
