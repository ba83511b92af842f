"""Philox4x32-10 counter-based generator (Salmon, Moraes, Dror, Shaw, SC'11), in numpy.

Oracle-side implementation used for stochastic rounding: the random number of an
element is a pure function of (seed, layer, element index), so the CPU oracle and the
GPU draw identical bits without sharing any state.

Mapping used by the quantizer:
    key     = (seed & 0xffffffff, seed >> 32)
    counter = ((i >> 2) & 0xffffffff, (i >> 2) >> 32, layer, 0)
    word    = output[i & 3]
    u       = float32(word >> 8) * 2**-24           in [0, 1)
"""
import numpy as np

_M0 = np.uint64(0xD2511F53)
_M1 = np.uint64(0xCD9E8D57)
_W0 = 0x9E3779B9
_W1 = 0xBB67AE85
_MASK = np.uint64(0xFFFFFFFF)
_S32 = np.uint64(32)


def philox4x32_10(c0, c1, c2, c3, k0: int, k1: int):
    """Ten rounds on arrays of 32-bit counter words (held in uint64). Returns 4 uint32 arrays."""
    c0 = np.asarray(c0, np.uint64) & _MASK
    c1 = np.asarray(c1, np.uint64) & _MASK
    c2 = np.asarray(c2, np.uint64) & _MASK
    c3 = np.asarray(c3, np.uint64) & _MASK
    k0 &= 0xFFFFFFFF
    k1 &= 0xFFFFFFFF
    for rnd in range(10):
        p0 = _M0 * c0                      # 32x32 -> 64 bit products, no overflow in uint64
        p1 = _M1 * c2
        hi0, lo0 = p0 >> _S32, p0 & _MASK
        hi1, lo1 = p1 >> _S32, p1 & _MASK
        c0, c1, c2, c3 = (hi1 ^ c1 ^ np.uint64(k0), lo1, hi0 ^ c3 ^ np.uint64(k1), lo0)
        k0 = (k0 + _W0) & 0xFFFFFFFF       # Weyl key schedule, bumped after each round
        k1 = (k1 + _W1) & 0xFFFFFFFF
    return (c0.astype(np.uint32), c1.astype(np.uint32), c2.astype(np.uint32), c3.astype(np.uint32))


def element_words(seed: int, layer: int, n: int) -> np.ndarray:
    """uint32[n]: the Philox word of elements 0..n-1 of one layer."""
    nblk = (n + 3) // 4
    blk = np.arange(nblk, dtype=np.uint64)
    out = philox4x32_10(blk & _MASK, blk >> _S32, np.full(nblk, layer, np.uint64),
                        np.zeros(nblk, np.uint64), seed & 0xFFFFFFFF, (seed >> 32) & 0xFFFFFFFF)
    return np.stack(out, axis=1).reshape(-1)[:n]


def element_uniform(seed: int, layer: int, n: int) -> np.ndarray:
    """float32[n] in [0,1): 24 high bits of each element's word, scaled by 2^-24 (exact)."""
    w = element_words(seed, layer, n)
    return (w >> np.uint32(8)).astype(np.float32) * np.float32(2.0 ** -24)
