"""Slow reference arithmetic for the oracle's pins, written directly from the
definitions with Python big integers and exact rationals.  It is independent of
oracle/ (which it checks) and of the HIP library.
"""
import math
from fractions import Fraction

import numpy as np

MASK32 = 0xFFFFFFFF


def philox4x32_10(ctr, key):
    """Philox4x32, 10 rounds, on Python integers (Salmon et al., SC'11)."""
    c = [int(v) & MASK32 for v in ctr]
    k = [int(v) & MASK32 for v in key]
    for rnd in range(10):
        if rnd:
            k = [(k[0] + 0x9E3779B9) & MASK32, (k[1] + 0xBB67AE85) & MASK32]
        p0 = 0xD2511F53 * c[0]
        p1 = 0xCD9E8D57 * c[2]
        c = [(p1 >> 32) ^ c[1] ^ k[0], p1 & MASK32, (p0 >> 32) ^ c[3] ^ k[1], p0 & MASK32]
    return c


def random_word(seed, step, worker, j):
    quad = j >> 2
    out = philox4x32_10([quad & MASK32, quad >> 32, worker, step],
                        [seed & MASK32, (seed >> 32) & MASK32])
    return out[j & 3]


def scale(alpha, g):
    """alpha o g in fp32 (one IEEE multiply)."""
    with np.errstate(all="ignore"):
        return np.float32(alpha) * np.float32(g)


def int_random_exact(t, word):
    """Int(t) of Section 2 for a finite fp32 t: floor(t)+1 iff u < t-floor(t),
    u = (word >> 8) / 2^24, all in exact rational arithmetic except p, which is
    the fp32 difference t - floor(t) as the contract states."""
    tf = Fraction(float(t))
    fl = math.floor(tf)
    p = np.float32(t) - np.float32(fl)          # fp32 subtraction
    u = Fraction(word >> 8, 1 << 24)
    return fl + (1 if u < Fraction(float(p)) else 0)


def int_nearest_exact(t):
    """Nearest integer of a finite fp32 t, ties to even."""
    return round(Fraction(float(t)))            # Python rounds Fractions half-to-even


def clip(r, L):
    if r > L:
        return L, 1
    if r < -L:
        return -L, 1
    return r, 0


def ulp32(v):
    return float(np.spacing(np.float32(abs(float(v)))))
