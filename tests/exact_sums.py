"""Exactly rounded row sums, independent of any order of addition (test infrastructure).

The coder's per-worker mean reference and its l2 scale are sums over a row.  The library and the
oracle add them in binary64 in one pinned order; these helpers give the value mathematics fixes
-- the binary32 number nearest to the exact real sum (ties to even) -- so that tests can hold the
pinned-order value against it.  Integer arithmetic only: every binary64 term is an integer mantissa
times a power of two; mantissas are added per exponent in 64-bit integers (two 27-bit halves, so
2^36 terms cannot overflow) and the per-exponent totals are combined as Python integers.
"""
from fractions import Fraction
from math import isqrt

import numpy as np


def exact_sum(x):
    """The exact sum of a float32 or float64 array as a Fraction."""
    x = np.asarray(x, dtype=np.float64).reshape(-1)
    if x.size == 0:
        return Fraction(0)
    assert np.isfinite(x).all()
    m, e = np.frexp(x)                                   # x = m 2^e, 0.5 <= |m| < 1 (m = 0 for x = 0)
    mi = np.ldexp(m, 53).astype(np.int64)                # exact: |m| 2^53 is an integer below 2^53
    hi, lo = mi >> 27, mi & ((1 << 27) - 1)              # mi = hi 2^27 + lo, 0 <= lo < 2^27
    e = e.astype(np.int16)
    order = np.argsort(e, kind="stable")                 # radix sort on 16-bit keys
    es = e[order]
    starts = np.flatnonzero(np.concatenate(([True], es[1:] != es[:-1])))
    exps = es[starts]
    acc_hi = np.add.reduceat(hi[order], starts)          # 64-bit integer sums: exact
    acc_lo = np.add.reduceat(lo[order], starts)
    emin = int(exps.min())
    total = 0
    for k in range(exps.size):
        total += ((int(acc_hi[k]) << 27) + int(acc_lo[k])) << (int(exps[k]) - emin)
    return Fraction(total) * Fraction(2) ** (emin - 53)


def round_to_f32(q):
    """The binary32 number nearest to the Fraction q (ties to even); q must round into the normal range."""
    q = Fraction(q)
    if q == 0:
        return np.float32(0.0)
    sign, a = (-1.0 if q < 0 else 1.0), abs(q)
    k = 23 - (a.numerator.bit_length() - a.denominator.bit_length())     # a 2^k is in (2^22, 2^24)
    while a * Fraction(2) ** k >= 1 << 24:
        k -= 1
    while a * Fraction(2) ** k < 1 << 23:
        k += 1
    scaled = a * Fraction(2) ** k                         # in [2^23, 2^24): 24 significant bits before the point
    n = scaled.numerator // scaled.denominator
    rem = scaled - n
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and (n & 1)):
        n += 1
    out = np.ldexp(np.float64(n), -k) * sign              # n <= 2^24: exact
    assert 2.0 ** -126 <= abs(out) < 2.0 ** 128
    return np.float32(out)


def sqrt_to_f32(q):
    """The binary32 number nearest to sqrt(q) for a Fraction q >= 0 (ties cannot occur for a square root
    of a number with a finite binary expansion unless it is exact)."""
    q = Fraction(q)
    assert q >= 0
    if q == 0:
        return np.float32(0.0)
    # scale by 4^k so that the integer square root carries at least 30 bits
    num, den = q.numerator, q.denominator
    k = max(0, 32 - (num.bit_length() - den.bit_length()) // 2)
    big = (num << (2 * k + 64)) // den                    # floor(q 4^(k+32)); the remainder only matters as "sticky"
    sticky = (num << (2 * k + 64)) % den != 0
    r = isqrt(big)
    sticky = sticky or r * r != big
    # sqrt(q) = (r + theta) 2^-(k+32), 0 <= theta < 1, theta > 0 iff sticky: add a half unit so that the
    # rounding below sees "just above r" and never an exact tie
    return round_to_f32((Fraction(2 * r + (1 if sticky else 0), 2)) * Fraction(2) ** (-(k + 32)))
