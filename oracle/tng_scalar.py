"""Element-at-a-time oracle for the TNG coder, in pure Python loops.

TEST INFRASTRUCTURE ONLY.  A second, independently written statement of the quantiser of
section "Gradient Compression" and of Eqs. 1-2 (arXiv 1901.08227): Python integers for the
counter-based RNG and the bit packing, numpy.float32 scalars (one IEEE rounding per
operation) for the arithmetic.  Meant for tiny inputs (d <= a few dozen); the vectorised
oracle is checked against it bit for bit.
"""
from __future__ import annotations

import numpy as np

f32 = np.float32
_M32 = (1 << 32) - 1


def philox_block(counter, key):
    """Philox4x32-10 (Salmon et al., SC'11) on Python integers.  counter: 4 words, key: 2 words."""
    c = [int(x) & _M32 for x in counter]
    k = [int(x) & _M32 for x in key]
    for _ in range(10):
        prod_a = 0xD2511F53 * c[0]
        prod_b = 0xCD9E8D57 * c[2]
        c = [((prod_b >> 32) ^ c[1] ^ k[0]) & _M32, prod_b & _M32,
             ((prod_a >> 32) ^ c[3] ^ k[1]) & _M32, prod_a & _M32]
        k = [(k[0] + 0x9E3779B9) & _M32, (k[1] + 0xBB67AE85) & _M32]
    return c


def draw(seed, it, m, stream, j):
    """32-bit draw number j of the sequence (seed, it, m, stream)."""
    blk = philox_block((j >> 2, m, it, stream), (seed & _M32, (seed >> 32) & _M32))
    return blk[j & 3]


def uniform(word):
    return f32(word >> 8) * f32(2.0 ** -24)


def batch_index(seed, it, m, j, n_rows):
    return (draw(seed, it, m, 1, j) * n_rows) >> 32


def safe_reference(r, eps):
    r = f32(r)
    eps = f32(eps)
    if abs(r) < eps:
        return f32(np.copysign(eps, r))
    return r


def normalized(gd, rd, norm, eps, r2d=None):
    gd = f32(gd)
    if norm == 0:
        return gd
    if norm == 1:
        return f32(gd - f32(rd))
    if norm == 2:
        return f32(gd / safe_reference(rd, eps))
    if norm == 3:
        return f32(f32(gd - f32(rd)) / safe_reference(r2d, eps))
    raise ValueError(norm)


def ordered_sum(terms):
    """Sum of Python floats (binary64) in the fixed order: 4096-element chunks, inside a chunk 256
    strided lanes each added in order, the lanes added in order; chunks added in order inside groups
    of 256; groups added in order."""
    n = len(terms)
    chunk_sums = []
    for c0 in range(0, n, 4096):
        lanes = [0.0] * 256
        for k in range(16):
            for j in range(256):
                e = c0 + 256 * k + j
                if e < n:
                    lanes[j] = lanes[j] + float(terms[e])
        acc = 0.0
        for j in range(256):
            acc = acc + lanes[j]
        chunk_sums.append(acc)
    total = 0.0
    for g0 in range(0, len(chunk_sums), 256):
        acc = 0.0
        for c in chunk_sums[g0:g0 + 256]:
            acc = acc + c
        total = total + acc
    return total


def row_mean(g_row):
    return f32(ordered_sum([float(f32(x)) for x in g_row]) / float(len(g_row)))


def encode_row(g_row, gref, norm, eps, bits, seed, it, m, gref2=None, scale_kind=0):
    """One worker: returns (list of packed 32-bit words, R)."""
    d = len(g_row)
    s = (1 << (bits - 1)) - 1
    if norm == 4:
        mu = row_mean(g_row)
        v = [f32(f32(g_row[e]) - mu) for e in range(d)]
    else:
        v = [normalized(g_row[e], gref[e], norm, eps, None if gref2 is None else gref2[e])
             for e in range(d)]
    R = f32(0.0)
    if scale_kind == 1:
        R = f32(np.sqrt(ordered_sum([float(x) * float(x) for x in v])))
    else:
        for e in range(d):
            if abs(v[e]) > R:
                R = f32(abs(v[e]))
    if R < f32(1.17549435e-38):
        R = f32(0.0)
    per = 32 // bits
    words = [0] * ((d + per - 1) // per)
    if R != 0:
        inv = f32(f32(1.0) / R)
        for e in range(d):
            t = f32(abs(v[e]) * inv)
            if t > f32(1.0):
                t = f32(1.0)
            x = f32(t * f32(s))
            lo = int(x)
            frac = f32(x - f32(lo))
            lvl = lo + (1 if uniform(draw(seed, it, m, 0, e)) < frac else 0)
            sign = 1 if (v[e] < 0 and lvl > 0) else 0
            code = lvl | (sign << (bits - 1))
            words[e // per] |= code << ((e % per) * bits)
    return words, R


def decode_mean(words_rows, scales, gref, norm, eps, bits, d, gref2=None, means=None):
    """Server: decode all rows, add in worker order, scale by 1/M, undo the normalisation."""
    M = len(words_rows)
    s = (1 << (bits - 1)) - 1
    per = 32 // bits
    inv_m = f32(f32(1.0) / f32(M))
    out = []
    for e in range(d):
        acc = f32(0.0)
        for m in range(M):
            code = (words_rows[m][e // per] >> ((e % per) * bits)) & ((1 << bits) - 1)
            lvl = code & ((1 << (bits - 1)) - 1)
            sign = (code >> (bits - 1)) & 1
            R = f32(scales[m])
            if lvl == s:
                mag = R
            else:
                mag = f32(f32(R / f32(s)) * f32(lvl))
            if sign and lvl > 0:
                mag = f32(-mag)
            if norm == 4:
                mag = f32(f32(means[m]) + mag)
            acc = f32(acc + mag)
        mean = f32(acc * inv_m)
        if norm == 0 or norm == 4:
            vb = mean
        elif norm == 1:
            vb = f32(f32(gref[e]) + mean)
        elif norm == 2:
            vb = f32(safe_reference(gref[e], eps) * mean)
        else:
            vb = f32(f32(safe_reference(gref2[e], eps) * mean) + f32(gref[e]))
        out.append(vb)
    return out
