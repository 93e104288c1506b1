"""The arithmetic claim behind the quotient modes' fast path (Eq. 2 and the combined form).

The scale and quantise kernels divide every worker's element by the same clamped reference.  They take
the binary64 reciprocal of the reference once per coordinate and form float32(float64(g) * inv) per
worker; a result that is a subnormal binary32 number is redone with the division itself.  The claim is
that this equals the correctly rounded binary32 quotient g / b for every pair.  The argument (a quotient
that is not a binary32 number stays 2^-49 away, relatively, from every rounding midpoint of normal
size, the product errs by 2^-52) is held here against integer arithmetic and IEEE division, on random
pairs, on the pairs closest to a midpoint that exist, and on the subnormal ties that make the fallback
necessary.  Host arithmetic only: numpy's float32 division and float64 -> float32 conversion are the
processor's correctly rounded ones.
"""
import fractions

import numpy as np


def by_reciprocal(a, b):
    inv = 1.0 / b.astype(np.float64)
    with np.errstate(all="ignore"):
        return (a.astype(np.float64) * inv).astype(np.float32)


def with_fallback(a, b):
    f = by_reciprocal(a, b)
    tiny = (f != 0) & (np.abs(f) < np.float32(2.0 ** -126))
    with np.errstate(all="ignore"):
        f[tiny] = (a / b)[tiny]
    return f


def same_bits(x, y):
    x, y = np.asarray(x, np.float32), np.asarray(y, np.float32)
    both_nan = np.isnan(x) & np.isnan(y)
    return bool(np.all((x.view(np.uint32) == y.view(np.uint32)) | both_nan))


def exact_quotient_float32(a, b):
    """Correctly rounded binary32 a / b of two finite float32 scalars from rational arithmetic."""
    q = fractions.Fraction(float(a)) / fractions.Fraction(float(b))
    if q == 0:
        return np.float32(0.0) * np.float32(np.sign(a) * np.sign(b))
    s, q = (-1 if q < 0 else 1), abs(q)
    e = q.numerator.bit_length() - q.denominator.bit_length()
    if fractions.Fraction(2) ** e > q:
        e -= 1
    ulp = fractions.Fraction(2) ** (max(e, -126) - 23)
    n, r = divmod(q, ulp)
    n = int(n)
    if r * 2 > ulp or (r * 2 == ulp and n % 2 == 1):
        n += 1
    with np.errstate(over="ignore"):
        return np.float32(s * float(n * ulp))  # n * ulp is a binary32 number (or 2^128 -> inf)


def test_random_pairs_of_every_size():
    rng = np.random.default_rng(11)
    n = 4_000_000
    a = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32).view(np.float32)
    b = rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32).view(np.float32)
    keep = np.isfinite(a) & (np.abs(b) >= np.float32(1e-8)) & ~np.isnan(b)  # the reference is clamped
    a, b = a[keep], b[keep]
    with np.errstate(all="ignore"):
        want = a / b
    assert same_bits(with_fallback(a, b), want)
    # gradient-like magnitudes: every quotient is of normal size and no fallback is needed
    a = (rng.standard_normal(n) * 10.0 ** rng.uniform(-6, 2, n)).astype(np.float32)
    b = (rng.standard_normal(n)).astype(np.float32)
    b = np.where(np.abs(b) < 1e-8, np.copysign(np.float32(1e-8), b), b).astype(np.float32)
    assert same_bits(by_reciprocal(a, b), a / b)


def test_pairs_closest_to_a_midpoint():
    # For an odd 24-bit B and a small odd r, N = -r / B (mod 2^25) makes A = (B N + r) / 2^25 an integer:
    # A / B = (N + r / B) 2^-25 misses the midpoint N 2^-25 by r / (B N) relatively -- with r = +-1 the
    # closest a quotient of binary32 numbers can come.
    rng = np.random.default_rng(5)
    n = 400_000
    B = rng.integers(2 ** 22, 2 ** 23, n) * 2 + 1
    for r in (1, -1, 3, -3):
        inv = B.copy()
        for _ in range(5):  # Newton iteration for the inverse modulo 2^25
            inv = (inv * (2 - B * inv)) % (1 << 25)
        N = (-r * inv) % (1 << 25)
        A, rem = np.divmod(B * N + r, 1 << 25)
        assert not rem.any()
        ok = (N > 2 ** 24) & (A >= 2 ** 23) & (A < 2 ** 24)
        assert ok.sum() > n // 8
        a, b, Nk = A[ok].astype(np.float32), B[ok].astype(np.float32), N[ok]
        for scale_a, scale_b in ((1.0, 1.0), (2.0 ** -60, 2.0 ** 20), (2.0 ** 40, 2.0 ** -25)):
            aa, bb = a * np.float32(scale_a), b * np.float32(scale_b)
            got = by_reciprocal(aa, bb)
            assert same_bits(got, aa / bb)
            # and against the integers: the quotient lies just above (r > 0) or below the midpoint
            want = ((Nk + (1 if r > 0 else -1)) // 2).astype(np.float64) * 2.0 ** -24 * (scale_a / scale_b)
            assert same_bits(got, want.astype(np.float32))


def test_against_rational_arithmetic():
    rng = np.random.default_rng(3)
    a = rng.integers(0, 2 ** 32, 3000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    b = rng.integers(0, 2 ** 32, 3000, dtype=np.uint64).astype(np.uint32).view(np.float32)
    keep = np.isfinite(a) & np.isfinite(b) & (np.abs(b) >= np.float32(1e-8))
    a, b = a[keep], b[keep]
    got = with_fallback(a, b)
    want = np.array([exact_quotient_float32(x, y) for x, y in zip(a, b)], np.float32)
    assert same_bits(got, want)


def test_subnormal_ties_need_the_division():
    # b = 2k (k odd), g = k (2j+1) 2^-149: g / b = (2j+1) 2^-150 is exactly half way between two subnormal
    # numbers; the reciprocal route lands on either side, the fallback restores round-half-even.
    rng = np.random.default_rng(0)
    k = rng.integers(1, 2 ** 11, 500_000) * 2 + 1
    j = rng.integers(0, 2 ** 11, 500_000)
    A = k * (2 * j + 1)
    ok = A < 2 ** 23
    k, j, A = k[ok], j[ok], A[ok]
    a = (A.astype(np.float64) * 2.0 ** -149).astype(np.float32)
    b = (2.0 * k).astype(np.float32)
    want = ((j + (j & 1)).astype(np.float64) * 2.0 ** -149).astype(np.float32)  # the even neighbour
    assert same_bits(a / b, want)
    assert not same_bits(by_reciprocal(a, b), want)  # the reason for the test on the result's class
    assert same_bits(with_fallback(a, b), want)
    # the example of the kernel's comment
    a1, b1 = np.array([9 * 2.0 ** -149], np.float32), np.array([6.0], np.float32)
    assert same_bits(a1 / b1, np.array([2.0 ** -148], np.float32))


def test_special_operands():
    inf, nan = np.float32(np.inf), np.float32(np.nan)
    a = np.array([0.0, -0.0, 0.0, inf, -inf, inf, nan, 1.0, 3.0e38, -3.0e38, 1e-45, 1.0], np.float32)
    b = np.array([2.0, 2.0, -3.0, 5.0, 5.0, inf, 1.0, inf, 1e-8, 1e-8, 1e-8, nan], np.float32)
    with np.errstate(all="ignore"):
        assert same_bits(with_fallback(a, b), a / b)


def test_the_largest_quotient_survives_one_late_rounding():
    # the scale pass keeps max |g| * inv in binary64 and rounds once: rounding is monotone
    rng = np.random.default_rng(2)
    a = rng.standard_normal((200, 4096)).astype(np.float32)
    b = rng.standard_normal((200, 4096)).astype(np.float32)
    b = np.where(np.abs(b) < 1e-8, np.copysign(np.float32(1e-8), b), b).astype(np.float32)
    m64 = np.abs(a.astype(np.float64) * (1.0 / b.astype(np.float64))).max(axis=1)
    assert same_bits(m64.astype(np.float32), np.abs(a / b).max(axis=1))
