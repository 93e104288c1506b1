"""The arithmetic claims behind the ternary coder that reads the gradients once (section "Gradient
Compression": P(z = 1) = |v| / R, coded as [u < fl(|v| fl(1 / R))] with u on the 24-bit grid).

The scale pass decides, before R is known, which elements can still code non-zero, against a lower bound
R^ <= R, with the three-operation test  float(word) < fma(|v|, c1, 258),
c1 = fl(fl(1 / R^) (2^32 + 2^12)); everything that fails it is coded 0 without being looked at again.  The
quantise pass sees a kept element only as a bracket [lo, hi] around tau = |v| / u, the scale up to which the
element codes non-zero (13 bits of the value's significand, a reciprocal good to one unit in the last place,
13 bits of the quotient's significand), and decides from the row's scale alone: level 1 for
R <= lo (1 - 2^-19), level 0 for R >= hi (1 + 2^-12), the value itself in between.  Both steps are only right if

  (1) an element that fails the test has level 0 for every R >= R^, and
  (2) the level is 1 at every scale below the bracket's lower threshold and 0 at every scale above the upper one.

Held here on the host in binary32 arithmetic (numpy's correctly rounded operations; the fused multiply-add
through exact rational arithmetic), on random operands and on draws placed right at the thresholds.
"""
import fractions

import numpy as np

F32 = np.float32
TWO32P = F32(2.0 ** 32 + 2.0 ** 12)  # 2^32 (1 + 2^-20), a binary32 number


def c1_of(r_hat):
    with np.errstate(over="ignore", divide="ignore"):
        c1 = (F32(1.0) / r_hat) * TWO32P
    return np.where(r_hat >= F32(2.0 ** -90), c1, F32(np.inf)).astype(F32)


def fma32(a, b, c):
    """Correctly rounded binary32 a * b + c: the product of two binary32 numbers is exact in binary64; where
    adding c could round twice, the sum is redone in rational arithmetic."""
    p = a.astype(np.float64) * b.astype(np.float64)
    with np.errstate(invalid="ignore", over="ignore"):
        s = p + np.float64(c)
        out = s.astype(F32)
    finite = np.isfinite(p)
    # binary64 was exact when the sum needed no rounding; otherwise (few) go through fractions
    inexact = finite & ((s - p != np.float64(c)) | (s - np.float64(c) != p))
    for i in np.flatnonzero(inexact):
        exact = fractions.Fraction(float(a[i])) * fractions.Fraction(float(b[i])) + fractions.Fraction(float(c))
        out[i] = round_to_f32(exact)
    return out


def round_to_f32(q):
    if q == 0:
        return F32(0.0)
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
        return F32(s * float(n * ulp))


def kept(word, absv, r_hat):
    """The scale pass's test, as the kernel makes it."""
    with np.errstate(invalid="ignore"):
        return word.astype(F32) < fma32(absv, c1_of(r_hat), F32(258.0))  # NaN (0 * inf) compares false


def level(word, absv, R):
    """The coder's level: [u < fl(|v| fl(1 / R))], u = (word >> 8) 2^-24."""
    u = (word >> np.uint32(8)).astype(F32) * F32(2.0 ** -24)
    inv_r = np.where(R == 0, F32(0.0), F32(1.0) / np.where(R == 0, F32(1.0), R)).astype(F32)
    return u < absv * inv_r


def operands(rng, n, spread):
    absv = np.abs(rng.standard_normal(n) * 10.0 ** rng.uniform(-spread, 1, n)).astype(F32)
    R = (absv * F32(1.0) + np.abs(rng.standard_normal(n)).astype(F32) * absv * F32(8.0) + F32(1e-30)).astype(F32)  # R >= |v|
    r_hat = (R * rng.uniform(0.05, 1.0, n).astype(F32)).astype(F32)
    r_hat = np.minimum(r_hat, R)
    return absv, R, r_hat


def words_at_threshold(rng, absv, r_hat):
    """Draws placed within a few hundred units of 2^32 fl(|v| / R^), where the two tests could part."""
    with np.errstate(over="ignore", invalid="ignore"):
        t = (absv * (F32(1.0) / r_hat)).astype(np.float64) * 2.0 ** 32
    t = np.clip(np.nan_to_num(t, nan=0.0, posinf=2.0 ** 32), 0, 2.0 ** 32 - 1)
    w = t + rng.integers(-600, 601, absv.shape[0])
    return np.clip(w, 0, 2.0 ** 32 - 1).astype(np.uint64).astype(np.uint32)


def test_what_the_scale_pass_drops_codes_to_zero():
    rng = np.random.default_rng(17)
    n = 1_000_000
    for spread, words in ((1, "uniform"), (6, "uniform"), (1, "threshold"), (6, "threshold")):
        absv, R, r_hat = operands(rng, n, spread)
        word = (rng.integers(0, 2 ** 32, n, dtype=np.uint64).astype(np.uint32) if words == "uniform"
                else words_at_threshold(rng, absv, r_hat))
        keep = kept(word, absv, r_hat)
        for scale in (R, r_hat):  # the real scale, and the case where the bound is the scale itself
            lv = level(word, absv, scale)
            assert not np.any(lv & ~keep), "an element that codes non-zero was dropped"
        # and it is a test worth making: at the scale R^ it keeps next to nothing that codes to 0
        if words == "uniform":
            extra = np.count_nonzero(keep & ~level(word, absv, r_hat))
            assert extra <= 1e-4 * n


def test_zeros_tiny_bounds_and_the_ends_of_the_draw():
    absv = np.array([0.0, 0.0, 1e-40, 3.0, 3.0, 1e-20, 2.5, 2.5], F32)
    r_hat = np.array([1.0, 1e-35, 1e-35, 3.0, 3.0, 1e-30, 2.5, 2.5], F32)  # below 2^-90: no bound is claimed
    word = np.array([0, 0, 2 ** 32 - 1, 2 ** 32 - 1, 0, 12345, 2 ** 32 - 256, 2 ** 32 - 257], np.uint64).astype(np.uint32)
    keep = kept(word, absv, r_hat)
    assert keep[0]                                       # a zero with a draw below the slack is kept (and then coded 0)
    assert not keep[1]                                   # a zero under "no bound": 0 * inf is no number, compares false
    assert keep[2] and keep[5]                           # with no bound every non-zero element is kept
    for R in (r_hat, (r_hat * F32(4.0)).astype(F32)):
        assert not np.any(level(word, absv, R) & ~keep)
    assert keep[3] and keep[4] and keep[6] and keep[7]   # |v| = R^: level 1 for every draw (u < 1)


def tau_entry(absv, word, rcp_ulps):
    """The slot entry's bracket as the scale pass forms it; rcp_ulps moves the reciprocal by that many units in
    the last place (the hardware's is good to one)."""
    v13 = (absv.view(np.uint32) & np.uint32(0x7FFFFC00)).view(F32)
    k = (word >> np.uint32(8)).astype(F32)
    with np.errstate(divide="ignore", over="ignore", invalid="ignore"):
        rc = (F32(1.0) / k).astype(F32)
        for _ in range(abs(rcp_ulps)):
            rc = np.nextafter(rc, F32(np.inf) if rcp_ulps > 0 else F32(0.0)).astype(F32)
        tau = (v13 * (rc * F32(2.0 ** 24)).astype(F32)).astype(F32)
    lo_bits = tau.view(np.uint32) & np.uint32(0x7FFFFC00)
    return lo_bits.view(F32), (lo_bits | np.uint32(0x3FF)).view(F32), (lo_bits & np.uint32(0x7F800000)) != np.uint32(0x7F800000)


def test_the_bracket_of_a_kept_element_decides_from_the_safe_side():
    rng = np.random.default_rng(23)
    n = 1_000_000
    c_lo, c_hi = F32(1.0 - 2.0 ** -19), F32(1.0 + 2.0 ** -12)
    for spread in (1, 5):
        absv, _, _ = operands(rng, n, spread)
        for draws in ("any", "small"):
            word = rng.integers(0, 2 ** 32, n, dtype=np.uint64)
            if draws == "small":
                word >>= rng.integers(8, 31, n).astype(np.uint64)  # small u: large tau, down to u = 0
            word = word.astype(np.uint32)
            for ulps in (-1, 0, 1):
                lo, hi, bounded = tau_entry(absv, word, ulps)
                with np.errstate(over="ignore", invalid="ignore"):
                    r_one = (lo * c_lo).astype(F32)    # the largest scale decided as level 1
                    r_zero = (hi * c_hi).astype(F32)   # the smallest scale decided as level 0
                # scales below the smallest normal number never reach the coder (they are taken as 0)
                ok1 = bounded & np.isfinite(r_one) & (r_one >= F32(2.0 ** -126))
                assert np.all(level(word[ok1], absv[ok1], r_one[ok1])), "decided 1 where the level is 0"
                ok0 = np.isfinite(r_zero) & (r_zero >= F32(2.0 ** -126))   # (an unbounded tau never compares >=)
                assert not np.any(level(word[ok0], absv[ok0], r_zero[ok0])), "decided 0 where the level is 1"
                # and between the thresholds lies only a sliver of the scales: what goes back to the value
                both = ok1 & ok0 & (lo > 0)
                assert np.all(r_zero[both] <= lo[both] * F32(1.0 + 2.0 ** -11))
