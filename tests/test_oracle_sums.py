"""Pins for the order-pinned sums of the oracle and for what is built on them: the per-worker
mean reference (section "Reference Vectors": g~ = mean(g) ones(D), one extra scalar on the wire)
and the l2-norm scale of the cited multi-level quantiser (QSGD, Alistarh et al.)."""
import math

import numpy as np
import pytest

from oracle import tng_oracle as O
from oracle import tng_scalar as S

F32 = np.float32


def test_ordered_sum_is_a_sum_and_has_the_stated_order():
    rng = np.random.default_rng(0)
    for n in (0, 1, 255, 256, 257, 4095, 4096, 4097, 70000, (1 << 20) + 3):
        x = rng.standard_normal(n) * 10.0 ** rng.integers(-3, 3)
        got = float(O.tree_sum64(x))
        exact = math.fsum(x.tolist())
        assert abs(got - exact) <= 1e-12 * (np.abs(x).sum() + 1e-300)
        if n <= 70000:
            assert got == S.ordered_sum(x.tolist())                 # two implementations, same bits
    ints = rng.integers(-1000, 1000, 100000).astype(np.float64)     # exact whatever the order
    assert float(O.tree_sum64(ints)) == float(ints.sum()) == float(sum(ints.tolist()))
    # the order is the stated one: lane 0 of the first chunk meets 2^53 and -2^53 before any 1.0
    x = np.zeros(600)
    x[0], x[1], x[256] = 2.0 ** 53, 1.0, -(2.0 ** 53)
    assert float(O.tree_sum64(x)) == 1.0 and S.ordered_sum(x.tolist()) == 1.0
    assert float(np.cumsum(x)[-1]) == 0.0                           # plain left-to-right order loses the 1.0
    # chunks are added in order: a cancelling pair in chunks 0 and 1 is met before the 1.0 in chunk 2
    y = np.zeros(3 * 4096)
    y[0], y[4096], y[2 * 4096] = 2.0 ** 53, -(2.0 ** 53), 1.0
    assert float(O.tree_sum64(y)) == 1.0 and S.ordered_sum(y.tolist()) == 1.0


def test_worker_mean_is_the_mean():
    rng = np.random.default_rng(1)
    for d in (1, 7, 4096, 10001):
        g = (rng.standard_normal(d) * 3 + 5).astype(F32)
        mu = O.worker_mean(g)
        assert mu.dtype == F32
        exact = math.fsum(g.astype(np.float64).tolist()) / d
        assert abs(float(mu) - exact) <= abs(exact) * 2.0 ** -24 + 1e-30     # correctly rounded (up to the tie)
        assert mu == S.row_mean(list(g))
    assert O.worker_mean(np.full(1000, 0.1, dtype=F32)) == F32(0.1)


def test_mean_reference_shrinks_the_coded_vector():
    # the inequality the paper gives for this choice: ||a - mean(a)||^2 <= ||a||^2
    rng = np.random.default_rng(2)
    for _ in range(20):
        g = (rng.standard_normal(500) * rng.uniform(0.1, 2) + rng.uniform(-5, 5)).astype(F32)
        v = O.normalize(g, None, O.NORM_MEAN)
        assert float((v.astype(np.float64) ** 2).sum()) <= float((g.astype(np.float64) ** 2).sum()) * (1 + 1e-6)
        assert np.array_equal(v, g - O.worker_mean(g))
        assert abs(float(v.astype(np.float64).mean())) < 1e-5 * (1 + abs(float(g.mean())))


@pytest.mark.parametrize("bits", [2, 4])
def test_mean_reference_round_trip_is_unbiased_and_matches_elementwise_oracle(bits):
    rng = np.random.default_rng(3 + bits)
    d, M, T = 40, 3, 3000
    g = (rng.standard_normal((M, d)) + np.array([[4.0], [-2.0], [0.5]])).astype(F32)
    cfg = O.Config(d=d, M=M, bits=bits, norm=O.NORM_MEAN, seed=5)
    means = O.worker_means(g)
    acc = np.zeros(d)
    for it in range(T):
        codes, scales = O.normalize_encode(cfg, it, g, None)
        acc += O.decode_aggregate(cfg, codes, scales, None, d, means=means)
        if it < 20:
            rows = []
            for m in range(M):
                words, R = S.encode_row(list(g[m]), [0.0] * d, O.NORM_MEAN, cfg.quot_eps, bits, cfg.seed, it, m)
                assert [int(x) for x in codes[m]] == words and scales[m] == R
                rows.append(words)
            vs = S.decode_mean(rows, list(scales), [0.0] * d, O.NORM_MEAN, cfg.quot_eps, bits, d, means=list(means))
            assert all(a == b for a, b in zip(O.decode_aggregate(cfg, codes, scales, None, d, means=means), vs))
    target = g.astype(np.float64).mean(axis=0)
    v = np.stack([O.normalize(g[m], None, O.NORM_MEAN) for m in range(M)])
    R = np.abs(v).max(axis=1).astype(np.float64)
    se = math.sqrt((R ** 2).sum()) / (2 * O.levels_of(bits) * M) / math.sqrt(T)
    assert np.all(np.abs(acc / T - target) < 5 * se + 1e-6)
    # a worker whose gradient is constant sends nothing but its mean
    flat = np.full((1, d), 3.25, dtype=F32)
    one = O.Config(d=d, M=1, bits=bits, norm=O.NORM_MEAN, seed=5)
    codes, scales = O.normalize_encode(one, 0, flat, None)
    assert not codes.any() and scales[0] == 0
    assert np.array_equal(O.decode_aggregate(one, codes, scales, None, d, means=O.worker_means(flat)), flat[0])


@pytest.mark.parametrize("bits", [2, 4])
def test_l2_scale(bits):
    rng = np.random.default_rng(6 + bits)
    d, T = 64, 4000
    v = rng.standard_normal(d).astype(F32)
    R = O.scale_of(v, O.SCALE_L2)
    exact = math.sqrt(math.fsum((v.astype(np.float64) ** 2).tolist()))
    assert R.dtype == F32 and abs(float(R) - exact) <= exact * 2.0 ** -23
    assert R >= np.abs(v).max()                                      # so |v|/R <= 1 still holds
    assert O.scale_of(np.zeros(5, dtype=F32), O.SCALE_L2) == 0
    words, Rs = S.encode_row(list(v), [0.0] * d, 0, 1e-8, bits, 9, 0, 0, scale_kind=O.SCALE_L2)
    cfg = O.Config(d=d, M=1, bits=bits, norm=O.NORM_NONE, seed=9, scale_kind=O.SCALE_L2)
    codes, scales = O.normalize_encode(cfg, 0, v[None, :], None)
    assert scales[0] == R == Rs and [int(x) for x in codes[0]] == words
    # unbiased, and the coding error obeys the bound of the cited quantiser:
    # E||Q_s(v) - v||^2 <= min(d / s^2, sqrt(d) / s) ||v||^2
    s = O.levels_of(bits)
    acc = np.zeros(d)
    err = 0.0
    for it in range(T):
        codes, scales = O.normalize_encode(cfg, it, v[None, :], None)
        q = O.decode_aggregate(cfg, codes, scales, None, d).astype(np.float64)
        acc += q
        err += ((q - v) ** 2).sum()
    assert np.all(np.abs(acc / T - v) < 5 * float(R) / (2 * s) / math.sqrt(T) + 1e-6)
    assert err / T <= min(d / s ** 2, math.sqrt(d) / s) * exact ** 2 * 1.05


def test_exact_sum_helpers_against_the_exactly_rounded_library_sum():
    # tests/exact_sums.py is what the pinned-order sums are held against; pin it first: exact_sum equals
    # math.fsum (exactly rounded to binary64) wherever binary64 can show it, round_to_f32 agrees with the
    # IEEE conversion on binary64 inputs and resolves ties to even, sqrt_to_f32 on exact squares and on 2
    from fractions import Fraction

    from exact_sums import exact_sum, round_to_f32, sqrt_to_f32

    rng = np.random.default_rng(11)
    for n in (1, 2, 17, 1000, 50000):
        x = (rng.standard_normal(n) * 10.0 ** rng.integers(-12, 12, n)).astype(F32)
        assert float(exact_sum(x)) == math.fsum(x.astype(np.float64).tolist())
        sq = x.astype(np.float64) ** 2
        assert float(exact_sum(sq)) == math.fsum(sq.tolist())
    assert exact_sum(np.array([2.0 ** 60, 1.0, -(2.0 ** 60)])) == 1                 # no order, no loss
    assert exact_sum(np.array([0.1, 0.2], dtype=F32)) == Fraction(float(F32(0.1))) + Fraction(float(F32(0.2)))
    for v in rng.standard_normal(300) * 10.0 ** rng.integers(-20, 20, 300):
        assert round_to_f32(Fraction(float(v))) == F32(v)
    assert round_to_f32(Fraction(2 ** 24 + 1)) == F32(2 ** 24) and round_to_f32(Fraction(2 ** 24 + 3)) == F32(2 ** 24 + 4)
    assert round_to_f32(Fraction(1, 3)) == F32(1.0 / 3.0) and round_to_f32(Fraction(-7, 5)) == F32(-1.4)
    assert sqrt_to_f32(Fraction(9, 4)) == F32(1.5) and sqrt_to_f32(Fraction(2)) == F32(math.sqrt(2.0))
    for v in rng.uniform(1e-6, 1e6, 200):
        assert sqrt_to_f32(Fraction(float(v))) == F32(math.sqrt(float(v)))            # 53 >= 2*24+2: no double rounding


def test_pinned_order_sums_round_to_what_the_exact_sums_round_to():
    # The mean reference and the l2 scale are DEFINED as float32(exact sum / D) and float32(sqrt(exact sum of
    # squares)); the oracle (and the library) add in binary64 in one pinned order, which could differ from that
    # only if the exact value sat within ~1e-13 relative of a binary32 rounding boundary.  Held against the
    # exact values on the inputs the parity tests use (the generator of the encode/decode benchmark, and
    # shifted / scaled rows), sizes up to 2^22.
    import torch

    from exact_sums import exact_sum, round_to_f32, sqrt_to_f32
    from paper_1901_08227_amd import synth

    checked = 0
    for d, M, seed in [(1, 2, 2), (5, 2, 7), (257, 3, 260), (4096, 2, 4098), (4099, 3, 1), (65536, 4, 3),
                       (4096 * 20 + 148, 3, 231), ((1 << 20) + 8200, 2, 5), (1 << 22, 2, 1)]:
        g, gref = (t.numpy() for t in synth.codec_inputs(M, d, seed))
        for m in range(M):
            for row in (g[m], g[m] * F32(1e-3) + F32(7.0)):
                assert O.worker_mean(row) == round_to_f32(exact_sum(row) / d), (d, m)
                for v in (row, row - gref, row - O.worker_mean(row)):
                    v = v.astype(F32)
                    want = sqrt_to_f32(exact_sum(v.astype(np.float64) ** 2))
                    assert O.scale_of(v, O.SCALE_L2) == (want if want >= O.FLT_MIN else 0), (d, m)
                    checked += 1
    assert checked > 100


def test_reciprocal_multiply_stays_within_two_roundings_of_the_quotient():
    # "Gradient Compression": P(z = 1) = |v_d| / R.  The coder evaluates |v| * fl(1/R), one reciprocal per
    # worker, instead of a division per element: two roundings instead of one.  The probability it realises
    # then differs from |v|/R by at most 2^-23 |v|/R (below two steps of the 24-bit uniform grid), it never
    # exceeds 1 after the clamp, and the arg-max element itself maps to 1 - 2^-24 or 1, i.e. is coded at
    # the top level with probability >= 1 - 2^-24.
    rng = np.random.default_rng(12)
    worst = 0.0
    for _ in range(200):
        R = F32(abs(rng.standard_normal()) * 10.0 ** rng.integers(-20, 20) + 1e-30)
        a = (rng.random(2000).astype(F32) * R).astype(F32)
        a[0] = R
        t = np.minimum(a * (F32(1.0) / R), F32(1.0))
        exact = a.astype(np.float64) / np.float64(R)
        worst = max(worst, float(np.max(np.abs(t.astype(np.float64) - exact) / np.maximum(exact, 1e-300))))
        assert t.max() <= 1.0 and t[0] >= F32(1.0) - F32(2.0 ** -24)
        one_ulp = np.abs(t - (a / R).astype(F32)) <= np.spacing(np.maximum(t, F32(2.0 ** -126)))
        assert one_ulp.all()                                   # at most one unit in the last place from fl(|v|/R)
    assert worst <= 2.0 ** -23
