"""Pins for the oracle's coder Q and the normalisation around it.

What fixes the expected values here is the paper (arXiv 1901.08227) and arithmetic, not the
oracle: unbiasedness E Q[v] = v (Background), P(z_d = 1) = |v_d| / R with R = max|v_d|
(section "Gradient Compression"), v = g~ + r and v = g~ (.) r (Eqs. 1, 2), the zero
reference degenerating to plain compressed SGD (remark after Proposition 2), the 2 bits per
ternary element of the bit accounting in "Nonconvex Problems", exact enumeration over the
2^24 possible uniforms, and brute force against a second, element-at-a-time implementation.
"""
import math
from fractions import Fraction

import numpy as np
import pytest

from oracle import tng_oracle as O
from oracle import tng_scalar as S

F32 = np.float32


def _decode_rows(cfg, codes, scales, d):
    return np.stack([O.dequantize(*O.unpack(codes[m], d, cfg.bits), scales[m], cfg.bits)
                     for m in range(codes.shape[0])])


# ------------------------------------------------------------------ unbiasedness (I1)
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("norm", [O.NORM_NONE, O.NORM_SUB, O.NORM_QUOT, O.NORM_COMB])
def test_decoded_mean_over_many_draws_converges_to_the_input(bits, norm):
    rng = np.random.default_rng(10 * bits + norm)
    d, M, T = 48, 2, 3000
    gref = rng.standard_normal(d).astype(F32)
    gref2 = (rng.standard_normal(d) + 3.0).astype(F32)
    g = (gref + 0.3 * rng.standard_normal((M, d))).astype(F32)
    cfg = O.Config(d=d, M=M, bits=bits, norm=norm, seed=77)
    s = O.levels_of(bits)
    acc = np.zeros(d)
    for it in range(T):
        codes, scales = O.normalize_encode(cfg, it, g, gref, gref2)
        acc += O.decode_aggregate(cfg, codes, scales, gref, d, gref2).astype(np.float64)
    est = acc / T
    target = g.astype(np.float64).mean(axis=0)
    # per-element standard error from the coder's variance (R/s)^2 f (1-f) <= (R/s)^2 / 4,
    # mapped back through the normalisation and the mean over M workers
    v = np.stack([O.normalize(g[m], gref, norm, cfg.quot_eps, gref2) for m in range(M)])
    R = np.abs(v).max(axis=1).astype(np.float64)
    gain = {O.NORM_NONE: 1.0, O.NORM_SUB: 1.0,
            O.NORM_QUOT: np.abs(gref.astype(np.float64)),
            O.NORM_COMB: np.abs(gref2.astype(np.float64))}[norm]
    se = gain * math.sqrt((R ** 2).sum()) / (2 * s * M) / math.sqrt(T)
    assert np.all(np.abs(est - target) < 5 * se + 1e-6 * np.abs(target) + 1e-7)
    # and the estimate is not trivially equal to the input (there is noise to average)
    assert np.abs(est - target).max() > 0


@pytest.mark.parametrize("bits", [2, 4])
def test_rounding_probability_is_exact_on_the_24_bit_grid(bits):
    """Enumerate every possible uniform: #{u < f} = ceil(f 2^24), so E[level] is known exactly."""
    s = O.levels_of(bits)
    all_u = O.uniform_from_word(np.arange(1 << 24, dtype=np.uint32) << np.uint32(8))
    R = F32(3.0)
    for a in [0.0, 1e-9, 0.1, 0.7499999, 1.5, 2.0, 2.9999998, 3.0, 1.0 / 3.0, 2.5]:
        v = np.full(1 << 24, a, dtype=F32)
        level, neg = O.quantize(v, R, bits, all_u)
        assert not neg.any()
        exact_x = Fraction(float(F32(a) * (F32(1.0) / R))) * s          # t as the oracle rounds it, times s
        exact_x = min(exact_x, Fraction(s))
        x32 = Fraction(float(F32(float(exact_x))))                      # one more rounding for t*s
        lo = math.floor(x32)
        frac = x32 - lo
        ups = int(np.count_nonzero(level == lo + 1))
        assert ups == math.ceil(frac * (1 << 24))
        assert ups + int(np.count_nonzero(level == lo)) == 1 << 24
        mean_val = (lo + ups / 2 ** 24) * float(R) / s
        # unbiased up to the 2^-24 grid and the two roundings of t and t*s
        assert abs(mean_val - float(F32(a))) <= float(R) / s * 2.0 ** -24 + 2 * float(R) * 2.0 ** -24


def test_ternary_probabilities_are_magnitude_over_R():
    rng = np.random.default_rng(3)
    d, T = 32, 20000
    v = rng.standard_normal(d).astype(F32)
    R = O.scale_of(v)
    assert float(R) == float(np.abs(v).max())
    ones = np.zeros(d)
    signs_ok = True
    for it in range(T):
        u = O.uniform_from_word(O.quant_draw_words(5, it, 0, d))
        level, neg = O.quantize(v, R, 2, u)
        assert level.max() <= 1
        ones += level
        signs_ok &= bool(np.all(neg == ((v < 0) & (level == 1))))
    assert signs_ok
    p = np.abs(v.astype(np.float64)) / float(R)
    assert np.all(np.abs(ones / T - p) < 5 * np.sqrt(p * (1 - p) / T) + 1e-6)
    assert ones[np.argmax(np.abs(v))] == T          # the largest element is always sent as +-1


@pytest.mark.parametrize("bits", [2, 4])
def test_second_moment_matches_closed_form(bits):
    """Ternary: E Q_d^2 = R |v_d|.  s levels: Var Q_d = (R/s)^2 f (1 - f), f = frac(s |v_d| / R)."""
    rng = np.random.default_rng(4)
    d, T = 24, 20000
    v = rng.standard_normal(d).astype(F32)
    R = O.scale_of(v)
    s = O.levels_of(bits)
    sq = np.zeros(d)
    sm = np.zeros(d)
    for it in range(T):
        u = O.uniform_from_word(O.quant_draw_words(6, it, 1, d))
        q = O.dequantize(*O.quantize(v, R, bits, u), R, bits).astype(np.float64)
        sq += q * q
        sm += q
    x = s * np.abs(v.astype(np.float64)) / float(R)
    f = x - np.floor(x)
    var = (float(R) / s) ** 2 * f * (1 - f)
    emp_var = sq / T - (sm / T) ** 2
    assert np.all(np.abs(emp_var - var) < 0.08 * (float(R) / s) ** 2)
    if bits == 2:
        assert np.all(np.abs(sq / T - float(R) * np.abs(v)) < 0.05 * float(R) ** 2)
        # summed over elements: E ||Q[v]||^2 = R ||v||_1
        assert abs(sq.sum() / T - float(R) * np.abs(v).sum()) < 0.02 * float(R) * np.abs(v).sum()


# ------------------------------------------------------------------ deterministic properties
@pytest.mark.parametrize("bits", [2, 4])
def test_decoded_value_is_one_of_the_two_grid_points_around_v(bits):
    rng = np.random.default_rng(5)
    s = O.levels_of(bits)
    for it in range(50):
        v = (rng.standard_normal(257) * 10.0 ** rng.integers(-20, 20)).astype(F32)
        R = O.scale_of(v)
        u = O.uniform_from_word(O.quant_draw_words(8, it, 0, v.size))
        level, neg = O.quantize(v, R, bits, u)
        q = O.dequantize(level, neg, R, bits).astype(np.float64)
        x = s * np.abs(v.astype(np.float64)) / float(R)
        assert level.min() >= 0 and level.max() <= s
        assert np.all(level >= np.floor(x * (1 - 2e-7)))
        assert np.all(level <= np.ceil(x * (1 + 2e-7)))
        assert np.all(np.abs(q - v) <= float(R) / s * (1 + 1e-6))
        assert np.all(np.sign(q) * np.sign(v) >= 0)
        assert not np.any(neg & (level == 0))                       # canonical zero


@pytest.mark.parametrize("bits", [2, 4])
def test_largest_element_keeps_its_full_magnitude(bits):
    """|v| = R must give t in {1 - 2^-24, 1}: level s (or s-1 with f ~ 1), never above s."""
    rng = np.random.default_rng(6)
    s = O.levels_of(bits)
    Rs = np.concatenate([rng.uniform(0.5, 2.0, 2000), 10.0 ** rng.uniform(-30, 30, 2000)]).astype(F32)
    for R in Rs[:400]:
        v = np.array([R, -R, F32(0.0)], dtype=F32)
        t = np.minimum(np.abs(v) * (F32(1.0) / R), F32(1.0))
        assert t[0] in (F32(1.0), F32(1.0 - 2.0 ** -24)) and t[0] <= 1
        level, neg = O.quantize(v, R, bits, np.zeros(3, dtype=F32))        # u = 0: rounds up whenever f > 0
        assert level[0] == s and level[1] == s and level[2] == 0
        assert list(neg) == [False, True, False]
        level, _ = O.quantize(v, R, bits, np.full(3, 1 - 2.0 ** -24, dtype=F32))   # largest u
        assert level[0] >= s - 1 and level[2] == 0
        assert np.array_equal(O.dequantize(np.array([s, s]), np.array([False, True]), R, bits),
                              np.array([R, -R], dtype=F32))               # level s decodes to R itself


def test_zero_and_tiny_scales():
    cfg = O.Config(d=9, M=2, bits=4, norm=O.NORM_NONE, seed=1)
    g = np.zeros((2, 9), dtype=F32)
    g[1, 3] = F32(1e-39)                                    # subnormal maximum -> scale taken as 0
    codes, scales = O.normalize_encode(cfg, 0, g, np.zeros(9, dtype=F32))
    assert not codes.any() and not scales.any()
    assert not O.decode_aggregate(cfg, codes, scales, np.zeros(9, dtype=F32), 9).any()
    g[1, 3] = F32(1.2e-38)                                  # just normal: coded
    codes, scales = O.normalize_encode(cfg, 0, g, np.zeros(9, dtype=F32))
    assert scales[1] == F32(1.2e-38) and codes[1].any() and not codes[0].any()
    assert O.scale_of(np.zeros(0, dtype=F32)) == 0


@pytest.mark.parametrize("bits", [2, 4])
def test_gradient_equal_to_reference_is_reconstructed_exactly(bits):
    rng = np.random.default_rng(7)
    d, M = 100, 3
    gref = rng.standard_normal(d).astype(F32)
    gref[5] = 0.0
    gref[6] = F32(1e-12)
    g = np.tile(gref, (M, 1))
    # Eq. 1: nothing to send, decoder returns the reference bit for bit
    cfg = O.Config(d=d, M=M, bits=bits, norm=O.NORM_SUB, seed=3)
    codes, scales = O.normalize_encode(cfg, 0, g, gref)
    assert not codes.any() and not scales.any()
    assert np.array_equal(O.decode_aggregate(cfg, codes, scales, gref, d), gref)
    # Eq. 2: quotient is 1 everywhere the reference is not clamped; R = 1; top level; product = reference
    cfg = O.Config(d=d, M=M, bits=bits, norm=O.NORM_QUOT, seed=3)
    keep = np.abs(gref) >= F32(1e-8)
    codes, scales = O.normalize_encode(cfg, 0, g[:, keep], gref[keep])
    assert np.all(scales == 1)
    level, neg = O.unpack(codes[0], int(keep.sum()), bits)
    assert np.all(level == O.levels_of(bits)) and not neg.any()
    assert np.array_equal(O.decode_aggregate(cfg, codes, scales, gref[keep], int(keep.sum())), gref[keep])


@pytest.mark.parametrize("bits", [2, 4])
def test_zero_reference_degenerates_to_plain_compressed_sgd(bits):
    rng = np.random.default_rng(8)
    d, M = 77, 4
    g = rng.standard_normal((M, d)).astype(F32)
    zero = np.zeros(d, dtype=F32)
    a = O.Config(d=d, M=M, bits=bits, norm=O.NORM_SUB, seed=9)
    b = O.Config(d=d, M=M, bits=bits, norm=O.NORM_NONE, seed=9)
    ca, sa = O.normalize_encode(a, 2, g, zero)
    cb, sb = O.normalize_encode(b, 2, g, zero)
    assert np.array_equal(ca, cb) and np.array_equal(sa, sb)
    assert np.array_equal(O.decode_aggregate(a, ca, sa, zero, d), O.decode_aggregate(b, cb, sb, zero, d))
    # and for ternary it is the randomised sign coder of the text: R * sign(v) * z
    if bits == 2:
        q = _decode_rows(b, cb, sb, d)
        for m in range(M):
            assert set(np.unique(q[m])) <= {-sb[m], F32(0.0), sb[m]}
            nz = q[m] != 0
            assert np.array_equal(np.sign(q[m][nz]), np.sign(g[m][nz]))


def test_codes_depend_only_on_the_normalised_vector():
    # Eq. 1: shifting g and g~ together changes nothing (integers keep the subtraction exact)
    rng = np.random.default_rng(9)
    d, M = 64, 2
    g = rng.integers(-50, 50, (M, d)).astype(F32)
    gref = rng.integers(-50, 50, d).astype(F32)
    shift = rng.integers(-1000, 1000, d).astype(F32)
    cfg = O.Config(d=d, M=M, bits=4, norm=O.NORM_SUB, seed=2)
    c1, s1 = O.normalize_encode(cfg, 1, g, gref)
    c2, s2 = O.normalize_encode(cfg, 1, g + shift, gref + shift)
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2)
    # scaling v by a power of two scales R and leaves every code alone
    v = rng.standard_normal((M, d)).astype(F32)
    cfg = O.Config(d=d, M=M, bits=4, norm=O.NORM_NONE, seed=2)
    c1, s1 = O.normalize_encode(cfg, 1, v, np.zeros(d, dtype=F32))
    c2, s2 = O.normalize_encode(cfg, 1, v * F32(1024.0), np.zeros(d, dtype=F32))
    assert np.array_equal(c1, c2) and np.array_equal(s1 * F32(1024.0), s2)
    # Eq. 2: scaling g and g~ by the same power of two leaves the quotient, hence the codes, alone
    cfg = O.Config(d=d, M=M, bits=2, norm=O.NORM_QUOT, seed=2)
    gr = (rng.standard_normal(d) + 2).astype(F32)
    c1, s1 = O.normalize_encode(cfg, 1, v, gr)
    c2, s2 = O.normalize_encode(cfg, 1, v * F32(8.0), gr * F32(8.0))
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2)


def test_reference_clamp_for_the_quotient():
    eps = 1e-8
    r = np.array([0.0, -0.0, 5e-9, -5e-9, 1e-8, -1e-8, 2.0, -3.0], dtype=F32)
    c = O.clamp_reference(r, eps)
    e = F32(eps)
    assert np.array_equal(c, np.array([e, -e, e, -e, F32(1e-8), F32(-1e-8), 2.0, -3.0], dtype=F32))
    assert np.signbit(c[1]) and not np.signbit(c[0])
    for x in r:
        assert S.safe_reference(x, eps) == O.clamp_reference(np.array([x]), eps)[0]
    # quotient normalisation and its inverse use the same clamped reference
    g = np.array([1.0, -2.0, 3.0, 4.0, 5.0, 6.0, 7.0, 8.0], dtype=F32)
    v = O.normalize(g, r, O.NORM_QUOT, eps)
    assert np.array_equal(v, g / c)
    assert np.array_equal(O.denormalize(v, r, O.NORM_QUOT, eps), c * v)


def test_combined_two_reference_form():
    rng = np.random.default_rng(11)
    d = 33
    g = rng.standard_normal(d).astype(F32)
    r1 = rng.standard_normal(d).astype(F32)
    r2 = (rng.standard_normal(d) + 4).astype(F32)
    v = O.normalize(g, r1, O.NORM_COMB, 1e-8, r2)
    assert np.array_equal(v, (g - r1) / r2)
    back = O.denormalize(v, r1, O.NORM_COMB, 1e-8, r2)
    assert np.array_equal(back, r2 * v + r1)
    assert np.allclose(back, g, rtol=0, atol=1e-5)
    # with g~' = ones it is Eq. 1; with g~ = zeros it is Eq. 2
    ones, zeros = np.ones(d, dtype=F32), np.zeros(d, dtype=F32)
    assert np.array_equal(O.normalize(g, r1, O.NORM_COMB, 1e-8, ones), O.normalize(g, r1, O.NORM_SUB))
    assert np.array_equal(O.normalize(g, zeros, O.NORM_COMB, 1e-8, r2), O.normalize(g, r2, O.NORM_QUOT, 1e-8))


# ------------------------------------------------------------------ packing (I8)
@pytest.mark.parametrize("bits", [2, 4])
def test_pack_layout_every_position_and_code_value(bits):
    per = 32 // bits
    s = O.levels_of(bits)
    for d in list(range(1, 2 * per + 2)) + [63, 64, 65, 1000]:
        assert O.words_per_row(d, bits) == -(-d * bits // 32)
        for pos in {0, d // 2, d - 1}:
            for lvl in range(0, s + 1):
                for sign in ((0,) if lvl == 0 else (0, 1)):
                    level = np.zeros(d, dtype=np.int32)
                    neg = np.zeros(d, dtype=bool)
                    level[pos], neg[pos] = lvl, bool(sign)
                    words = O.pack(level, neg, bits)
                    expect = [0] * O.words_per_row(d, bits)
                    expect[pos // per] = (lvl | (sign << (bits - 1))) << ((pos % per) * bits)
                    assert [int(w) for w in words] == expect
                    l2, n2 = O.unpack(words, d, bits)
                    assert np.array_equal(l2, level) and np.array_equal(n2, neg)
    rng = np.random.default_rng(12)
    for d in (1, 15, 16, 17, 31, 33, 255):
        level = rng.integers(0, s + 1, d).astype(np.int32)
        neg = rng.integers(0, 2, d).astype(bool) & (level > 0)
        words = O.pack(level, neg, bits)
        used = d * bits - 32 * (len(words) - 1)
        assert int(words[-1]) >> used == 0                       # padding bits are zero
        l2, n2 = O.unpack(words, d, bits)
        assert np.array_equal(l2, level) and np.array_equal(n2, neg)


def test_ternary_costs_two_bits_per_element():
    # bit accounting of "Nonconvex Problems": one 16-bit vector = 8 ternary transmissions
    with open(__import__("os").path.join(__import__("os").path.dirname(__file__), "golden", "paper_constants.txt")) as fh:
        consts = dict(line.split()[:2] for line in fh if line.strip() and not line.startswith("#"))
    bits_per_elem = Fraction(int(consts["reference_vector_bits"]), int(consts["ternary_iterations_per_reference"]))
    assert bits_per_elem == 2
    for d in (16, 1000, 1 << 20):
        assert O.words_per_row(d, 2) * 32 == -(-d // 16) * 32
        assert O.words_per_row(d, 2) * 32 - d * bits_per_elem < 32
    assert O.levels_of(2) == 1                                   # {-1, 0, +1}


def test_unemitted_code_decodes_to_zero():
    for bits in (2, 4):
        word = np.array([1 << (bits - 1)], dtype=np.uint32)      # sign bit with level 0
        level, neg = O.unpack(word, 1, bits)
        assert level[0] == 0 and not neg[0]
        assert O.dequantize(level, neg, F32(2.0), bits)[0] == 0
        assert not np.signbit(O.dequantize(level, neg, F32(2.0), bits)[0])


# ------------------------------------------------------------------ brute force (I9)
@pytest.mark.parametrize("bits", [2, 4])
@pytest.mark.parametrize("norm", [O.NORM_NONE, O.NORM_SUB, O.NORM_QUOT, O.NORM_COMB])
def test_vectorised_oracle_equals_elementwise_oracle_on_tiny_inputs(bits, norm):
    rng = np.random.default_rng(100 + 10 * bits + norm)
    cases = 0
    for trial in range(130):
        d = int(rng.integers(1, 17))
        M = int(rng.choice([1, 2, 3, 8]))
        seed = int(rng.integers(0, 1 << 63))
        it = int(rng.integers(0, 1 << 31))
        gref = rng.standard_normal(d).astype(F32)
        gref2 = rng.standard_normal(d).astype(F32)
        if trial % 5 == 0:
            gref[rng.integers(0, d)] = 0.0
            gref2[rng.integers(0, d)] = F32(-1e-10)
        g = (gref + rng.standard_normal((M, d)) * 10.0 ** rng.integers(-3, 3)).astype(F32)
        if trial % 7 == 0:
            g[0] = gref                                          # one worker with nothing to send
        cfg = O.Config(d=d, M=M, bits=bits, norm=norm, seed=seed)
        codes, scales = O.normalize_encode(cfg, it, g, gref, gref2)
        rows = []
        for m in range(M):
            words, R = S.encode_row([x for x in g[m]], list(gref), norm, cfg.quot_eps, bits, seed, it, m,
                                    list(gref2))
            assert [int(x) for x in codes[m]] == words
            assert scales[m] == R and scales.dtype == F32
            rows.append(words)
        vb = O.decode_aggregate(cfg, codes, scales, gref, d, gref2)
        vs = S.decode_mean(rows, list(scales), list(gref), norm, cfg.quot_eps, bits, d, list(gref2))
        assert vb.dtype == F32
        assert all(a == b or (np.isnan(a) and np.isnan(b)) for a, b in zip(vb, vs))
        cases += 1
    assert cases >= 125                                          # x 8 parametrisations >= 1000 (seed, t) pairs
