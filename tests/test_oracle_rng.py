"""Pins for the oracle's counter-based RNG (Philox4x32-10, Salmon et al., SC'11).

No library on the CPU side implements Philox4x32, and the published known-answer vectors
are not available here, so the generator is pinned by: constants that have a closed form,
the invertibility its round structure implies, two independently written implementations
agreeing, and distribution / diffusion statistics that a dropped round, a swapped lane or a
wrong shift would break.  A cross-check against rocRAND's generator runs with the GPU tests.
"""
import math

import numpy as np

from oracle import tng_oracle as O
from oracle import tng_scalar as S

M0, M1 = 0xD2511F53, 0xCD9E8D57
MASK = 0xFFFFFFFF


def test_weyl_constants_have_their_closed_form():
    # key increments are the fractional parts of the golden ratio and of sqrt(3), scaled by 2^32
    golden = (math.isqrt(5 << 64) - (1 << 32)) >> 1
    sqrt3m1 = math.isqrt(3 << 64) - (1 << 32)
    assert O.PHILOX_W0 == golden == 0x9E3779B9
    assert O.PHILOX_W1 == sqrt3m1 == 0xBB67AE85
    # the multipliers must be odd (otherwise a round is not a bijection)
    assert O.PHILOX_M0 % 2 == 1 and O.PHILOX_M1 % 2 == 1


def test_vector_and_scalar_implementations_agree():
    rng = np.random.default_rng(1)
    ctr = rng.integers(0, 1 << 32, size=(500, 4), dtype=np.uint64)
    key = rng.integers(0, 1 << 32, size=(500, 2), dtype=np.uint64)
    for i in range(500):
        vec = O.philox4x32_10(ctr[i, 0:1], int(ctr[i, 1]), int(ctr[i, 2]), int(ctr[i, 3]),
                              int(key[i, 0]), int(key[i, 1]))
        assert [int(x[0]) for x in vec] == S.philox_block(ctr[i], key[i])
    # extreme words
    for c in [(0, 0, 0, 0), (MASK, MASK, MASK, MASK), (1, 0, 0, 0), (0, 0, 0, 1)]:
        for k in [(0, 0), (MASK, MASK)]:
            vec = O.philox4x32_10(np.array([c[0]]), c[1], c[2], c[3], k[0], k[1])
            assert [int(x[0]) for x in vec] == S.philox_block(c, k)


def _invert(block, key):
    """Undo 10 rounds using the modular inverses of the multipliers (test-only code)."""
    inv0, inv1 = pow(M0, -1, 1 << 32), pow(M1, -1, 1 << 32)
    keys = [((key[0] + r * 0x9E3779B9) & MASK, (key[1] + r * 0xBB67AE85) & MASK) for r in range(10)]
    y = list(block)
    for r in reversed(range(10)):
        c2 = (y[1] * inv1) & MASK
        c0 = (y[3] * inv0) & MASK
        c1 = y[0] ^ ((M1 * c2) >> 32) ^ keys[r][0]
        c3 = y[2] ^ ((M0 * c0) >> 32) ^ keys[r][1]
        y = [c0, c1, c2, c3]
    return y


def test_rounds_are_a_bijection_of_the_counter():
    rng = np.random.default_rng(2)
    for _ in range(200):
        c = [int(x) for x in rng.integers(0, 1 << 32, size=4, dtype=np.uint64)]
        k = [int(x) for x in rng.integers(0, 1 << 32, size=2, dtype=np.uint64)]
        out = O.philox4x32_10(np.array([c[0]]), c[1], c[2], c[3], k[0], k[1])
        assert _invert([int(x[0]) for x in out], k) == c


def test_single_bit_of_counter_or_key_flips_half_the_output_bits():
    # full diffusion after 10 rounds: avalanche close to 64 of 128 bits for every input bit
    base_c = np.arange(2000, dtype=np.uint64)

    def bits(words):
        return np.unpackbits(np.stack(words, 1).astype(">u4").view(np.uint8), axis=1)

    ref = bits(O.philox4x32_10(base_c, 3, 5, 0, 11, 13))
    for word in range(4):
        for bit in (0, 7, 31):
            c = [base_c, np.uint64(3), np.uint64(5), np.uint64(0)]
            c[word] = c[word] ^ np.uint64(1 << bit)
            flipped = bits(O.philox4x32_10(c[0], c[1], c[2], c[3], 11, 13)) ^ ref
            assert abs(flipped.mean() - 0.5) < 0.01
            assert np.all(np.abs(flipped.mean(axis=0) - 0.5) < 0.06)   # every output bit moves
    for kbit in (0, 31):
        flipped = bits(O.philox4x32_10(base_c, 3, 5, 0, 11 ^ (1 << kbit), 13)) ^ ref
        assert abs(flipped.mean() - 0.5) < 0.01
        flipped = bits(O.philox4x32_10(base_c, 3, 5, 0, 11, 13 ^ (1 << kbit))) ^ ref
        assert abs(flipped.mean() - 0.5) < 0.01


def test_draws_are_uniform_and_uncorrelated():
    n = 1 << 20
    x = O.quant_draw_words(seed=42, it=7, m=3, d=n)
    u = O.uniform_from_word(x).astype(np.float64)
    assert u.min() >= 0.0 and u.max() < 1.0
    assert abs(u.mean() - 0.5) < 5 * math.sqrt(1 / 12 / n)
    assert abs(u.var() - 1 / 12) < 1e-3
    for lane in range(4):                                  # each Philox output lane on its own
        counts = np.bincount((x[lane::4] >> 24).astype(np.int64), minlength=256)
        expected = (n // 4) / 256
        chi2 = ((counts - expected) ** 2 / expected).sum()
        assert chi2 < 255 + 6 * math.sqrt(2 * 255)
    low = np.bincount((x & 0xFF).astype(np.int64), minlength=256)   # low byte too
    assert ((low - n / 256) ** 2 / (n / 256)).sum() < 255 + 6 * math.sqrt(2 * 255)
    lag1 = np.corrcoef(u[:-1], u[1:])[0, 1]
    assert abs(lag1) < 5 / math.sqrt(n)


def test_sequences_differ_across_iteration_worker_stream_and_seed():
    a = O.quant_draw_words(1, 0, 0, 4096)
    assert not np.array_equal(a, O.quant_draw_words(1, 1, 0, 4096))
    assert not np.array_equal(a, O.quant_draw_words(1, 0, 1, 4096))
    assert not np.array_equal(a, O.quant_draw_words(2, 0, 0, 4096))
    assert not np.array_equal(a, O.quant_draw_words(1 + (1 << 32), 0, 0, 4096))   # high seed word is used
    assert not np.array_equal(a, O._draw_words(1, 0, 0, O.STREAM_BATCH, 0, 4096))
    # agreement rate between different sequences is what chance gives (2^-32): none expected
    assert np.count_nonzero(a == O.quant_draw_words(1, 1, 0, 4096)) == 0


def test_draw_is_a_function_of_the_element_index_only():
    # element e always gets lane e & 3 of block e >> 2, whatever window is asked for
    whole = O.quant_draw_words(9, 4, 2, 1000)
    for first, count in [(0, 1), (1, 7), (3, 2), (4, 4), (997, 3), (250, 333)]:
        assert np.array_equal(O.quant_draw_words(9, 4, 2, count, first=first), whole[first:first + count])
    for e in (0, 1, 5, 999):
        assert int(whole[e]) == S.draw(9, 4, 2, 0, e)
        assert int(whole[e]) == S.philox_block((e >> 2, 2, 4, 0), (9, 0))[e & 3]


def test_uniform_is_the_24_bit_grid():
    k = np.arange(1 << 24, dtype=np.uint32)
    u = O.uniform_from_word(k << np.uint32(8))
    assert u.dtype == np.float32
    assert np.array_equal(u.astype(np.float64) * (1 << 24), k.astype(np.float64))   # exact, no rounding
    # the low 8 bits of the word are ignored
    assert np.array_equal(O.uniform_from_word((k[:4096] << np.uint32(8)) | np.uint32(0xFF)), u[:4096])
    assert float(S.uniform(0xFFFFFFFF)) == 1.0 - 2.0 ** -24


def test_minibatch_indices_definition_range_and_uniformity():
    for n_rows in (1, 2, 7, 2000, 65536, (1 << 32) - 1):
        idx = O.minibatch_indices(seed=5, it=3, m=1, batch=37, n_rows=n_rows)
        assert idx.shape == (37,) and idx.min() >= 0 and idx.max() < n_rows
        for j in range(37):
            x = S.philox_block((j >> 2, 1, 3, 1), (5, 0))[j & 3]
            assert int(idx[j]) == (x * n_rows) // (1 << 32) == S.batch_index(5, 3, 1, j, n_rows)
    n_rows, batch = 64, 1 << 16
    counts = np.bincount(O.minibatch_indices(0, 0, 0, batch, n_rows), minlength=n_rows)
    chi2 = ((counts - batch / n_rows) ** 2 / (batch / n_rows)).sum()
    assert chi2 < 63 + 6 * math.sqrt(2 * 63)
    # different workers and iterations draw different batches
    assert not np.array_equal(O.minibatch_indices(0, 0, 0, 64, 2000), O.minibatch_indices(0, 0, 1, 64, 2000))
    assert not np.array_equal(O.minibatch_indices(0, 0, 0, 64, 2000), O.minibatch_indices(0, 1, 0, 64, 2000))
