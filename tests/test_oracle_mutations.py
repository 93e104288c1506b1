"""Are the pins sharp?  Plant one plausible mistake at a time in the oracle (on the CPU, by
monkeypatching) and require that some pin test fails.  Each mistake is one a reader of the
paper could really make, several of them being the paper's own slips in Algorithm 1.
"""
import numpy as np
import pytest

from oracle import tng_oracle as O

import test_oracle_gradients as TG
import test_oracle_quantizer as TQ
import test_oracle_rng as TR
import test_oracle_step as TS

F32 = np.float32


def _fails(checks):
    for fn, args in checks:
        try:
            fn(*args)
        except AssertionError:
            return True
    return False


QUANT_PINS = [   # cheapest first: a mutation test stops at the first pin that fails
    (TQ.test_reference_clamp_for_the_quotient, ()),
    (TQ.test_pack_layout_every_position_and_code_value, (4,)),
    (TS.test_server_average_is_the_mean_of_decoded_workers_plus_reference, ()),
    (TQ.test_gradient_equal_to_reference_is_reconstructed_exactly, (4,)),
    (TQ.test_largest_element_keeps_its_full_magnitude, (4,)),
    (TQ.test_ternary_probabilities_are_magnitude_over_R, ()),
    (TQ.test_decoded_mean_over_many_draws_converges_to_the_input, (4, O.NORM_SUB)),
    (TQ.test_decoded_mean_over_many_draws_converges_to_the_input, (2, O.NORM_QUOT)),
    (TQ.test_rounding_probability_is_exact_on_the_24_bit_grid, (2,)),
]


def test_pins_pass_on_the_unmodified_oracle():
    assert not _fails(QUANT_PINS)


def _m_round_up_on_tie(mp):
    def quantize(v, R, bits, u):
        v = np.asarray(v, dtype=F32)
        s = O.levels_of(bits)
        if R == 0:
            z = np.zeros(v.shape, dtype=np.int32)
            return z, z.astype(bool)
        x = np.minimum(np.abs(v) * (F32(1) / F32(R)), F32(1)) * F32(s)
        lo = x.astype(np.int32)
        level = lo + (np.asarray(u, dtype=F32) <= x - lo.astype(F32)).astype(np.int32)
        return np.minimum(level, s), (v < 0) & (level > 0)
    mp.setattr(O, "quantize", quantize)


def _m_sign_of_g_instead_of_normalised(mp):          # Algorithm 1 as printed: sign(g), not sign(g - g~)
    orig_ne = O.normalize_encode

    def normalize_encode(cfg, it, g, gref, gref2=None, means=None):
        codes, scales = orig_ne(cfg, it, g, gref, gref2, means)
        for m in range(g.shape[0]):
            level, _ = O.unpack(codes[m], g.shape[1], cfg.bits)
            codes[m] = O.pack(level, (g[m] < 0) & (level > 0), cfg.bits)
        return codes, scales
    mp.setattr(O, "normalize_encode", normalize_encode)


def _m_server_forgets_reference(mp):                 # Algorithm 1 as printed: average without + g~
    mp.setattr(O, "denormalize", lambda mean, gref, norm, eps=1e-8, gref2=None: np.asarray(mean, dtype=F32).copy())


def _m_signed_max(mp):
    mp.setattr(O, "scale_of", lambda v, kind=0: F32(np.max(v)) if np.size(v) else F32(0))


def _m_subtraction_reversed(mp):
    orig = O.normalize
    mp.setattr(O, "normalize", lambda g, gref, norm, eps=1e-8, gref2=None, mu=None:
               (np.asarray(gref, dtype=F32) - np.asarray(g, dtype=F32)) if norm == O.NORM_SUB
               else orig(g, gref, norm, eps, gref2, mu))


def _m_top_level_through_step(mp):
    def dequantize(level, neg, R, bits):
        mag = (F32(R) / F32(O.levels_of(bits))) * np.asarray(level).astype(F32)
        return np.where(neg, -mag, mag).astype(F32)
    mp.setattr(O, "dequantize", dequantize)


def _m_big_endian_packing(mp):
    def pack(level, neg, bits):
        code = np.asarray(level).astype(np.uint32) | (np.asarray(neg).astype(np.uint32) << np.uint32(bits - 1))
        per = 32 // bits
        nw = O.words_per_row(code.shape[0], bits)
        padded = np.zeros(nw * per, dtype=np.uint32)
        padded[:code.shape[0]] = code
        shifts = ((per - 1 - np.arange(per, dtype=np.uint32)) * np.uint32(bits))[None, :]
        return np.bitwise_or.reduce(padded.reshape(nw, per) << shifts, axis=1).astype(np.uint32)
    mp.setattr(O, "pack", pack)


def _m_clamp_loses_sign(mp):
    mp.setattr(O, "clamp_reference", lambda gref, eps: np.where(np.abs(gref) < F32(eps), F32(eps), gref).astype(F32))


def _m_mean_over_wrong_count(mp):
    orig = O.decode_aggregate

    def decode_aggregate(cfg, codes, scales, gref, d, gref2=None, means=None):
        extra = np.concatenate([codes, np.zeros_like(codes[:1])])
        return orig(cfg, extra, np.concatenate([scales, np.zeros(1, dtype=F32)]), gref, d, gref2, means)
    mp.setattr(O, "decode_aggregate", decode_aggregate)


@pytest.mark.parametrize("mutate", [
    _m_round_up_on_tie, _m_sign_of_g_instead_of_normalised, _m_server_forgets_reference, _m_signed_max,
    _m_subtraction_reversed, _m_top_level_through_step, _m_big_endian_packing, _m_clamp_loses_sign,
    _m_mean_over_wrong_count,
])
def test_a_planted_mistake_in_the_coder_is_caught(mutate, monkeypatch):
    mutate(monkeypatch)
    assert _fails(QUANT_PINS)


def test_planted_mistakes_in_rng_use_are_caught(monkeypatch):
    with monkeypatch.context() as mp:                            # 23-bit uniforms
        mp.setattr(O, "uniform_from_word",
                   lambda x: (np.asarray(x, dtype=np.uint32) >> np.uint32(9)).astype(F32) * F32(2.0 ** -23))
        assert _fails([(TR.test_uniform_is_the_24_bit_grid, ())])
    with monkeypatch.context() as mp:                            # counter words for worker and iteration swapped
        orig = O.philox4x32_10
        mp.setattr(O, "philox4x32_10", lambda c0, c1, c2, c3, k0, k1: orig(c0, c2, c1, c3, k0, k1))
        assert _fails([(TR.test_draw_is_a_function_of_the_element_index_only, ())])
    with monkeypatch.context() as mp:                            # nine rounds
        def nine(c0, c1, c2, c3, k0, k1):
            c = [np.asarray(x, dtype=np.uint64) for x in np.broadcast_arrays(c0, c1, c2, c3)]
            for _ in range(9):
                p0, p1 = c[0] * np.uint64(O.PHILOX_M0), c[2] * np.uint64(O.PHILOX_M1)
                c = [(p1 >> np.uint64(32)) ^ c[1] ^ np.uint64(k0), p1 & np.uint64(0xFFFFFFFF),
                     (p0 >> np.uint64(32)) ^ c[3] ^ np.uint64(k1), p0 & np.uint64(0xFFFFFFFF)]
                k0, k1 = (k0 + O.PHILOX_W0) & 0xFFFFFFFF, (k1 + O.PHILOX_W1) & 0xFFFFFFFF
            return tuple(x.astype(np.uint32) for x in c)
        mp.setattr(O, "philox4x32_10", nine)
        assert _fails([(TR.test_vector_and_scalar_implementations_agree, ())])
    with monkeypatch.context() as mp:                            # batch index scaled by the wrong power of two
        mp.setattr(O, "minibatch_indices", lambda seed, it, m, batch, n_rows:
                   ((O._draw_words(seed, it, m, 1, 0, batch).astype(np.uint64) * np.uint64(n_rows)) >> np.uint64(33))
                   .astype(np.int64))
        assert _fails([(TR.test_minibatch_indices_definition_range_and_uniformity, ())])


def test_planted_mistakes_in_gradients_and_updates_are_caught(monkeypatch):
    with monkeypatch.context() as mp:                            # Rosenbrock with the roles swapped as the paper prints it
        def swapped(x, noise=None):
            x = np.asarray(x, dtype=F32)
            g = np.zeros_like(x)
            g[:-1] += F32(200) * (x[:-1] - x[1:] * x[1:]) + F32(2) * (x[:-1] - F32(1))
            g[1:] += F32(-400) * x[1:] * (x[:-1] - x[1:] * x[1:])
            return g if noise is None else g + noise
        mp.setattr(O, "grad_rosenbrock", swapped)
        assert _fails([(TG.test_rosenbrock_chain_against_scipy_and_finite_differences, ())])
    with monkeypatch.context() as mp:                            # sum instead of mean over the batch
        orig = O.grad_logreg_dense
        mp.setattr(O, "grad_logreg_dense", lambda X, y, w, idx, l2=0.0: orig(X, y, w, idx, l2) * len(idx))
        assert _fails([(TG.test_logistic_gradient_against_finite_differences_of_the_loss, ())])
    with monkeypatch.context() as mp:                            # labels taken as -1/+1
        orig = O.grad_logreg_dense
        mp.setattr(O, "grad_logreg_dense", lambda X, y, w, idx, l2=0.0: orig(X, 2 * np.asarray(y) - 1, w, idx, l2))
        assert _fails([(TG.test_logistic_gradient_single_sample_closed_form_and_sigmoid, ())])
    with monkeypatch.context() as mp:                            # refresh at the start of a period, not its end
        def early(cfg, it, vbar, gref, history=None):
            return np.asarray(vbar if it % cfg.ref_period == 0 else gref, dtype=F32).copy()
        mp.setattr(O, "update_reference", early)
        assert _fails([(TS.test_reference_refresh_rule_and_period, ())])
    with monkeypatch.context() as mp:                            # ascent instead of descent
        mp.setattr(O, "update_iterate", lambda w, v, lr: np.asarray(w, dtype=F32) + F32(lr) * np.asarray(v, dtype=F32))
        assert _fails([(TS.test_iterate_update_is_plain_sgd_on_the_decoded_average, ())])


def test_planted_mistakes_in_row_sums_mean_reference_and_noise_are_caught(monkeypatch):
    import test_oracle_noise as TN
    import test_oracle_sums as TSUM
    with monkeypatch.context() as mp:                            # plain left-to-right float64 sum
        mp.setattr(O, "tree_sum64", lambda x: np.float64(np.cumsum(np.asarray(x, dtype=np.float64))[-1])
                   if np.size(x) else np.float64(0.0))
        assert _fails([(TSUM.test_ordered_sum_is_a_sum_and_has_the_stated_order, ())])
    with monkeypatch.context() as mp:                            # mean accumulated in float32
        mp.setattr(O, "worker_mean", lambda g: F32(np.add.reduce(np.asarray(g, dtype=F32), dtype=F32) / F32(len(g))))
        assert _fails([(TSUM.test_worker_mean_is_the_mean, ())])
    with monkeypatch.context() as mp:                            # the server does not add the workers' means back
        orig = O.decode_aggregate
        mp.setattr(O, "decode_aggregate", lambda cfg, codes, scales, gref, d, gref2=None, means=None:
                   orig(cfg, codes, scales, gref, d, gref2, None if means is None else np.zeros_like(means)))
        assert _fails([(TSUM.test_mean_reference_round_trip_is_unbiased_and_matches_elementwise_oracle, (2,))])
    with monkeypatch.context() as mp:                            # squared norm instead of the norm
        orig = O.scale_of
        mp.setattr(O, "scale_of", lambda v, kind=0: orig(v, kind) if kind == 0 else F32(float(orig(v, kind)) ** 2))
        assert _fails([(TSUM.test_l2_scale, (2,))])
    with monkeypatch.context() as mp:                            # Box-Muller radius without the factor 2
        orig = O.gaussian_noise
        mp.setattr(O, "gaussian_noise", lambda seed, it, m, d, variance: orig(seed, it, m, d, variance) / np.sqrt(2.0))
        assert _fails([(TN.test_noise_is_normal_with_the_requested_variance, ())])
    with monkeypatch.context() as mp:                            # cosine and sine branches swapped
        orig = O.gaussian_noise

        def swapped(seed, it, m, d, variance):
            z = orig(seed, it, m, d + (d & 1), variance).reshape(-1, 2)[:, ::-1].reshape(-1)
            return z[:d]
        mp.setattr(O, "gaussian_noise", swapped)
        assert _fails([(TN.test_element_to_draw_mapping_with_the_scalar_generator, ())])
