"""Pins for the server-side half of the oracle and for the whole iteration.

Fixed by the paper (arXiv 1901.08227): w_{t+1} = w_t - eta (1/M) sum_m Q[g^m] (Background),
v = g~ + r (Eq. 1), the reference "updated to be the averaged compressed TNG from the last
iteration" (Convex Problems), the refresh period (16 in Nonconvex Problems), g~ = zeros at
the start (Algorithm 1), and the claim that normalisation shrinks what has to be coded
(Proposition 2: E||g - g~||^2 <= C_nz E||g||^2 with C_nz <= 1).
"""
import os

import numpy as np

from oracle import tng_oracle as O

F32 = np.float32


def _consts():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")
    with open(path) as fh:
        return dict(line.split()[:2] for line in fh if line.strip() and not line.startswith("#"))


def test_server_average_is_the_mean_of_decoded_workers_plus_reference():
    rng = np.random.default_rng(0)
    d, M = 200, 5
    gref = rng.standard_normal(d).astype(F32)
    g = (gref + 0.1 * rng.standard_normal((M, d))).astype(F32)
    for bits in (2, 4):
        cfg = O.Config(d=d, M=M, bits=bits, norm=O.NORM_SUB, seed=4)
        codes, scales = O.normalize_encode(cfg, 0, g, gref)
        rows = np.stack([O.dequantize(*O.unpack(codes[m], d, bits), scales[m], bits) for m in range(M)])
        expect = gref.astype(np.float64) + rows.astype(np.float64).mean(axis=0)     # Eq. 1 on the server
        got = O.decode_aggregate(cfg, codes, scales, gref, d)
        assert got.dtype == F32
        assert np.allclose(got, expect, rtol=1e-6, atol=1e-7)
        # with one worker and the top level everywhere the decode is exact
    one = O.Config(d=4, M=1, bits=2, norm=O.NORM_NONE, seed=0)
    codes = O.pack(np.array([1, 1, 0, 1]), np.array([False, True, False, False]), 2)[None, :]
    out = O.decode_aggregate(one, codes, np.array([2.5], dtype=F32), np.zeros(4, dtype=F32), 4)
    assert np.array_equal(out, np.array([2.5, -2.5, 0.0, 2.5], dtype=F32))


def test_iterate_update_is_plain_sgd_on_the_decoded_average():
    rng = np.random.default_rng(1)
    w = rng.standard_normal(100).astype(F32)
    v = rng.standard_normal(100).astype(F32)
    out = O.update_iterate(w, v, 0.1)
    assert out.dtype == F32
    assert np.allclose(out, w.astype(np.float64) - 0.1 * v.astype(np.float64), rtol=1e-6, atol=1e-7)
    assert np.array_equal(out, w - F32(0.1) * v)                # product rounded, then difference rounded
    assert np.array_equal(O.update_iterate(w, np.zeros(100, dtype=F32), 0.1), w)


def test_reference_refresh_rule_and_period():
    K = int(_consts()["reference_update_period"])                # 16 in the non-convex experiments
    d = 8
    gref = np.arange(d, dtype=F32)
    cfg = O.Config(d=d, M=1, ref_policy=O.REF_LAST_AVG, ref_period=K)
    refreshed = []
    for it in range(3 * K):
        vbar = np.full(d, it, dtype=F32)
        new = O.update_reference(cfg, it, vbar, gref)
        if not np.array_equal(new, gref):
            refreshed.append(it)
            assert np.array_equal(new, vbar)
        gref = new
    assert refreshed == [K - 1, 2 * K - 1, 3 * K - 1]           # once every K iterations
    every = O.Config(d=d, M=1, ref_policy=O.REF_LAST_AVG, ref_period=1)
    assert np.array_equal(O.update_reference(every, 0, np.ones(d, dtype=F32), gref), np.ones(d, dtype=F32))
    never = O.Config(d=d, M=1, ref_policy=O.REF_ZERO, ref_period=1)
    z = np.zeros(d, dtype=F32)
    assert np.array_equal(O.update_reference(never, 0, np.ones(d, dtype=F32), z), z)


def test_window_average_reference():
    d = 5
    cfg = O.Config(d=d, M=1, ref_policy=O.REF_WINDOW_AVG, ref_period=1, ref_window=4)
    hist = []
    gref = np.zeros(d, dtype=F32)
    for it in range(8):
        vbar = np.full(d, float(it + 1), dtype=F32)
        hist.append(vbar)
        gref = O.update_reference(cfg, it, vbar, gref, hist)
        last = [float(x[0]) for x in hist[-4:]]
        assert np.allclose(gref, sum(last) / 4.0)               # missing history counts as zeros


def test_whole_iteration_composes_the_parts():
    rng = np.random.default_rng(2)
    d, M = 130, 3
    cfg = O.Config(d=d, M=M, bits=4, norm=O.NORM_SUB, seed=8, lr=0.05, ref_period=2)
    w = rng.standard_normal(d).astype(F32)
    gref = rng.standard_normal(d).astype(F32)
    g = rng.standard_normal((M, d)).astype(F32)
    for it in (0, 1):
        w2, gref2, codes, scales, vbar = O.step(cfg, it, w, gref, g)
        c, s = O.normalize_encode(cfg, it, g, gref)
        assert np.array_equal(c, codes) and np.array_equal(s, scales)
        assert np.array_equal(vbar, O.decode_aggregate(cfg, c, s, gref, d))
        assert np.array_equal(w2, O.update_iterate(w, vbar, cfg.lr))
        assert np.array_equal(gref2, vbar if it == 1 else gref)


def test_threaded_composition_used_by_the_large_gpu_tests_equals_the_whole_iteration():
    # tests/gpu_util.oracle_step_threaded shares the oracle's work between host threads (workers, then
    # blocks of coordinates); it must give what O.step gives, bit for bit, ragged blocks included
    from gpu_util import oracle_step_threaded

    rng = np.random.default_rng(4)
    for d, M, bits, norm, block in [(1000, 5, 2, O.NORM_SUB, 64), (4099, 3, 4, O.NORM_QUOT, 1024),
                                    (333, 2, 4, O.NORM_NONE, 16), (70, 9, 2, O.NORM_SUB, 1 << 22)]:
        cfg = O.Config(d=d, M=M, bits=bits, norm=norm, seed=21, lr=0.05, ref_period=2)
        w = rng.standard_normal(d).astype(F32)
        gref = rng.standard_normal(d).astype(F32)
        gref[::5] = 0
        g = rng.standard_normal((M, d)).astype(F32)
        for it in (0, 1):
            want = O.step(cfg, it, w, gref, g)
            got = oracle_step_threaded(cfg, it, w, gref, g, threads=3, block=block)
            for a, b in zip(want, got):
                assert np.array_equal(a, b)


def _run_logistic(norm_cfg, T=60):
    """Small copy of the dense logistic workload: returns (losses, C_nz estimates, coder MSE)."""
    rng = np.random.default_rng(5)
    M, n, d, B = 4, 400, 100, 64
    w_star = rng.standard_normal(d) / np.sqrt(d)
    X = rng.standard_normal((M, n, d)).astype(F32)
    y = (rng.random((M, n)) < 1 / (1 + np.exp(-(X @ w_star)))).astype(F32)
    w = np.zeros(d, dtype=F32)
    gref = np.zeros(d, dtype=F32)
    losses, cnz, mse = [], [], []
    Xa, ya = X.reshape(-1, d).astype(np.float64), y.reshape(-1).astype(np.float64)
    for it in range(T):
        g = np.stack([O.grad_logreg_dense(X[m], y[m], w, O.minibatch_indices(norm_cfg.seed, it, m, B, n))
                      for m in range(M)]).astype(F32)
        w2, gref2, codes, scales, vbar = O.step(norm_cfg, it, w, gref, g)
        z = Xa @ w.astype(np.float64)
        losses.append(float(np.mean(np.logaddexp(0, z) - ya * z)))
        cnz.append(float(((g - gref) ** 2).sum() / (g ** 2).sum()))
        mse.append(float(((vbar - g.mean(axis=0)) ** 2).sum()))
        w, gref = w2, gref2
    return np.array(losses), np.array(cnz), np.array(mse)


def test_logistic_runs_optimise_with_and_without_a_trajectory_reference():
    tng = O.Config(d=100, M=4, bits=2, norm=O.NORM_SUB, ref_policy=O.REF_LAST_AVG, ref_period=1, seed=0, lr=0.1)
    base = O.Config(d=100, M=4, bits=2, norm=O.NORM_SUB, ref_policy=O.REF_ZERO, ref_period=1, seed=0, lr=0.1)
    loss_t, cnz_t, mse_t = _run_logistic(tng)
    loss_b, cnz_b, mse_b = _run_logistic(base)
    assert np.all(cnz_b == 1.0)                                  # zeros reference: the trivial C_nz = 1
    assert loss_t[-1] < 0.9 * loss_t[0] and loss_b[-1] < 0.9 * loss_b[0]     # both optimise
    assert abs(loss_t[0] - np.log(2.0)) < 1e-12 and loss_t[0] == loss_b[0]   # w_0 = 0
    assert mse_t[0] == mse_b[0]                                  # iteration 0 codes against zeros in both runs
    assert np.all(np.isfinite(loss_t)) and np.all(np.isfinite(cnz_t))


def test_trajectory_reference_shrinks_the_coded_vector_when_gradients_are_persistent():
    """Sanity, not parity: on the noisy Rosenbrock chain consecutive gradients are close, so
    coding g - g~ (g~ = last decoded average) has C_nz << 1 and a smaller coding error than
    coding g itself at equal bits -- the effect the paper is about."""
    rng = np.random.default_rng(6)
    d, M, T = 512, 8, 40
    x0 = rng.uniform(-2, 2, d).astype(F32)
    noise = (0.1 * rng.standard_normal((T, M, d))).astype(F32)

    def run(policy):
        cfg = O.Config(d=d, M=M, bits=2, norm=O.NORM_SUB, ref_policy=policy, ref_period=1, seed=1, lr=1e-5)
        x, gref = x0.copy(), np.zeros(d, dtype=F32)
        cnz, err = [], []
        for it in range(T):
            g = np.stack([O.grad_rosenbrock(x, noise[it, m]) for m in range(M)])
            x2, gref2, _, _, vbar = O.step(cfg, it, x, gref, g)
            cnz.append(float(((g - gref) ** 2).sum() / (g ** 2).sum()))
            err.append(float(((vbar - g.mean(axis=0)) ** 2).sum()))
            x, gref = x2, gref2
        return np.array(cnz), np.array(err)

    cnz_t, err_t = run(O.REF_LAST_AVG)
    cnz_b, err_b = run(O.REF_ZERO)
    assert np.all(cnz_b == 1.0) and cnz_t[0] == 1.0
    assert np.median(cnz_t[5:]) < 0.05
    assert np.median(err_t[5:]) < 0.05 * np.median(err_b[5:])
