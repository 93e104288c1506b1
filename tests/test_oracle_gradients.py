"""Pins for the oracle's local-gradient functions.

Rosenbrock (section "Nonconvex Problems" of arXiv 1901.08227, generalised to the usual
d-dimensional chain): scipy's rosen / rosen_der, finite differences, the paper's minimum
f(1,1) = 0, and the textbook 2-D gradient.  Logistic regression (section "Convex
Problems"): finite differences of the mean log-loss written out here, the one-sample
closed form, and scipy's expit.
"""
import os

import numpy as np
import scipy.optimize
import scipy.special

from oracle import tng_oracle as O

F32 = np.float32


def _paper_constants():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")
    with open(path) as fh:
        return dict(line.split()[:2] for line in fh if line.strip() and not line.startswith("#"))


def test_rosenbrock_minimum_printed_in_the_paper():
    c = _paper_constants()
    xmin = np.array([float(c["rosenbrock_min_x"]), float(c["rosenbrock_min_y"])], dtype=F32)
    assert scipy.optimize.rosen(xmin.astype(np.float64)) == float(c["rosenbrock_min_f"])
    assert np.array_equal(O.grad_rosenbrock(xmin), np.zeros(2, dtype=F32))
    for d in (2, 3, 17, 1000):
        g = O.grad_rosenbrock(np.ones(d, dtype=F32))
        assert g.dtype == F32 and not g.any()                    # exactly zero at all-ones


def test_rosenbrock_two_dimensional_textbook_gradient():
    rng = np.random.default_rng(0)
    for _ in range(100):
        x, y = rng.uniform(-2, 2, 2)
        g = O.grad_rosenbrock(np.array([x, y], dtype=F32)).astype(np.float64)
        x, y = float(F32(x)), float(F32(y))
        expect = np.array([-400 * x * (y - x * x) - 2 * (1 - x), 200 * (y - x * x)])
        assert np.allclose(g, expect, rtol=1e-5, atol=1e-3)


def test_rosenbrock_chain_against_scipy_and_finite_differences():
    rng = np.random.default_rng(1)
    for d in (2, 3, 4, 5, 64, 1001):
        x = rng.uniform(-2, 2, d).astype(F32)
        g = O.grad_rosenbrock(x).astype(np.float64)
        ref = scipy.optimize.rosen_der(x.astype(np.float64))
        # forward error of the binary32 evaluation: a few ulps of the largest term (|terms| <= ~5e3)
        assert np.all(np.abs(g - ref) <= 8 * 2.0 ** -24 * 6000)
        if d <= 5:
            x64 = x.astype(np.float64)
            for i in range(d):
                e = np.zeros(d)
                e[i] = 1e-5
                fd = (scipy.optimize.rosen(x64 + e) - scipy.optimize.rosen(x64 - e)) / 2e-5
                assert abs(fd - ref[i]) < 1e-3 * max(1.0, abs(ref[i]))
    # end elements have one-sided stencils; d = 1 has an empty sum
    assert np.array_equal(O.grad_rosenbrock(np.array([0.3], dtype=F32)), np.zeros(1, dtype=F32))


def test_rosenbrock_noise_is_added_last_in_binary32():
    rng = np.random.default_rng(2)
    x = rng.uniform(-2, 2, 50).astype(F32)
    noise = (0.1 * rng.standard_normal(50)).astype(F32)
    clean = O.grad_rosenbrock(x)
    assert np.array_equal(O.grad_rosenbrock(x, noise), clean + noise)
    assert np.array_equal(O.grad_rosenbrock(x, np.zeros(50, dtype=F32)), clean)


def _logloss(X, y, w, l2):
    z = X @ w
    # -[y log s(z) + (1-y) log(1 - s(z))] = log(1 + e^z) - y z
    return np.mean(np.logaddexp(0.0, z) - y * z) + 0.5 * l2 * (w @ w)


def test_logistic_gradient_against_finite_differences_of_the_loss():
    rng = np.random.default_rng(3)
    n, d, B = 50, 7, 12
    X = rng.standard_normal((n, d)).astype(F32)
    y = rng.integers(0, 2, n).astype(F32)
    w = (0.5 * rng.standard_normal(d)).astype(F32)
    idx = rng.integers(0, n, B)
    idx[3] = idx[0]                                             # a repeated row counts twice
    for l2 in (0.0, 0.25):
        g = O.grad_logreg_dense(X, y, w, idx, l2)
        assert g.dtype == np.float64
        Xb, yb, w64 = X[idx].astype(np.float64), y[idx].astype(np.float64), w.astype(np.float64)
        for k in range(d):
            e = np.zeros(d)
            e[k] = 1e-6
            fd = (_logloss(Xb, yb, w64 + e, l2) - _logloss(Xb, yb, w64 - e, l2)) / 2e-6
            assert abs(fd - g[k]) < 1e-8 + 1e-6 * abs(g[k])


def test_logistic_gradient_single_sample_closed_form_and_sigmoid():
    rng = np.random.default_rng(4)
    X = rng.standard_normal((5, 9)).astype(F32)
    y = np.array([0, 1, 1, 0, 1], dtype=F32)
    w = rng.standard_normal(9).astype(F32)
    for i in range(5):
        g = O.grad_logreg_dense(X, y, w, np.array([i]))
        x = X[i].astype(np.float64)
        assert np.allclose(g, (scipy.special.expit(x @ w.astype(np.float64)) - y[i]) * x, rtol=1e-13, atol=0)
    z = np.array([-800.0, -40.0, -1.0, 0.0, 1.0, 40.0, 800.0])
    assert np.allclose(O.sigmoid64(z), scipy.special.expit(z), rtol=1e-15, atol=0)
    assert O.sigmoid64(np.array([0.0]))[0] == 0.5
    # at w = 0 the gradient is (1/B) sum (1/2 - y_i) x_i
    g0 = O.grad_logreg_dense(X, y, np.zeros(9, dtype=F32), np.arange(5))
    assert np.allclose(g0, ((0.5 - y.astype(np.float64))[:, None] * X.astype(np.float64)).mean(axis=0), rtol=1e-12)


def test_csr_gradient_equals_dense_gradient_of_the_same_matrix():
    rng = np.random.default_rng(5)
    n, d, k = 20, 40, 6
    dense = np.zeros((n, d), dtype=F32)
    rowptr = np.arange(n + 1, dtype=np.int64) * k
    col = np.zeros(n * k, dtype=np.int32)
    val = rng.standard_normal(n * k).astype(F32)
    for i in range(n):
        c = np.sort(rng.choice(d, k, replace=False))
        col[i * k:(i + 1) * k] = c
        dense[i, c] = val[i * k:(i + 1) * k]
    y = rng.integers(0, 2, n).astype(F32)
    w = rng.standard_normal(d).astype(F32)
    idx = rng.integers(0, n, 9)
    for l2 in (0.0, 0.1):
        a = O.grad_logreg_csr(rowptr, col, val, y, w, idx, d, l2)
        b = O.grad_logreg_dense(dense, y, w, idx, l2)
        assert np.allclose(a, b, rtol=1e-12, atol=1e-15)


def test_condition_term_of_the_gradient_tolerance_sparse_equals_dense():
    # the GPU tests bound fp32 cancellation by cond_k = (1/B) sum_i (|r_i| + Z_i/4) |x_ik| + |l2 w_k|; the
    # CSR form of that helper must equal the dense one on the densified rows
    from gpu_util import logistic_condition, logistic_condition_csr

    rng = np.random.default_rng(3)
    n, d, nnz = 20, 64, 7
    cols = np.stack([np.sort(rng.choice(d, nnz, replace=False)) for _ in range(n)]).astype(np.int32)
    vals = rng.standard_normal((n, nnz)).astype(np.float32)
    rowptr = np.arange(n + 1, dtype=np.int64) * nnz
    y = (rng.random(n) < 0.5).astype(np.float32)
    w = rng.standard_normal(d).astype(np.float32)
    ids = rng.integers(0, n, 13)
    Xb = np.zeros((len(ids), d), dtype=np.float32)
    for j, i in enumerate(ids):
        Xb[j, cols[i]] = vals[i]
    a = logistic_condition(Xb, y[ids], w, 0.01)
    b = logistic_condition_csr(rowptr, cols.reshape(-1), vals.reshape(-1), y, w, ids, d, 0.01)
    assert np.allclose(a, b, rtol=1e-12, atol=0)
