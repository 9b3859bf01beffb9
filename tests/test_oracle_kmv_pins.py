"""Pins for the oracle of the kernel matrix-vector product (paper section 5.1, appendix):
y = K v with the squared-exponential kernel k(x, z) = variance * exp(-|x - z|^2 / (2 l^2))."""
import numpy as np
import pytest

import workloads as W


def dense(X, Z, variance, l):
    Xd, Zd = X.astype(np.float64), Z.astype(np.float64)
    D = ((Xd[:, None, :] - Zd[None, :, :]) ** 2).sum(axis=2)
    return variance * np.exp(-0.5 * D / (l * l))


@pytest.mark.parametrize("seed,n,m,d,var,l", [(40, 30, 50, 1, 1.0, 1.0), (41, 25, 64, 3, 2.5, 0.7),
                                               (42, 10, 33, 8, 0.3, 3.0)])
def test_dense_matrix_times_vector(oracle, seed, n, m, d, var, l):
    X, Z = W.random_case(seed, n, m, d)  # (Q, X) of the generator serve as (X, Z)
    v = np.random.Generator(np.random.PCG64(seed)).standard_normal(m).astype(np.float32)
    y = oracle.kmv(X, Z, v, var, l)
    ref = dense(X, Z, var, l) @ v.astype(np.float64)
    np.testing.assert_allclose(y, ref, rtol=1e-12, atol=1e-13)


def test_closed_forms(oracle):
    # one point on itself: k = variance
    assert oracle.kmv([[1.5, -2.0]], [[1.5, -2.0]], [3.0], 0.25, 2.0)[0] == 0.75
    # two points at squared distance 2 l^2: k = variance / e
    y = oracle.kmv([[0.0, 0.0]], [[3.0, 3.0]], [1.0], 2.0, 3.0)
    assert y[0] == pytest.approx(2.0 / np.e, rel=1e-15)
    # lengthscale far beyond the data: every entry is the variance, y_i = variance * sum(v)
    X, Z = W.random_case(43, 5, 40, 4)
    v = np.arange(40, dtype=np.float32)
    y = oracle.kmv(X, Z, v, 1.5, 1e9)
    np.testing.assert_allclose(y, 1.5 * v.sum(), rtol=1e-12)
    # lengthscale far below the spacing of distinct points: only coincident points contribute
    Zs = np.array([[0.0], [1.0], [2.0]], dtype=np.float32)
    y = oracle.kmv(Zs, Zs, [5.0, 7.0, 11.0], 1.0, 1e-3)
    assert y.tolist() == [5.0, 7.0, 11.0]


def test_symmetry_linearity_and_positive_definiteness(oracle):
    X, _ = W.random_case(44, 60, 60, 2)
    g = np.random.Generator(np.random.PCG64(7))
    v = g.standard_normal(60).astype(np.float32)
    w = g.standard_normal(60).astype(np.float32)
    Kv = oracle.kmv(X, X, v, 1.3, 0.8)
    Kw = oracle.kmv(X, X, w, 1.3, 0.8)
    assert np.dot(w.astype(np.float64), Kv) == pytest.approx(np.dot(v.astype(np.float64), Kw), rel=1e-12)
    K2v = oracle.kmv(X, X, 2 * v, 1.3, 0.8)  # scaling by 2 is exact
    assert np.array_equal(K2v, 2 * Kv)
    assert np.dot(v.astype(np.float64), Kv) > 0
    rows = np.array([7, 0, 59], dtype=np.int64)
    assert np.array_equal(oracle.kmv(X, X, v, 1.3, 0.8, rows=rows), Kv[rows])
    assert np.array_equal(oracle.kmv(X, X, v, 1.3, 0.8, nthreads=1), Kv)


# ---- the fp64-input routine (the precision in which section 5.1 evaluates the product) ----
def test_f64_dense_matrix_times_vector(oracle):
    g = np.random.Generator(np.random.PCG64(45))
    for n, m, d, var, l in ((30, 50, 1, 1.0, 1.0), (12, 40, 5, 0.7, 1.9), (7, 33, 11, 2.0, 4.0)):
        X, Z, v = g.standard_normal((n, d)), g.standard_normal((m, d)), g.standard_normal(m)
        D = ((X[:, None, :] - Z[None, :, :]) ** 2).sum(axis=2)
        ref = (var * np.exp(-0.5 * D / (l * l))) @ v
        np.testing.assert_allclose(oracle.kmv_f64(X, Z, v, var, l), ref, rtol=1e-12, atol=1e-13)


def test_f64_closed_forms_and_structure(oracle):
    assert oracle.kmv_f64([[1.5, -2.0]], [[1.5, -2.0]], [3.0], 0.25, 2.0)[0] == 0.75
    assert oracle.kmv_f64([[0.0, 0.0]], [[3.0, 3.0]], [1.0], 2.0, 3.0)[0] == pytest.approx(2.0 / np.e, rel=1e-15)
    # inputs that fp32 cannot hold: a shift of 1e-9 at coordinate 1 moves the entry by the
    # derivative of the kernel, -k * (x - z) / l^2 * shift
    base = oracle.kmv_f64([[1.0]], [[0.0]], [1.0], 1.0, 1.0)[0]
    moved = oracle.kmv_f64([[1.0 + 1e-9]], [[0.0]], [1.0], 1.0, 1.0)[0]
    assert base == pytest.approx(np.exp(-0.5), rel=1e-15)
    assert (moved - base) == pytest.approx(-np.exp(-0.5) * 1e-9, rel=1e-6)
    g = np.random.Generator(np.random.PCG64(46))
    X, v, w = g.standard_normal((50, 3)), g.standard_normal(50), g.standard_normal(50)
    Kv, Kw = oracle.kmv_f64(X, X, v, 1.3, 0.8), oracle.kmv_f64(X, X, w, 1.3, 0.8)
    assert np.dot(w, Kv) == pytest.approx(np.dot(v, Kw), rel=1e-12)
    assert np.array_equal(oracle.kmv_f64(X, X, 2 * v, 1.3, 0.8), 2 * Kv)
    assert np.dot(v, Kv) > 0
    rows = np.array([7, 0, 49], dtype=np.int64)
    assert np.array_equal(oracle.kmv_f64(X, X, v, 1.3, 0.8, rows=rows), Kv[rows])
    assert np.array_equal(oracle.kmv_f64(X, X, v, 1.3, 0.8, nthreads=1), Kv)


def test_f64_routine_equals_the_f32_input_routine_on_f32_values(oracle):
    X, Z = W.random_case(47, 20, 70, 6)
    v = np.random.Generator(np.random.PCG64(47)).standard_normal(70).astype(np.float32)
    a = oracle.kmv(X, Z, v, 0.9, 1.7)
    b = oracle.kmv_f64(X.astype(np.float64), Z.astype(np.float64), v.astype(np.float64), 0.9, 1.7)
    assert np.array_equal(a, b)
