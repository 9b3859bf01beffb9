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
