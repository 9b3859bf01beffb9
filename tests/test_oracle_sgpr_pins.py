"""Pins for the oracle of the SGPR accumulations (paper section 5.3): A = K_uf K_fu and
b = K_uf y with the squared-exponential kernel between m inducing points and n data points."""
import numpy as np
import pytest

import workloads as W


def dense_kuf(U, X, variance, l):
    Ud, Xd = U.astype(np.float64), X.astype(np.float64)
    D = ((Ud[:, None, :] - Xd[None, :, :]) ** 2).sum(axis=2)
    return variance * np.exp(-0.5 * D / (l * l))


@pytest.mark.parametrize("seed,m,n,d,var,l", [(60, 7, 50, 1, 1.0, 1.0), (61, 20, 133, 3, 2.5, 0.7),
                                               (62, 5, 64, 11, 0.3, 3.0)])
def test_dense_products(oracle, seed, m, n, d, var, l):
    U, X = W.random_case(seed, m, n, d)  # (Q, X) of the generator serve as (U, X)
    y = np.random.Generator(np.random.PCG64(seed)).standard_normal(n).astype(np.float32)
    A, b = oracle.sgpr_accumulate(U, X, y, var, l)
    Kuf = dense_kuf(U, X, var, l)
    np.testing.assert_allclose(A, Kuf @ Kuf.T, rtol=1e-12, atol=1e-14)
    np.testing.assert_allclose(b, Kuf @ y.astype(np.float64), rtol=1e-12, atol=1e-13)


def test_closed_forms(oracle):
    # one inducing point on one data point: K_uf = variance
    A, b = oracle.sgpr_accumulate([[1.0, 2.0]], [[1.0, 2.0]], [3.0], 0.5, 1.0)
    assert A[0, 0] == 0.25 and b[0] == 1.5
    # squared distance 2 l^2: K_uf = variance / e
    A, b = oracle.sgpr_accumulate([[0.0, 0.0]], [[3.0, 3.0]], [2.0], 2.0, 3.0)
    assert A[0, 0] == pytest.approx(4.0 / np.e ** 2, rel=1e-15)
    assert b[0] == pytest.approx(4.0 / np.e, rel=1e-15)
    # lengthscale far beyond the data: every K_uf entry is the variance
    U, X = W.random_case(63, 4, 30, 3)
    y = np.arange(30, dtype=np.float32)
    A, b = oracle.sgpr_accumulate(U, X, y, 1.5, 1e9)
    np.testing.assert_allclose(A, np.full((4, 4), 30 * 1.5 ** 2), rtol=1e-12)
    np.testing.assert_allclose(b, np.full(4, 1.5 * y.sum()), rtol=1e-12)
    # inducing points = data points, lengthscale far below their spacing: K_uf = variance * I
    P = np.array([[0.0], [1.0], [2.0]], dtype=np.float32)
    A, b = oracle.sgpr_accumulate(P, P, [5.0, 7.0, 11.0], 2.0, 1e-3)
    assert np.array_equal(A, 4.0 * np.eye(3)) and b.tolist() == [10.0, 14.0, 22.0]


def test_structure_and_the_matvec_oracle(oracle):
    U, X = W.random_case(64, 12, 90, 2)
    g = np.random.Generator(np.random.PCG64(9))
    y = g.standard_normal(90).astype(np.float32)
    v = g.standard_normal(12).astype(np.float32)
    A, b = oracle.sgpr_accumulate(U, X, y, 1.3, 0.8)
    assert np.array_equal(A, A.T)
    assert np.linalg.eigvalsh(A).min() > -1e-12 * np.abs(A).max()
    # b is a kernel matrix-vector product: the other oracle routine must agree
    np.testing.assert_allclose(b, oracle.kmv(U, X, y, 1.3, 0.8), rtol=1e-13)
    # v' A v = |K_fu v|^2, again through the matvec oracle
    Kfu_v = oracle.kmv(X, U, v, 1.3, 0.8)
    assert v.astype(np.float64) @ A @ v.astype(np.float64) == pytest.approx(Kfu_v @ Kfu_v, rel=1e-12)
    # the trace is the squared Frobenius norm of K_uf
    assert np.trace(A) == pytest.approx((dense_kuf(U, X, 1.3, 0.8) ** 2).sum(), rel=1e-13)
    assert np.array_equal(oracle.sgpr_accumulate(U, X, y, 1.3, 0.8, nthreads=1)[0], A)


def test_single_entries_match_the_full_routine(oracle):
    U, X = W.random_case(65, 9, 70, 4)
    y = np.zeros(70, dtype=np.float32)
    A, _ = oracle.sgpr_accumulate(U, X, y, 0.9, 1.4)
    ii, jj = np.array([0, 3, 8, 5]), np.array([0, 7, 8, 2])
    np.testing.assert_allclose(oracle.sgpr_entries(U, X, ii, jj, 0.9, 1.4), A[ii, jj], rtol=1e-14)
