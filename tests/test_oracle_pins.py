"""Pins for the CPU oracle: each test checks it against something other than itself.

The paper (section 5.2) gives only the definition of the result, so the pins are
closed forms, brute force through numpy/torch library routines on tiny inputs,
and invariants of the definition.  A dropped term, a wrong sign, a transposed
operand, a broken tie-break or an off-by-one in the heap fails at least one.
"""
import numpy as np
import pytest
import torch

import workloads as W


def np_bruteforce(Q, X, k):
    """numpy: broadcast differences in fp64, stable argsort (ties -> lower index)."""
    Qd = Q.astype(np.float64)
    Xd = X.astype(np.float64)
    D = ((Qd[:, None, :] - Xd[None, :, :]) ** 2).sum(axis=2)
    order = np.argsort(D, axis=1, kind="stable")[:, :k]
    return order, np.take_along_axis(D, order, axis=1), D


@pytest.mark.parametrize("seed,m,n,d", [(0, 7, 13, 1), (1, 5, 64, 3), (2, 9, 33, 8), (3, 4, 50, 5)])
def test_bruteforce_every_k(oracle, seed, m, n, d):
    Q, X = W.random_case(seed, m, n, d)
    for k in range(1, n + 1):
        ref_idx, ref_dist, D = np_bruteforce(Q, X, k)
        for fn in (oracle.knn, oracle.knn_fullsort):
            idx, dist, nxt = fn(Q, X, k)
            assert np.array_equal(idx, ref_idx), (fn.__name__, k)
            np.testing.assert_allclose(dist, ref_dist, rtol=1e-13, atol=0)
            if k < n:
                ref_next = np.sort(D, axis=1)[:, k]
                np.testing.assert_allclose(nxt, ref_next, rtol=1e-13)
            else:
                assert np.all(np.isinf(nxt))


def test_ties_on_integer_grid_match_stable_argsort(oracle):
    # small integer coordinates: distances are exact integers with many ties
    Q, X = W.random_case(11, 20, 200, 3, kind="grid")
    for k in (1, 2, 7, 50, 200):
        ref_idx, ref_dist, _ = np_bruteforce(Q, X, k)
        for fn in (oracle.knn, oracle.knn_fullsort):
            idx, dist, _ = fn(Q, X, k)
            assert np.array_equal(idx, ref_idx)
            assert np.array_equal(dist, ref_dist)  # integers: exact


def integer_line_expected(i, n, k):
    """d=1, X[j]=j, query i: neighbours i, i-1, i+1, i-2, ... (lower index first on ties)."""
    out = [(0, i)]
    for step in range(1, n):
        for j in (i - step, i + step):
            if 0 <= j < n:
                out.append((step * step, j))
    out = out[:k]
    return [j for _, j in out], [float(dd) for dd, _ in out]


def test_closed_form_integer_line(oracle):
    n = 41
    X = np.arange(n, dtype=np.float32).reshape(n, 1)
    for k in (1, 2, 3, 6, 9, n):
        idx, dist, _ = oracle.knn(X, X, k)
        idx2, dist2, _ = oracle.knn_fullsort(X, X, k)
        for i in range(n):
            e_idx, e_dist = integer_line_expected(i, n, k)
            assert idx[i].tolist() == e_idx
            assert dist[i].tolist() == e_dist
            assert idx2[i].tolist() == e_idx and dist2[i].tolist() == e_dist


def test_closed_form_scaled_orthogonal_basis(oracle):
    # X[j] = a_j e_j  =>  D[i][j] = a_i^2 + a_j^2 (i != j), 0 (i == j)
    n = 12
    a = np.array([3, 1, 4, 1.5, 5, 9, 2, 6, 5.5, 3.5, 8, 7], dtype=np.float32)
    X = np.diag(a).astype(np.float32)
    idx, dist, _ = oracle.knn(X, X, n)
    for i in range(n):
        expect = sorted(((0.0 if j == i else float(a[i]) ** 2 + float(a[j]) ** 2), j) for j in range(n))
        assert idx[i].tolist() == [j for _, j in expect]
        np.testing.assert_allclose(dist[i], [v for v, _ in expect], rtol=1e-15)


def test_duplicated_points_come_in_index_pairs(oracle):
    Q, X = W.random_case(5, 6, 40, 4)
    X2 = np.repeat(X, 2, axis=0)  # rows 2j and 2j+1 are the same point
    k = 11
    idx, dist, _ = oracle.knn(Q, X2, k)
    base_idx, base_dist, _ = oracle.knn(Q, X, (k + 1) // 2)
    for i in range(Q.shape[0]):
        for p in range(k):
            assert idx[i, p] == 2 * base_idx[i, p // 2] + (p % 2)
            assert dist[i, p] == base_dist[i, p // 2]


def test_k1_is_argmin_and_kn_is_stable_argsort(oracle):
    Q, X = W.random_case(6, 30, 300, 6)
    _, _, D = np_bruteforce(Q, X, 1)
    idx, dist, _ = oracle.knn(Q, X, 1)
    assert np.array_equal(idx[:, 0], np.argmin(D, axis=1))
    idx, dist, _ = oracle.knn(Q, X, 300)
    assert np.array_equal(idx, np.argsort(D, axis=1, kind="stable"))


def test_against_torch_cdist(oracle):
    # library routine, different code: cdist in fp64, squared, stable argsort
    w = W.scaled(1, m=200, n=3000)
    Q, X = W.make(w)
    D = torch.cdist(torch.from_numpy(Q).double(), torch.from_numpy(X).double()) ** 2
    order = torch.argsort(D, dim=1, stable=True)[:, : w.k].numpy()
    idx, dist, nxt = oracle.knn(Q, X, w.k)
    assert np.array_equal(idx, order)
    np.testing.assert_allclose(dist, np.take_along_axis(D.numpy(), order, 1), rtol=1e-9)


def test_difference_form_equals_norm_expansion(oracle):
    # section 4.1: sum (x-y)^2 == sum x^2 + y^2 - 2xy, each side in fp64
    Q, X = W.random_case(8, 50, 50, 16)
    for i in range(50):
        a = oracle.sqdist(Q[i], X[i])
        b = oracle.sqdist_expanded(Q[i], X[i])
        assert abs(a - b) <= 1e-12 * max(a, 1.0)
    # and a hand-computed value
    assert oracle.sqdist([1, 2, 3], [4, 6, 3]) == 25.0
    assert oracle.sqdist([0.5], [-0.25]) == 0.5625


def test_rows_sorted_and_self_distance_zero(oracle):
    w = W.scaled(2, n=2000)
    Q, X = W.make(w)
    idx, dist, nxt = oracle.knn(Q, X, w.k)
    assert np.all(np.diff(dist, axis=1) >= 0)
    assert np.all(dist[:, 0] == 0.0)
    assert np.array_equal(idx[:, 0], np.arange(2000))  # no duplicates in continuous data
    assert np.all(nxt >= dist[:, -1])
    assert np.all(dist >= 0)


def test_permuting_points_permutes_indices(oracle):
    Q, X = W.random_case(9, 25, 400, 5)
    perm = np.random.Generator(np.random.PCG64(99)).permutation(400)
    idx, dist, _ = oracle.knn(Q, X, 12)
    idx_p, dist_p, _ = oracle.knn(Q, X[perm], 12)
    # continuous data: no ties, so the mapped indices agree position by position
    assert np.array_equal(perm[idx_p], idx)
    assert np.array_equal(dist_p, dist)


def test_translation_invariance(oracle):
    # shift by a value exactly representable next to the data: results identical
    Q, X = W.random_case(10, 20, 300, 4, kind="grid")
    shift = np.float32(8.0)
    idx, dist, _ = oracle.knn(Q, X, 9)
    idx_s, dist_s, _ = oracle.knn(Q + shift, X + shift, 9)
    assert np.array_equal(idx, idx_s)
    assert np.array_equal(dist, dist_s)


def test_row_subset_matches_full(oracle):
    Q, X = W.random_case(12, 40, 500, 7)
    rows = np.array([3, 3, 39, 0, 17], dtype=np.int64)
    idx, dist, nxt = oracle.knn(Q, X, 5)
    idx_r, dist_r, nxt_r = oracle.knn(Q, X, 5, rows=rows)
    assert np.array_equal(idx_r, idx[rows])
    assert np.array_equal(dist_r, dist[rows])
    assert np.array_equal(nxt_r, nxt[rows])
    # thread count must not change anything
    idx_1, dist_1, _ = oracle.knn(Q, X, 5, nthreads=1)
    assert np.array_equal(idx_1, idx) and np.array_equal(dist_1, dist)


def test_argument_errors(oracle):
    Q, X = W.random_case(13, 3, 10, 2)
    with pytest.raises(ValueError):
        oracle.knn(Q, X, 11)  # k > n
    with pytest.raises(ValueError):
        oracle.knn(Q, X, 0)
    with pytest.raises(ValueError):
        oracle.knn(Q, X[:, :1], 2)  # dimension mismatch
    with pytest.raises(ValueError):
        oracle.knn(Q, X, 2, rows=[5])


# ---------------------------------------------------------------------------------------
# cosine metric (the cosine rows of the paper's kNN table)
# ---------------------------------------------------------------------------------------
def np_cosine_bruteforce(Q, X, k):
    Qd, Xd = Q.astype(np.float64), X.astype(np.float64)
    qn = np.sqrt((Qd * Qd).sum(1))
    xn = np.sqrt((Xd * Xd).sum(1))
    with np.errstate(divide="ignore", invalid="ignore"):
        C = 1.0 - (Qd @ Xd.T) / (qn[:, None] * xn[None, :])
    C = np.where((qn[:, None] == 0) | (xn[None, :] == 0), 1.0, C)
    C = np.maximum(C, 0.0)
    order = np.argsort(C, axis=1, kind="stable")[:, :k]
    return order, np.take_along_axis(C, order, axis=1), C


@pytest.mark.parametrize("seed,m,n,d", [(20, 6, 40, 2), (21, 5, 64, 7), (22, 4, 33, 20)])
def test_cosine_bruteforce_every_k(oracle, seed, m, n, d):
    Q, X = W.random_case(seed, m, n, d)
    X[3] = 0.0  # a zero vector has distance 1 to everything
    for k in (1, 2, 5, n // 2, n):
        ref_idx, ref_dist, C = np_cosine_bruteforce(Q, X, k)
        for fn in (oracle.knn, oracle.knn_fullsort):
            idx, dist, nxt = fn(Q, X, k, metric="cosine")
            # numpy's matmul sums in another order: compare distances, and indices where
            # the neighbouring distances are not within rounding of each other
            np.testing.assert_allclose(dist, ref_dist, rtol=0, atol=1e-12)
            clear = np.ones_like(idx, dtype=bool)
            srt = np.sort(C, axis=1)
            gaps = np.diff(srt[:, : k + 1 if k < n else k], axis=1)
            if k > 1:
                close = gaps[:, : k - 1] < 1e-11
                clear[:, 1:] &= ~close
                clear[:, :-1] &= ~close
            if k < n:
                clear[:, -1] &= gaps[:, k - 1] >= 1e-11
            assert np.array_equal(idx[clear], ref_idx[clear])


def test_cosine_closed_forms(oracle):
    # axis vectors: distance 0 to the same axis (any positive scale), 1 across axes, 2 antipodal
    X = np.array([[2, 0, 0], [0, 3, 0], [0, 0, 0.5], [-4, 0, 0], [5, 0, 0], [0, 0, 0]], dtype=np.float32)
    Q = np.array([[1, 0, 0], [0, 0, 7]], dtype=np.float32)
    idx, dist, _ = oracle.knn(Q, X, 6, metric="cosine")
    assert idx[0].tolist() == [0, 4, 1, 2, 5, 3]
    assert dist[0].tolist() == [0.0, 0.0, 1.0, 1.0, 1.0, 2.0]
    assert idx[1].tolist() == [2, 0, 1, 3, 4, 5]
    assert dist[1].tolist() == [0.0, 1.0, 1.0, 1.0, 1.0, 1.0]
    assert oracle.cosdist([1, 1], [1, 0]) == pytest.approx(1 - 1 / np.sqrt(2), abs=1e-15)
    assert oracle.cosdist([0, 0], [1, 0]) == 1.0


def test_cosine_invariant_under_power_of_two_scaling(oracle):
    # scaling by powers of two is exact in fp32 and fp64, so nothing may change
    Q, X = W.random_case(23, 15, 300, 9)
    idx, dist, nxt = oracle.knn(Q, X, 10, metric="cosine")
    scale = (2.0 ** np.random.Generator(np.random.PCG64(5)).integers(-6, 7, size=(300, 1))).astype(np.float32)
    idx_s, dist_s, nxt_s = oracle.knn(Q * np.float32(8.0), X * scale, 10, metric="cosine")
    assert np.array_equal(idx, idx_s) and np.array_equal(dist, dist_s) and np.array_equal(nxt, nxt_s)


def test_cosine_matches_euclidean_on_unit_vectors(oracle):
    # |q - x|^2 = 2 - 2 cos for unit vectors: same neighbours as the Euclidean oracle
    Q, X = W.random_case(24, 30, 500, 12)
    Qn = (Q / np.linalg.norm(Q.astype(np.float64), axis=1, keepdims=True)).astype(np.float32)
    Xn = (X / np.linalg.norm(X.astype(np.float64), axis=1, keepdims=True)).astype(np.float32)
    c_idx, c_dist, _ = oracle.knn(Qn, Xn, 8, metric="cosine")
    e_idx, e_dist, _ = oracle.knn(Qn, Xn, 8, metric="l2")
    assert np.array_equal(c_idx, e_idx)  # continuous data: no ties at this resolution
    np.testing.assert_allclose(2.0 * c_dist, e_dist, rtol=0, atol=1e-6)  # fp32 normalisation error
    assert np.all(np.diff(c_dist, axis=1) >= 0)


# ---------------------------------------------------------------------------------------
# L1 metric (the L1 rows of the paper's kNN table)
# ---------------------------------------------------------------------------------------
@pytest.mark.parametrize("seed,m,n,d", [(30, 6, 40, 1), (31, 5, 64, 3), (32, 4, 33, 20)])
def test_l1_bruteforce_every_k(oracle, seed, m, n, d):
    Q, X = W.random_case(seed, m, n, d, kind="grid")  # integers: every sum is exact
    M = np.abs(Q.astype(np.float64)[:, None, :] - X.astype(np.float64)[None, :, :]).sum(axis=2)
    for k in range(1, n + 1):
        order = np.argsort(M, axis=1, kind="stable")[:, :k]
        for fn in (oracle.knn, oracle.knn_fullsort):
            idx, dist, nxt = fn(Q, X, k, metric="l1")
            assert np.array_equal(idx, order)
            assert np.array_equal(dist, np.take_along_axis(M, order, axis=1))
            if k < n:
                assert np.array_equal(nxt, np.sort(M, axis=1)[:, k])


def test_l1_integer_line_and_scipy(oracle):
    from scipy.spatial.distance import cdist
    n = 31
    X = np.arange(n, dtype=np.float32).reshape(n, 1)
    idx, dist, _ = oracle.knn(X, X, 5, metric="l1")
    for i in range(n):
        want = sorted((abs(i - j), j) for j in range(n))[:5]
        assert idx[i].tolist() == [j for _, j in want]
        assert dist[i].tolist() == [float(v) for v, _ in want]
    Q, X = W.random_case(33, 40, 700, 9)
    M = cdist(Q.astype(np.float64), X.astype(np.float64), metric="cityblock")
    order = np.argsort(M, axis=1, kind="stable")[:, :12]
    idx, dist, _ = oracle.knn(Q, X, 12, metric="l1")
    assert np.array_equal(idx, order)
    np.testing.assert_allclose(dist, np.take_along_axis(M, order, 1), rtol=1e-13)
    assert oracle.l1dist([1, -2, 3], [4, 6, 3]) == 11.0


def test_l1_norm_inequalities(oracle):
    # ||v||_2 <= ||v||_1 <= sqrt(d) ||v||_2 for every pair
    Q, X = W.random_case(34, 10, 50, 7)
    for i in range(10):
        for j in range(50):
            l1 = oracle.l1dist(Q[i], X[j])
            l2 = np.sqrt(oracle.sqdist(Q[i], X[j]))
            assert l2 <= l1 * (1 + 1e-12) and l1 <= np.sqrt(7) * l2 * (1 + 1e-12)
