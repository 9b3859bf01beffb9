"""CPU-only tests of kmv_plan (include/kmv.h): host arithmetic, no GPU call."""
import pytest

import paper_2206_14148_amd as K
import workloads as W


def test_low_d_needs_no_workspace_when_rows_fill_the_gpu():
    # the appendix case of the paper: 1-D inputs of size 1e6, 1GB threshold
    p = K.kmv_plan(10 ** 6, 10 ** 6, 1, W.GB)
    assert (p.path, p.n_splits, p.workspace_bytes, p.min_limit_bytes) == (K.KMV_PATH_LOWD, 1, 0, 0)
    assert p.tile_rows == 256
    assert K.kmv_plan(10 ** 6, 10 ** 6, 1, 0).workspace_bytes == 0  # even a zero limit runs


def test_matrix_core_path_keeps_scaled_norms():
    p = K.kmv_plan(200_000, 200_000, 32, W.GB)
    assert p.path == K.KMV_PATH_MFMA and p.tile_rows == 128
    assert p.norms_bytes >= 4 * 200_000 and p.norms_bytes % 256 == 0
    assert p.min_limit_bytes == p.norms_bytes
    with pytest.raises(K.KnnError) as ei:
        K.kmv_plan(200_000, 200_000, 32, p.norms_bytes - 1)
    assert ei.value.status == K.KNN_ERR_MEM_LIMIT_TOO_SMALL
    assert K.kmv_plan(200_000, 200_000, 32, p.norms_bytes).n_splits == 1


def test_matrix_core_path_cuts_ranges_to_even_out_its_rounds():
    # 1563 workgroups of equal length on 3 x 256 places would run three rounds for two rounds'
    # worth of work; ranges shorten the rounds when their partial sums fit under the limit
    n = m = 200_000
    p = K.kmv_plan(n, m, 32, W.GB)
    assert p.n_splits in (2, 3, 4, 6, 8) and m // p.n_splits >= 2048
    assert p.partials_bytes == (8 * n * p.n_splits + 255) // 256 * 256
    assert p.workspace_bytes == p.norms_bytes + p.partials_bytes <= W.GB
    # no room for partial sums: one range, the sums go straight to y
    q = K.kmv_plan(n, m, 32, p.norms_bytes + 8 * n)
    assert (q.n_splits, q.partials_bytes) == (1, 0)
    # a launch that fills whole rounds anyway stays at one range
    r = K.kmv_plan(2 * 768 * 128, m, 32, W.GB)
    assert r.n_splits == 1


@pytest.mark.parametrize("d", [2, 16])
def test_ranges_grow_only_while_they_fit(d):
    n, m = 300, 10 ** 6
    prev = None
    for limit in (0 if d <= 8 else 4 * 10 ** 6 + 256, 5 * 10 ** 6, 64 * 10 ** 6, 10 ** 9):
        p = K.kmv_plan(n, m, d, limit)
        assert p.workspace_bytes <= limit
        assert p.workspace_bytes == p.norms_bytes + p.partials_bytes
        assert p.n_splits in (1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64)
        assert (p.partials_bytes == 0) == (p.n_splits == 1)
        if p.n_splits > 1:
            assert p.partials_bytes >= 8 * n * p.n_splits
            assert m // p.n_splits >= 2048
        if prev is not None:
            assert p.n_splits >= prev.n_splits  # a larger limit never gives fewer ranges
        prev = p
    assert prev.n_splits == 64


def test_empty_and_invalid_shapes():
    assert K.kmv_plan(0, 100, 3, 10 ** 6).workspace_bytes == 0
    assert K.kmv_plan(100, 0, 30, 10 ** 6).workspace_bytes == 0
    for bad in ((-1, 5, 3, 10), (5, -1, 3, 10), (5, 5, 0, 10), (5, 5, 3, -1)):
        with pytest.raises(K.KnnError) as ei:
            K.kmv_plan(*bad)
        assert ei.value.status == K.KNN_ERR_INVALID_ARG
    with pytest.raises(K.KnnError) as ei:
        K.kmv_plan(2 ** 31, 5, 3, 10 ** 9)
    assert ei.value.status == K.KNN_ERR_UNSUPPORTED
