"""CPU-only tests of knn_plan_host_x: data points in host memory, streamed in blocks through
staging buffers that count against the limit (no GPU call)."""
import pytest

import paper_2206_14148_amd as K
import workloads as W

ALIGN = 256


def up(v):
    return (v + ALIGN - 1) // ALIGN * ALIGN


def test_roomy_limit_stages_everything_as_one_block():
    p = K.knn_plan_host_x(1000, 10_000, 16, 10, 64 * W.MB)
    assert (p.n_blocks, p.block_rows) == (1, 10_000)
    assert p.staging_bytes == up(10_000 * 16 * 4)
    # a block's winners (index, list key, fp64 distance) and the running result's fp64 distances
    assert p.block_out_bytes == 2 * up(1000 * 10 * 4) + 2 * up(1000 * 10 * 8)
    assert p.workspace_bytes == p.staging_bytes + p.block_out_bytes + p.inner.workspace_bytes
    assert p.workspace_bytes <= 64 * W.MB
    assert (p.inner.m, p.inner.n, p.inner.k) == (1000, 10_000, 10)


@pytest.mark.parametrize("m,n,d,k,limit", [
    (10_000, 1_000_000, 784, 10, 2 * W.GB),      # the image-like workload: X is 3.1 GB
    (1000, 200_000, 16, 10, 2 * W.MB),
    (5000, 1_000_000, 3, 16, 8 * W.MB),
    (100_000, 10_000_000, 128, 100, 8 * W.GB),
])
def test_tight_limits_cut_the_points_into_blocks(m, n, d, k, limit):
    p = K.knn_plan_host_x(m, n, d, k, limit)
    assert p.n_blocks > 1 and p.n_blocks == -(-n // p.block_rows)
    assert p.block_rows % 128 == 0 and p.block_rows >= k
    assert p.staging_bytes == 2 * up(p.block_rows * d * 4)
    assert p.staging_bytes <= (limit - p.block_out_bytes) / 2 + 2 * ALIGN or p.block_rows <= max(k, 1024)
    assert p.inner_limit_bytes == limit - p.block_out_bytes - p.staging_bytes
    assert p.inner.workspace_bytes <= p.inner_limit_bytes
    assert p.workspace_bytes <= limit
    assert (p.inner.n, p.inner.k) == (p.block_rows, k)


def test_minimum_limit_is_feasible_and_one_byte_less_is_not():
    m, n, d, k = 300, 50_000, 20, 7
    with pytest.raises(K.KnnError) as ei:
        K.knn_plan_host_x(m, n, d, k, 1000)
    assert ei.value.status == K.KNN_ERR_MEM_LIMIT_TOO_SMALL
    need = ei.value.min_limit_bytes
    assert need > 0
    p = K.knn_plan_host_x(m, n, d, k, need)
    assert p.workspace_bytes <= need and p.block_rows == 1024
    with pytest.raises(K.KnnError):
        K.knn_plan_host_x(m, n, d, k, need - 1)


def test_short_last_block_and_k_above_it():
    # n = 2 blocks + 5 points with k = 16: the last block holds fewer than k points
    p = K.knn_plan_host_x(100, 2 * 1024 + 5, 3, 16, K.knn_plan_host_x(100, 2 * 1024 + 5, 3, 16, 10 ** 9).min_limit_bytes)
    assert p.block_rows == 1024 and p.n_blocks == 3
    assert p.workspace_bytes <= p.min_limit_bytes


def test_metrics_empty_and_invalid():
    assert K.knn_plan_host_x(0, 100, 3, 5, 10 ** 6).workspace_bytes == 0
    assert K.knn_plan_host_x(100, 5000, 30, 5, 10 ** 6, "cosine").inner.metric == K.KNN_METRIC_COSINE
    assert K.knn_plan_host_x(100, 5000, 30, 5, 10 ** 6, "l1").inner.path == K.KNN_PATH_L1
    for bad in ((5, 0, 3, 1), (5, 10, 0, 1), (5, 10, 3, 0), (5, 10, 3, 11), (-1, 10, 3, 1)):
        with pytest.raises(K.KnnError) as ei:
            K.knn_plan_host_x(*bad, 10 ** 6)
        assert ei.value.status == K.KNN_ERR_INVALID_ARG


def test_every_reported_minimum_is_feasible_and_plans_stay_under_their_limit():
    import random
    rnd = random.Random(1)
    for _ in range(400):
        m = rnd.choice([1, 5, 100, 300, 1000, 5000])
        n = rnd.choice([1, 7, 100, 1024, 1025, 2053, 5000, 50_000, 10 ** 6])
        d = rnd.choice([1, 3, 8, 9, 16, 100, 784])
        k = min(n, rnd.choice([1, 5, 16, 100, 1024]))
        metric = rnd.choice(["l2", "cosine", "l1"])
        need = K.knn_plan_host_x(m, n, d, k, 10 ** 12, metric).min_limit_bytes
        for limit in (need, 2 * need, 10 * need + 12345, 10 ** 9):
            p = K.knn_plan_host_x(m, n, d, k, limit, metric)
            assert p.workspace_bytes <= limit, (m, n, d, k, metric, limit)
            assert p.block_rows * (p.n_blocks - 1) < n <= p.block_rows * p.n_blocks
