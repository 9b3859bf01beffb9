"""GPU parity tests of knn_search_host_x: data points in HOST memory, streamed block by block
through staging buffers inside the workspace, against the CPU oracle and against the resident
search (paper section 5.1: data sets beyond the device's capacity once everything the library
keeps is bounded)."""
import sys

import numpy as np
import pytest

import workloads as W
from parity import check

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def K():
    import paper_2206_14148_amd as K
    assert torch.cuda.is_available(), "these tests need the GPU"
    K.load()
    return K


def run_both(K, oracle, Q, X, k, limit, metric="l2", pinned=True, min_blocks=2):
    plan = K.knn_plan_host_x(Q.shape[0], X.shape[0], X.shape[1], k, limit, metric)
    assert plan.n_blocks >= min_blocks and plan.workspace_bytes <= limit
    say(f"   host plan: {plan.n_blocks} blocks of {plan.block_rows}, workspace {plan.workspace_bytes} B")
    Qd = torch.from_numpy(Q).cuda()
    Xh = torch.from_numpy(X).pin_memory() if pinned else X
    guard = 4096
    buf = torch.full((plan.workspace_bytes + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    idx, dist = K.knn_search_host_x(Qd, Xh, k, limit, workspace=buf[:plan.workspace_bytes],
                                    metric=metric)
    torch.cuda.synchronize()
    assert (buf[plan.workspace_bytes:] == 0xA5).all()
    idx, dist = idx.cpu().numpy(), dist.cpu().numpy()
    o_idx, o_dist, o_next = oracle.knn(Q, X, k, metric=metric)
    stats = check(idx, dist, o_idx, o_dist, o_next, X.shape[0])
    say("   parity", stats)
    # the resident search on a device copy gives the same bits on every row: the blocks are folded
    # in the order of the list keys, the order in which a resident search merges its point ranges,
    # and the final order comes from the fp64 distances
    r_idx, r_dist = K.knn_search(Qd, torch.from_numpy(X).cuda(), k, 64 * W.MB, metric=metric)
    torch.cuda.synchronize()
    r_idx, r_dist = r_idx.cpu().numpy(), r_dist.cpu().numpy()
    assert np.array_equal(idx, r_idx) and np.array_equal(dist.view(np.int32), r_dist.view(np.int32))
    return idx, dist


# (seed, m, n, d, k, kind, limit, metric)
CASES = [
    (0, 500, 20_000, 16, 10, "normal", 1 * W.MB, "l2"),       # matrix-core path per block
    (1, 700, 30_000, 3, 16, "uniform", 400_000, "l2"),        # packed low-d path per block
    (2, 300, 2 * 1024 + 5, 3, 16, "normal", None, "l2"),      # last block shorter than k
    (3, 257, 9_000, 8, 5, "normal", 500_000, "l2"),           # vector-ALU path per block
    (4, 200, 12_345, 40, 33, "normal", 2 * W.MB, "cosine"),
    (5, 200, 12_345, 24, 8, "normal", 1 * W.MB, "l1"),
    (6, 64, 8_000, 2, 4, "grid", 60_000, "l2"),               # many exact ties across blocks
    (7, 100, 5_000, 300, 3, "normal", 4 * W.MB, "l2"),        # streamed-query kernel per block
    (8, 2100, 400_000, 32, 10, "normal", 60 * W.MB, "l2"),    # packed path per block, thresholds carried on
    (9, 2100, 300_000, 272, 10, "normal", 300 * W.MB, "l2"),  # wide path per block (5 blocks), the same
    (10, 2100, 400_000, 32, 10, "normal", 70 * W.MB, "cosine"),  # cosine on the packed path per block, the same
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "s%d_m%d_n%d_d%d_k%d_%s" % (c[0], c[1], c[2], c[3], c[4], c[7]))
def test_blocks_from_pinned_host_memory(K, oracle, case):
    seed, m, n, d, k, kind, limit, metric = case
    say("case", case)
    Q, X = W.random_case(200 + seed, m, n, d, kind)
    if limit is None:
        limit = K.knn_plan_host_x(m, n, d, k, 10 ** 9, metric).min_limit_bytes
        with pytest.raises(K.KnnError):
            K.knn_plan_host_x(m, n, d, k, limit - 1, metric)
    if kind == "grid":
        # ties everywhere: compare with the oracle through the parity rule only
        plan = K.knn_plan_host_x(m, n, d, k, limit, metric)
        assert plan.n_blocks >= 2
        idx, dist = K.knn_search_host_x(torch.from_numpy(Q).cuda(), torch.from_numpy(X).pin_memory(),
                                        k, limit, metric=metric)
        torch.cuda.synchronize()
        o_idx, o_dist, o_next = oracle.knn(Q, X, k, metric=metric)
        idx, dist = idx.cpu().numpy(), dist.cpu().numpy()
        say("   parity", check(idx, dist, o_idx, o_dist, o_next, n))
        # on equal distances the lower index wins, across blocks too
        assert np.array_equal(idx, o_idx.astype(np.int32))
        return
    run_both(K, oracle, Q, X, k, limit, metric)


def test_pageable_numpy_array_and_strided_host_rows(K, oracle):
    Q, X = W.random_case(220, 300, 15_000, 12, "normal")
    run_both(K, oracle, Q, X, 9, 1 * W.MB, pinned=False)
    wide = torch.full((15_000, 20), 77.0).pin_memory()
    wide[:, :12] = torch.from_numpy(X)
    Qd = torch.from_numpy(Q).cuda()
    i1, d1 = K.knn_search_host_x(Qd, wide[:, :12], 9, 1 * W.MB)
    i2, d2 = K.knn_search_host_x(Qd, X, 9, 1 * W.MB)
    torch.cuda.synchronize()
    assert torch.equal(i1, i2) and torch.equal(d1, d2)


def test_one_block_and_back_to_back_calls_share_a_workspace(K, oracle):
    Q, X = W.random_case(221, 400, 6_000, 16, "normal")
    run_both(K, oracle, Q, X, 10, 64 * W.MB, min_blocks=1)   # everything staged at once
    # two calls in a row on one stream and one workspace, the second on fewer points
    limit = 400_000
    plan = K.knn_plan_host_x(400, 6_000, 16, 10, limit)
    assert plan.n_blocks >= 2
    plan_b = K.knn_plan_host_x(400, 2_500, 16, 10, limit)
    ws = torch.empty(max(plan.workspace_bytes, plan_b.workspace_bytes), dtype=torch.uint8,
                     device="cuda")
    Qd = torch.from_numpy(Q).cuda()
    Xh = torch.from_numpy(X).pin_memory()
    a = K.knn_search_host_x(Qd, Xh, 10, limit, workspace=ws)
    b = K.knn_search_host_x(Qd, Xh[:2500], 10, limit, workspace=ws)
    torch.cuda.synchronize()
    for (idx, dist), n in ((a, 6_000), (b, 2_500)):
        o_idx, o_dist, o_next = oracle.knn(Q, X[:n], 10)
        check(idx.cpu().numpy(), dist.cpu().numpy(), o_idx, o_dist, o_next, n)


def test_errors(K):
    Q, X = W.random_case(222, 50, 5_000, 16, "normal")
    Qd = torch.from_numpy(Q).cuda()
    with pytest.raises(K.KnnError) as ei:
        K.knn_search_host_x(Qd, X, 10, 1000)
    assert ei.value.status == K.KNN_ERR_MEM_LIMIT_TOO_SMALL
    with pytest.raises(K.KnnError) as ei:
        K.knn_search_host_x(Qd, X[:, :8].copy(), 10, W.MB)   # d mismatch
    assert ei.value.status == K.KNN_ERR_INVALID_ARG
    with pytest.raises(K.KnnError) as ei:
        K.knn_search_host_x(Qd, torch.from_numpy(X).cuda(), 10, W.MB)  # X must be in host memory
    assert ei.value.status == K.KNN_ERR_INVALID_ARG
    plan = K.knn_plan_host_x(50, 5_000, 16, 10, W.MB)
    small = torch.empty(plan.workspace_bytes - 256, dtype=torch.uint8, device="cuda")
    with pytest.raises(K.KnnError) as ei:
        K.knn_search_host_x(Qd, X, 10, W.MB, workspace=small)
    assert ei.value.status == K.KNN_ERR_WORKSPACE_TOO_SMALL


def test_image_like_workload_under_its_limit(K, oracle):
    # config 3's shape with fewer points: X (627 MB) stays in host memory, the limit is 256 MB
    w = W.scaled(3, m=2_000, n=200_000)
    Q, X = W.make(w)
    limit = 256 * W.MB
    plan = K.knn_plan_host_x(w.m, w.n, w.d, w.k, limit)
    say(f"   host plan: {plan.n_blocks} blocks of {plan.block_rows}, workspace {plan.workspace_bytes} B")
    assert plan.n_blocks >= 4 and plan.workspace_bytes <= limit < X.nbytes
    idx, dist = K.knn_search_host_x(torch.from_numpy(Q).cuda(), torch.from_numpy(X).pin_memory(),
                                    w.k, limit)
    torch.cuda.synchronize()
    rows = W.sample_rows(w, 200)
    o_idx, o_dist, o_next = oracle.knn(Q, X, w.k, rows=rows)
    say("   parity", check(idx.cpu().numpy()[rows], dist.cpu().numpy()[rows], o_idx, o_dist, o_next, w.n))


@pytest.mark.parametrize("order", ["nearest_first", "nearest_last"])
@pytest.mark.parametrize("metric", ["l2", "cosine"])
def test_thresholds_carried_from_block_to_block(K, oracle, order, metric):
    # d > 8: from the second block on, the lists start under the thresholds the earlier blocks
    # reached.  With the nearest points first, the later blocks find nothing below them and
    # hand back empty lists (fillers only); with the nearest points last, every block improves
    # on the one before.  Either way the result is that of the resident search.
    g = np.random.Generator(np.random.PCG64(W.SEED_BASE + 15_000_000))
    n, m, d, k = 24_000, 260, 24, 12
    X = g.standard_normal((n, d)).astype(np.float32)
    Q = (0.05 * g.standard_normal((m, d))).astype(np.float32) + np.float32(0.3)
    centre = Q.mean(axis=0, dtype=np.float64)
    Xc = X.astype(np.float64)
    if metric == "cosine":
        score = -(Xc @ centre) / np.linalg.norm(Xc, axis=1)
    else:
        score = ((Xc - centre) ** 2).sum(axis=1)
    perm = np.argsort(score if order == "nearest_first" else -score)
    X = np.ascontiguousarray(X[perm])
    limit = K.knn_plan_host_x(m, n, d, k, 10 ** 9, metric).min_limit_bytes + 600_000
    plan = K.knn_plan_host_x(m, n, d, k, limit, metric)
    assert plan.n_blocks >= 4 and plan.inner.q_chunks == 1 and plan.inner.path == K.KNN_PATH_MFMA_SPLIT
    run_both(K, oracle, Q, X, k, limit, metric)
