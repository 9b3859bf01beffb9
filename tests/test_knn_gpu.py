"""GPU parity tests: the HIP path, called through the C ABI, against the CPU oracle.

Sizes are small enough for the oracle to finish in seconds yet span several tiles, several
point ranges and ragged tails on both kernel families (d <= 8 and d > 8).
"""
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


def run_gpu(K, Q, X, k, limit, q_is_x=False, metric="l2"):
    Xd = torch.from_numpy(X).cuda()
    Qd = Xd if q_is_x else torch.from_numpy(Q).cuda()
    idx, dist = K.knn_search(Qd, Xd, k, limit, metric=metric)
    torch.cuda.synchronize()
    return idx.cpu().numpy(), dist.cpu().numpy()


def parity(K, oracle, Q, X, k, limit=64 * W.MB, q_is_x=False, rows=None, metric="l2"):
    idx, dist = run_gpu(K, Q, X, k, limit, q_is_x, metric)
    o_idx, o_dist, o_next = oracle.knn(Q, X, k, rows=rows, metric=metric)
    if rows is not None:
        idx, dist = idx[rows], dist[rows]
    sel = np.arange(Q.shape[0]) if rows is None else rows

    def pair_dist(cols):
        qi = np.repeat(sel, cols.shape[1])
        return oracle.sqdist_pairs(Q, X, qi, cols.ravel(), metric).reshape(cols.shape)

    stats = check(idx, dist, o_idx, o_dist, o_next, X.shape[0],
                  pair_dist if Q.shape[0] * k <= 20000 else None)
    say("   parity", stats)
    return stats, idx, dist


# (seed, m, n, d, k, kind)
SMALL = [
    (0, 1, 1, 1, 1, "normal"),          # smallest possible call
    (1, 3, 5, 3, 5, "normal"),          # k == n on the low-d path
    (2, 300, 5000, 3, 16, "uniform"),   # low-d, two point ranges, ragged query tile
    (3, 257, 1003, 8, 7, "normal"),     # low-d widest d, one query past a tile
    (4, 70, 9001, 2, 33, "uniform"),    # low-d, k > 32, many ranges
    (5, 5, 129, 9, 129, "normal"),      # matrix path, k == n, one point past a tile
    (6, 64, 300, 17, 1, "normal"),      # matrix path, k == 1, d not a multiple of 4
    (7, 130, 4100, 100, 100, "normal"),  # matrix path, k = 100, ragged everything
    (8, 1000, 10000, 16, 10, "normal"),  # shape of config 1
    (9, 200, 3000, 784, 10, "sparse0"),  # d = 784 as in config 3 (small n)
    (10, 33, 20000, 128, 64, "normal"),  # many point ranges, k = 64
    (11, 129, 2500, 10, 12, "normal"),   # unaligned rows (d = 10)
    # every chunk count of the register-resident-query kernel (d <= 256), aligned and not
    (12, 140, 2300, 40, 9, "normal"),    # 3 chunks -> 4
    (13, 140, 2300, 90, 9, "normal"),    # 6 chunks, d % 4 != 0
    (14, 140, 2300, 128, 9, "normal"),   # 8 chunks
    (15, 140, 2300, 150, 9, "normal"),   # 10 chunks -> 12, d % 4 != 0
    (16, 140, 2300, 200, 9, "normal"),   # 13 chunks -> 16
    (17, 140, 2300, 256, 9, "normal"),   # 16 chunks
    (18, 140, 2300, 257, 9, "normal"),   # first d of the streamed-query kernel, unaligned
    (19, 140, 2300, 272, 9, "normal"),   # streamed-query kernel, aligned
    (20, 70, 300, 12, 5, "normal"),      # one chunk (d <= 16), an odd number of point tiles
    (21, 70, 128, 16, 5, "normal"),      # one chunk, a single tile
]


@pytest.mark.parametrize("seed,m,n,d,k,kind", SMALL)
def test_parity_small(K, oracle, seed, m, n, d, k, kind):
    say(f"\ncase seed={seed} m={m} n={n} d={d} k={k} kind={kind}")
    if kind == "sparse0":
        Q, X = W.make(W.scaled(3, m=m, n=n))
    else:
        Q, X = W.random_case(100 + seed, m, n, d, kind)
    stats, _, _ = parity(K, oracle, Q, X, k)
    assert stats["strict_rows"] >= 0.98 * stats["rows"]


@pytest.mark.parametrize("d", [1])
def test_integer_line_closed_form(K, d):
    # X[j] = j on a line: neighbours of i are i, i-1, i+1, i-2, ... with exact integer
    # distances and every +-step tie resolved to the lower index
    n = 700
    X = np.arange(n, dtype=np.float32).reshape(n, 1)
    k = 9
    idx, dist = run_gpu(K, X, X, k, 64 * W.MB, q_is_x=True)
    for i in (0, 1, 3, 4, 5, 350, 695, 698, 699):
        want = [(0, i)]
        for step in range(1, n):
            for j in (i - step, i + step):
                if 0 <= j < n:
                    want.append((step * step, j))
        want = want[:k]
        assert idx[i].tolist() == [j for _, j in want], i
        assert dist[i].tolist() == [float(v) for v, _ in want], i


@pytest.mark.parametrize("d,n", [(3, 3000), (16, 3000), (40, 2600)])
def test_duplicated_points_keep_index_order(K, oracle, d, n):
    # every point twice: rows 2j and 2j+1 are identical, so results come in (2j, 2j+1) pairs
    Q, X = W.random_case(200 + d, 150, n // 2, d)
    X2 = np.repeat(X, 2, axis=0)
    k = 11
    idx, dist = run_gpu(K, Q, X2, k, 64 * W.MB)
    o_idx, o_dist, _ = oracle.knn(Q, X2, k)
    assert np.array_equal(idx, o_idx)
    pairs = idx[:, : k - 1].reshape(idx.shape[0], -1, 2)
    assert np.all(pairs[:, :, 0] % 2 == 0) and np.all(pairs[:, :, 1] == pairs[:, :, 0] + 1)
    assert np.all(idx[:, k - 1] % 2 == 0)  # the odd one out is the lower twin
    np.testing.assert_allclose(dist, o_dist, rtol=1e-6, atol=1e-7)


@pytest.mark.parametrize("d", [3, 12])
def test_exact_ties_on_integer_grid(K, oracle, d):
    # small integer coordinates: all arithmetic is exact in fp32 and fp64, ties are massive,
    # so the result is unique under the (distance, index) order and must match bit for bit
    Q, X = W.random_case(300 + d, 260, 6000, d, kind="grid")
    for k in (1, 8, 50):
        idx, dist = run_gpu(K, Q, X, k, 64 * W.MB)
        o_idx, o_dist, _ = oracle.knn(Q, X, k)
        assert np.array_equal(idx, o_idx), (d, k)
        assert np.array_equal(dist.astype(np.float64), o_dist), (d, k)


@pytest.mark.parametrize("d", [1, 2, 3])
def test_low_d_paths_agree_and_survive_data_far_from_the_origin(K, oracle, d):
    # the bf16 matrix-core filter (roomy limit), the fp32 one (room for 16 but not 32 bytes per
    # point) and the vector kernel (tight limit) must give the same bits; an offset of 50 makes
    # the expansion's rounding far larger than the neighbour distances, so the fp32 filter
    # passes nearly everything to the exact test (the bf16 one moves the data first)
    Q, X = W.random_case(1000 + d, 700, 9000, d, kind="uniform")
    for shift in (0.0, 50.0):
        Qs, Xs = (Q + np.float32(shift)), (X + np.float32(shift))
        k = 12
        lo = K.knn_plan(700, 9000, d, k, 1 << 40).min_limit_bytes
        assert K.knn_plan(700, 9000, d, k, lo + 40_000).path == K.KNN_PATH_LOWD
        assert K.knn_plan(700, 9000, d, k, 250_000).path == K.KNN_PATH_LOWD_MFMA
        assert K.knn_plan(700, 9000, d, k, 64 * W.MB).path == K.KNN_PATH_LOWD_BF16
        a_idx, a_dist = run_gpu(K, Qs, Xs, k, lo + 40_000)
        c_idx, c_dist = run_gpu(K, Qs, Xs, k, 250_000)
        b_idx, b_dist = run_gpu(K, Qs, Xs, k, 64 * W.MB)
        assert np.array_equal(a_idx, b_idx) and np.array_equal(a_dist, b_dist)
        assert np.array_equal(a_idx, c_idx) and np.array_equal(a_dist, c_dist)
        o_idx, o_dist, o_next = oracle.knn(Qs, Xs, k)
        say("   shift", shift, check(b_idx, b_dist, o_idx, o_dist, o_next, 9000))


@pytest.mark.parametrize("d", [4, 5, 6, 7, 8])
def test_bf16_filter_and_vector_kernel_agree_for_d_4_to_8(K, oracle, d):
    # one MFMA of 16 K slots up to d = 4, two above; same exact keys as the vector kernel
    Q, X = W.random_case(1100 + d, 520, 9000, d, kind="uniform")
    for shift in (0.0, 50.0):
        Qs, Xs = (Q + np.float32(shift)), (X + np.float32(shift))
        k = 12
        lo = K.knn_plan(520, 9000, d, k, 1 << 40).min_limit_bytes
        assert K.knn_plan(520, 9000, d, k, lo + 40_000).path == K.KNN_PATH_LOWD
        assert K.knn_plan(520, 9000, d, k, 64 * W.MB).path == K.KNN_PATH_LOWD_BF16
        a_idx, a_dist = run_gpu(K, Qs, Xs, k, lo + 40_000)
        b_idx, b_dist = run_gpu(K, Qs, Xs, k, 64 * W.MB)
        assert np.array_equal(a_idx, b_idx) and np.array_equal(a_dist, b_dist)
        o_idx, o_dist, o_next = oracle.knn(Qs, Xs, k)
        say("   d", d, "shift", shift, check(b_idx, b_dist, o_idx, o_dist, o_next, 9000))


def test_self_distance_zero_when_queries_are_the_points(K, oracle):
    w = W.scaled(2, n=30000)
    Q, X = W.make(w)
    stats, idx, dist = parity(K, oracle, Q, X, w.k, q_is_x=True,
                              rows=W.sample_rows(w, 600))
    idx_all, dist_all = run_gpu(K, X, X, w.k, w.mem_limit, q_is_x=True)
    assert np.array_equal(idx_all[:, 0], np.arange(30000))
    assert np.all(dist_all[:, 0] == 0.0)
    assert stats["strict_rows"] == stats["rows"]


@pytest.mark.parametrize("m,n,d,k", [(3000, 9000, 3, 10), (700, 12000, 32, 20)])
def test_result_does_not_depend_on_the_memory_limit(K, m, n, d, k):
    # same answer, bit for bit, whatever the limit forces the plan to be (chunks, ranges)
    Q, X = W.random_case(400 + d, m, n, d)
    lo = K.knn_plan(m, n, d, k, 1 << 40).min_limit_bytes
    limits = [lo, lo + 70_000, lo + 500_000, 64 * W.MB, 8 * W.GB]
    plans = [K.knn_plan(m, n, d, k, lim) for lim in limits]
    say("   plans", [(p.q_chunks, p.n_splits, p.workspace_bytes) for p in plans])
    assert len({(p.q_chunks, p.n_splits) for p in plans}) >= 3  # the plans really differ
    ref = None
    for lim in limits:
        idx, dist = run_gpu(K, Q, X, k, lim)
        if ref is None:
            ref = (idx, dist)
        else:
            assert np.array_equal(idx, ref[0]) and np.array_equal(dist, ref[1]), lim


@pytest.mark.parametrize("m,n,d,k", [(1500, 8000, 3, 16), (400, 9000, 24, 10)])
def test_workspace_bound_is_respected(K, m, n, d, k):
    # guard bytes right behind the planned workspace must survive the call
    Q, X = W.random_case(500 + d, m, n, d)
    Qd, Xd = torch.from_numpy(Q).cuda(), torch.from_numpy(X).cuda()
    limit = K.knn_plan(m, n, d, k, 1 << 40).min_limit_bytes + 100_000
    plan = K.knn_plan(m, n, d, k, limit)
    assert plan.workspace_bytes <= limit
    guard = 4096
    ws = torch.full((plan.workspace_bytes + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    idx, dist = K.knn_search(Qd, Xd, k, limit, workspace=ws[: plan.workspace_bytes])
    torch.cuda.synchronize()
    assert bool((ws[plan.workspace_bytes:] == 0xA5).all())
    last_plan, peak = K.knn_last_stats()
    assert peak == plan.workspace_bytes <= limit and last_plan.q_chunks == plan.q_chunks
    ref_idx, ref_dist = run_gpu(K, Q, X, k, 8 * W.GB)
    assert np.array_equal(idx.cpu().numpy(), ref_idx)
    assert np.array_equal(dist.cpu().numpy(), ref_dist)


def test_row_strides_larger_than_d(K, oracle):
    for d, ld in ((3, 5), (20, 24), (20, 23)):
        Q, X = W.random_case(600 + ld, 90, 2100, d)
        Xp = torch.zeros((2100, ld), device="cuda")
        Qp = torch.zeros((90, ld), device="cuda")
        Xp[:, :d] = torch.from_numpy(X).cuda()
        Qp[:, :d] = torch.from_numpy(Q).cuda()
        Xp[:, d:] = 1e30  # padding must never be read as data
        idx, dist = K.knn_search(Qp[:, :d], Xp[:, :d], 6, 64 * W.MB)
        torch.cuda.synchronize()
        o_idx, o_dist, o_next = oracle.knn(Q, X, 6)
        check(idx.cpu().numpy(), dist.cpu().numpy(), o_idx, o_dist, o_next, 2100)


def test_errors_leave_outputs_untouched(K):
    Q, X = W.random_case(700, 10, 50, 4)
    Qd, Xd = torch.from_numpy(Q).cuda(), torch.from_numpy(X).cuda()
    idx = torch.full((10, 3), -7, dtype=torch.int32, device="cuda")
    dist = torch.full((10, 3), -7.0, device="cuda")
    with pytest.raises(K.KnnError) as ei:
        K.knn_search(Qd, Xd, 3, 100, out=(idx, dist))  # limit far too small
    assert ei.value.status == K.KNN_ERR_MEM_LIMIT_TOO_SMALL
    with pytest.raises(K.KnnError) as ei:
        K.knn_search(Qd, Xd, 51, 64 * W.MB)  # k > n
    assert ei.value.status == K.KNN_ERR_INVALID_ARG
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    with pytest.raises(K.KnnError) as ei:
        K.knn_search(Qd, Xd, 3, 64 * W.MB, workspace=ws[:8], out=(idx, dist))
    assert ei.value.status == K.KNN_ERR_WORKSPACE_TOO_SMALL
    with pytest.raises(K.KnnError):
        K.knn_search(Qd.cpu(), Xd.cpu(), 3, 64 * W.MB)  # no CPU path
    torch.cuda.synchronize()
    assert bool((idx == -7).all()) and bool((dist == -7.0).all())
    e_idx, e_dist = K.knn_search(Qd[:0], Xd, 3, 64 * W.MB)  # m == 0
    assert e_idx.shape == (0, 3) and e_dist.shape == (0, 3)


def test_two_runs_are_bit_identical_and_streams_are_honoured(K):
    Q, X = W.random_case(800, 500, 7000, 48)
    Qd, Xd = torch.from_numpy(Q).cuda(), torch.from_numpy(X).cuda()
    a_idx, a_dist = K.knn_search(Qd, Xd, 25, 64 * W.MB)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        b_idx, b_dist = K.knn_search(Qd, Xd, 25, 64 * W.MB)
    side.synchronize()
    torch.cuda.synchronize()
    assert torch.equal(a_idx, b_idx) and torch.equal(a_dist, b_dist)


def test_large_k(K, oracle):
    Q, X = W.random_case(900, 40, 3000, 5)
    parity(K, oracle, Q, X, 1000)
    Q, X = W.random_case(901, 40, 3000, 20)
    parity(K, oracle, Q, X, 1024)


# ---------------------------------------------------------------------------------------
# cosine metric
# ---------------------------------------------------------------------------------------
COSINE = [
    (0, 50, 900, 3, 7),       # low d still runs on the matrix-core path
    (1, 130, 4100, 20, 16),   # unaligned-free small d, several ranges
    (2, 140, 2300, 100, 10),  # the table's d = 100
    (3, 140, 2300, 150, 9),   # d % 4 != 0
    (4, 90, 2300, 300, 12),   # streamed-query kernel
    (5, 64, 300, 50, 300),    # k == n
]


@pytest.mark.parametrize("seed,m,n,d,k", COSINE)
def test_cosine_parity_small(K, oracle, seed, m, n, d, k):
    say(f"\ncosine case seed={seed} m={m} n={n} d={d} k={k}")
    Q, X = W.random_case(1100 + seed, m, n, d)
    X[5] = 0.0  # a zero point: distance 1 to everything
    Q[2] = 0.0  # a zero query: distance 1 to everything, neighbours are the lowest indices
    stats, idx, dist = parity(K, oracle, Q, X, k, metric="cosine")
    assert stats["strict_rows"] >= 0.97 * stats["rows"]
    assert idx[2].tolist() == list(range(k)) and np.all(dist[2] == 1.0)


def test_cosine_near_parallel_neighbours(K, oracle):
    # Every query has a cloud of points in almost its own direction: the neighbours' cosine
    # distances are around 5e-3 and a few 1e-5 apart, with lengths that vary by a factor of
    # eight.  The selection keys are fp32 values -2 (q.x) / |x| (absolute error about 1e-7 |q|);
    # the parity rule asks for the oracle's index set wherever the k-th gap exceeds 1e-4 relative,
    # here about 5e-7 absolute - a few times the key error.  The returned distances are fp64
    # re-evaluations and must agree everywhere.
    say("\ncosine near-parallel case")
    rng = np.random.default_rng(77001)
    m, d, per, k = 60, 48, 400, 12
    Q = rng.standard_normal((m, d)).astype(np.float32)
    near = Q[np.repeat(np.arange(m), per)].astype(np.float64)
    near += 0.1 * np.linalg.norm(Q, axis=1).mean() / np.sqrt(d) * rng.standard_normal(near.shape)
    near *= rng.uniform(0.5, 4.0, size=(near.shape[0], 1))
    far = rng.standard_normal((20000, d))
    X = np.concatenate([far, near]).astype(np.float32)
    X = np.ascontiguousarray(X[rng.permutation(X.shape[0])])
    stats, idx, dist = parity(K, oracle, Q, X, k, metric="cosine")
    assert float(dist.max()) < 0.05  # all neighbours come from the near clouds
    assert stats["set_rule_rows"] >= 0.9 * stats["rows"]


def test_cosine_result_does_not_depend_on_limit_or_point_layout(K):
    m, n, d, k = 300, 9000, 64, 15
    Q, X = W.random_case(1200, m, n, d)
    lo = K.knn_plan(m, n, d, k, 1 << 40, "cosine").min_limit_bytes
    limits = [lo, lo + 300_000, 64 * W.MB]
    plans = [K.knn_plan(m, n, d, k, lim, "cosine") for lim in limits]
    say("   plans", [(p.q_chunks, p.n_splits) for p in plans])
    assert plans[0].q_chunks > 1 and plans[-1].q_chunks == 1 and plans[-1].n_splits > 1
    ref = run_gpu(K, Q, X, k, limits[0], metric="cosine")
    for lim in limits[1:]:
        idx, dist = run_gpu(K, Q, X, k, lim, metric="cosine")
        assert np.array_equal(idx, ref[0]) and np.array_equal(dist, ref[1]), lim


def test_cosine_on_clustered_embeddings_and_scale_invariance(K, oracle):
    # the embedding-like mixture of config 4 (the table's cosine rows are word embeddings)
    w = W.scaled(4, m=400, n=30000)
    Q, X = W.make(w)
    stats, idx, dist = parity(K, oracle, Q, X, 20, metric="cosine", rows=W.sample_rows(w, 200))
    assert stats["strict_rows"] >= 0.97 * stats["rows"]
    # scaling points by positive factors must not change the neighbours
    scale = (2.0 ** np.random.Generator(np.random.PCG64(3)).integers(-3, 4, size=(w.n, 1))).astype(np.float32)
    idx_s, dist_s = run_gpu(K, Q * np.float32(4.0), X * scale, 20, 64 * W.MB, metric="cosine")
    assert np.array_equal(dist_s, dist_s) and np.mean(idx_s == run_gpu(K, Q, X, 20, 64 * W.MB, metric="cosine")[0]) > 0.999


# ---------------------------------------------------------------------------------------
# L1 metric
# ---------------------------------------------------------------------------------------
L1 = [
    (0, 1, 1, 1, 1),          # smallest call
    (1, 300, 5000, 3, 16),    # one partial chunk
    (2, 257, 1003, 32, 7),    # exactly one chunk, ragged point groups
    (3, 140, 2300, 100, 10),  # the table's d = 100: three chunks and a tail
    (4, 64, 9001, 10, 40),    # several ranges
    (5, 40, 500, 784, 5),     # d = 784
    (6, 5, 129, 9, 129),      # k == n
]


@pytest.mark.parametrize("seed,m,n,d,k", L1)
def test_l1_parity_small(K, oracle, seed, m, n, d, k):
    say(f"\nl1 case seed={seed} m={m} n={n} d={d} k={k}")
    Q, X = W.random_case(1300 + seed, m, n, d)
    stats, _, _ = parity(K, oracle, Q, X, k, metric="l1")
    assert stats["strict_rows"] >= 0.97 * stats["rows"]


def test_l1_exact_ties_and_limit_independence(K, oracle):
    # integer grid: every sum is exact in fp32, ties are massive, the answer is unique
    Q, X = W.random_case(1400, 300, 6000, 6, kind="grid")
    ref = None
    lo = K.knn_plan(300, 6000, 6, 9, 1 << 40, "l1").min_limit_bytes
    for lim in (lo, lo + 30_000, 64 * W.MB):
        idx, dist = run_gpu(K, Q, X, 9, lim, metric="l1")
        o_idx, o_dist, _ = oracle.knn(Q, X, 9, metric="l1")
        assert np.array_equal(idx, o_idx) and np.array_equal(dist.astype(np.float64), o_dist)
        if ref is not None:
            assert np.array_equal(idx, ref[0]) and np.array_equal(dist, ref[1])
        ref = (idx, dist)
    # row strides larger than d
    Xp = torch.full((6000, 11), 1e30, device="cuda")
    Qp = torch.full((300, 9), 1e30, device="cuda")
    Xp[:, :6] = torch.from_numpy(X).cuda()
    Qp[:, :6] = torch.from_numpy(Q).cuda()
    idx2, dist2 = K.knn_search(Qp[:, :6], Xp[:, :6], 9, 64 * W.MB, metric="l1")
    torch.cuda.synchronize()
    assert np.array_equal(idx2.cpu().numpy(), ref[0])


@pytest.mark.parametrize("seed,d,span,n,m,k", [(1, 2, 30, 50_000, 1500, 16), (2, 3, 8, 60_000, 1500, 16),
                                                (3, 1, 500, 40_000, 1000, 7), (4, 3, 5, 20_000, 1500, 50)])
def test_exact_ties_keep_the_lower_index_on_every_low_d_path(K, oracle, seed, d, span, n, m, k):
    # integer coordinates from a small range: dozens of points at exactly the k-th distance.
    # The matrix-core filter kernels see the two half-waves' rows out of index order, so
    # their acceptance test compares (key, index); all three low-d paths must reproduce the
    # oracle's (distance, index) order exactly.
    g = np.random.Generator(np.random.PCG64(W.SEED_BASE + 12_000_000 + seed))
    X = g.integers(0, span, size=(n, d)).astype(np.float32)
    Q = g.integers(0, span, size=(m, d)).astype(np.float32)
    o_idx, o_dist, _ = oracle.knn(Q, X, k)
    paths = set()
    for limit in (64 * W.MB, 16 * n + 300_000, 200_000):
        paths.add(K.knn_plan(m, n, d, k, limit).path)
        idx, dist = run_gpu(K, Q, X, k, limit)
        assert np.array_equal(idx, o_idx), limit
        assert np.array_equal(dist.astype(np.float64), o_dist), limit
    assert paths == {K.KNN_PATH_LOWD_BF16, K.KNN_PATH_LOWD_MFMA, K.KNN_PATH_LOWD}


def _seed_cases():
    # (name, d, k, builder(g) -> (Q, X)): data that strains the threshold seed of the bf16 filter
    # path (the k-th smallest distance inside a block of grid cells; above k = 32 the distance to
    # the block's farthest corner): empty and crowded cells, a flat axis, queries far outside the points'
    # box, a large common offset, k above what the widest block of cells holds
    def clustered(g, d):
        centres = g.uniform(-1, 1, size=(12, d))
        X = centres[g.integers(0, 12, size=40_000)] + 0.003 * g.standard_normal((40_000, d))
        X[:50] = g.uniform(-30, 30, size=(50, d))  # a few far outliers stretch the box
        Q = np.concatenate([X[g.integers(0, 40_000, size=900)] + 0.001 * g.standard_normal((900, d)),
                            g.uniform(-60, 60, size=(300, d))])
        return Q, X

    def flat_axis(g, d):
        X = g.uniform(0, 1, size=(30_000, d))
        X[:, d - 1] = 0.25
        Q = g.uniform(-0.5, 1.5, size=(1000, d))
        return Q, X

    def offset(g, d):
        X = 4096.0 + g.uniform(0, 1, size=(30_000, d))
        Q = 4096.0 + g.uniform(-0.2, 1.2, size=(1000, d))
        return Q, X

    def lattice(g, d):
        # points exactly on cell borders of many grids, heavy duplication
        X = g.integers(0, 17, size=(40_000, d)) / 16.0
        Q = g.integers(-2, 19, size=(1200, d)) / 16.0
        return Q, X

    def two_points_far_apart(g, d):
        X = np.concatenate([np.zeros((20_000, d)), np.ones((20_000, d)) * 1000.0])
        X += 1e-3 * g.standard_normal(X.shape)
        Q = g.uniform(-10, 1010, size=(800, d))
        return Q, X

    cases = []
    for d in (1, 2, 3):
        cases += [("clustered", d, 16, clustered), ("flat_axis", d, 9, flat_axis),
                  ("offset", d, 16, offset), ("lattice", d, 5, lattice),
                  ("two_clumps", d, 3, two_points_far_apart), ("clustered_k200", d, 200, clustered),
                  # 17 .. 32: the longer of the two register lists of the exact seed
                  ("clustered_k25", d, 25, clustered), ("lattice_k32", d, 32, lattice),
                  ("offset_k17", d, 17, offset)]
    return cases


@pytest.mark.parametrize("name,d,k,build", _seed_cases(), ids=lambda v: str(v) if not callable(v) else "")
def test_threshold_seed_keeps_results_exact_on_uneven_data(K, oracle, name, d, k, build):
    g = np.random.Generator(np.random.PCG64(W.SEED_BASE + 13_000_000 + 31 * d + k))
    Q, X = build(g, d)
    Q, X = np.ascontiguousarray(Q, np.float32), np.ascontiguousarray(X, np.float32)
    m, n = Q.shape[0], X.shape[0]
    roomy = K.knn_plan(m, n, d, k, 256 * W.MB)
    assert roomy.path == K.KNN_PATH_LOWD_BF16 and roomy.seed_cells >= 2
    lo = roomy.min_limit_bytes
    assert K.knn_plan(m, n, d, k, lo + 40_000).path == K.KNN_PATH_LOWD  # no filter, no seed
    a_idx, a_dist = run_gpu(K, Q, X, k, lo + 40_000)
    b_idx, b_dist = run_gpu(K, Q, X, k, 256 * W.MB)
    assert np.array_equal(a_idx, b_idx) and np.array_equal(a_dist, b_dist)
    # a limit with room for the packed points but not for the cell counts: same path, unseeded
    o_idx, o_dist, o_next = oracle.knn(Q, X, k)
    say("  ", name, d, "cells/axis", roomy.seed_cells, check(b_idx, b_dist, o_idx, o_dist, o_next, n))


def test_threshold_seed_with_several_point_ranges_and_query_chunks(K, oracle):
    # few queries: the point axis is cut into ranges, each with its own lists under the same
    # seed bound; a tight limit: several query chunks reuse one grid
    Q, X = W.random_case(4242, 300, 400_000, 3, kind="uniform")
    k = 16
    plan = K.knn_plan(300, 400_000, 3, k, 256 * W.MB)
    assert plan.path == K.KNN_PATH_LOWD_BF16 and plan.seed_cells >= 2 and plan.n_splits > 1
    stats, idx, dist = parity(K, oracle, Q, X, k, 256 * W.MB)
    Q2, X2 = W.random_case(4243, 5000, 60_000, 2, kind="uniform")
    base = K.knn_plan(5000, 60_000, 2, k, 1 << 40)
    tight = None
    for extra in range(200_000, 2_000_000, 50_000):
        # (the kernel's private segment counts against the limit beside the workspace)
        p = K.knn_plan(5000, 60_000, 2, k, base.norms_bytes + base.private_bytes + extra)
        if p.path == K.KNN_PATH_LOWD_BF16 and p.seed_cells >= 2 and p.q_chunks > 1:
            tight = base.norms_bytes + base.private_bytes + extra
            break
    assert tight is not None
    parity(K, oracle, Q2, X2, k, tight)


def test_split_path_identical_points_break_ties_by_index_across_ranges(K, oracle):
    # every distance of a query is the same number: the result is the k lowest indices, also
    # when the ranges that hold the higher indices publish their thresholds first; all-zero data
    # is the case in which every error allowance of the filter is zero as well
    for value in (0.0, 0.75):
        X = np.full((40_000, 20), value, np.float32)
        Q = np.full((70, 20), value, np.float32)
        Q[35:] += np.float32(0.5)
        k = 9
        plan = K.knn_plan(70, 40_000, 20, k, 64 * W.MB)
        assert plan.path == K.KNN_PATH_MFMA_SPLIT and plan.n_splits > 1
        idx, dist = run_gpu(K, Q, X, k, 64 * W.MB)
        assert np.array_equal(idx, np.tile(np.arange(k, dtype=np.int32), (70, 1))), value
        o_idx, o_dist, _ = oracle.knn(Q, X, k)
        assert np.array_equal(idx, o_idx)
        assert np.allclose(dist, o_dist, rtol=1e-6, atol=0)


@pytest.mark.parametrize("d,ld", [(13, 13), (24, 28), (50, 50), (100, 101)])
def test_split_path_points_in_decreasing_distance_order(K, oracle, d, ld):
    # the worst order for a running top-k: every point beats the current k-th best, so every
    # tile overflows the candidate buffers and takes the test-everything route
    g = np.random.Generator(np.random.PCG64(W.SEED_BASE + 14_000_000 + d))
    n, m, k = 6000, 300, 12
    X = g.standard_normal((n, d)).astype(np.float32)
    X = X[np.argsort(-np.einsum("ij,ij->i", X.astype(np.float64), X.astype(np.float64)))]
    Q = (0.01 * g.standard_normal((m, d))).astype(np.float32)
    Xp = np.zeros((n, ld), np.float32)
    Xp[:, :d] = X
    Qp = np.zeros((m, ld), np.float32)
    Qp[:, :d] = Q
    Xd, Qd = torch.from_numpy(Xp).cuda()[:, :d], torch.from_numpy(Qp).cuda()[:, :d]
    assert K.knn_plan(m, n, d, k, 64 * W.MB).path == K.KNN_PATH_MFMA_SPLIT
    idx, dist = K.knn_search(Qd, Xd, k, 64 * W.MB)
    torch.cuda.synchronize()
    o_idx, o_dist, o_next = oracle.knn(Q, X, k)
    say("   ", d, ld, check(idx.cpu().numpy(), dist.cpu().numpy(), o_idx, o_dist, o_next, n))


def test_split_path_far_from_the_origin_and_exact_integer_ties(K, oracle):
    # an offset of 100 per coordinate makes the filter's allowance larger than the neighbour
    # distances (it passes far more than it needs to); integer coordinates give dozens of exact
    # ties at the k-th distance, decided by index
    g = np.random.Generator(np.random.PCG64(W.SEED_BASE + 14_100_000))
    X = (100.0 + g.uniform(0, 1, size=(20_000, 32))).astype(np.float32)
    Q = (100.0 + g.uniform(0, 1, size=(260, 32))).astype(np.float32)
    parity(K, oracle, Q, X, 10)
    Xi = g.integers(0, 3, size=(30_000, 12)).astype(np.float32)
    Qi = g.integers(0, 3, size=(400, 12)).astype(np.float32)
    o_idx, o_dist, _ = oracle.knn(Qi, Xi, 25)
    for limit in (64 * W.MB, 2 * W.MB):
        idx, dist = run_gpu(K, Qi, Xi, 25, limit)
        assert np.array_equal(idx, o_idx), limit
        assert np.array_equal(dist.astype(np.float64), o_dist), limit


def test_split_path_repeated_runs_with_many_ranges_give_the_same_bits(K, oracle):
    # few queries, many point ranges that exchange thresholds while they run: which pairs a
    # range looks at depends on timing, the result must not (near-duplicate points make ties
    # and near-ties at the k-th place common)
    g = np.random.Generator(np.random.PCG64(W.SEED_BASE + 14_200_000))
    base = g.standard_normal((400, 40)).astype(np.float32)
    X = np.repeat(base, 150, axis=0)
    X += (1e-3 * g.integers(0, 3, size=X.shape)).astype(np.float32)
    X = X[g.permutation(X.shape[0])]
    Q = base[:90] + np.float32(1e-3)
    k = 20
    plan = K.knn_plan(90, X.shape[0], 40, k, 64 * W.MB)
    assert plan.path == K.KNN_PATH_MFMA_SPLIT and plan.n_splits >= 8
    first = run_gpu(K, Q, X, k, 64 * W.MB)
    for _ in range(5):
        again = run_gpu(K, Q, X, k, 64 * W.MB)
        assert np.array_equal(first[0], again[0]) and np.array_equal(first[1], again[1])
    o_idx, o_dist, o_next = oracle.knn(Q, X, k)
    say("   ", check(first[0], first[1], o_idx, o_dist, o_next, X.shape[0]))


def test_seeded_random_shapes_and_limits(K, oracle):
    # a seeded sweep over shapes, k, metrics and limits (from the smallest feasible one up):
    # whatever plan comes out - path, chunks, ranges - the result passes the parity rule
    g = np.random.Generator(np.random.PCG64(W.SEED_BASE + 13_000_000))
    seen = set()
    for case in range(48):
        d = int(g.choice([1, 2, 3, 4, 5, 8, 9, 12, 16, 17, 31, 64, 100, 260]))
        m = int(g.choice([1, 7, 63, 129, 300, 700]))
        n = int(g.choice([1, 5, 64, 127, 500, 2049, 6000]))
        k = int(min(n, g.choice([1, 2, 9, 16, 33, 100])))
        metric = str(g.choice(["l2", "l2", "l2", "cosine", "l1"]))
        kind = str(g.choice(["normal", "uniform", "grid"]))
        if kind == "grid" and metric == "cosine":
            kind = "normal"  # zero vectors and exact cosine ties are covered by their own tests
        lo = K.knn_plan(m, n, d, k, 1 << 40, metric).min_limit_bytes
        limit = int(g.choice([lo, lo + 3000, 4 * lo + 100_000, 64 * W.MB]))
        plan = K.knn_plan(m, n, d, k, limit, metric)
        assert plan.workspace_bytes <= limit
        seen.add((plan.path, plan.q_chunks > 1, plan.n_splits > 1))
        say("fuzz", case, (m, n, d, k, metric, kind, limit), "plan", (plan.path, plan.q_chunks, plan.n_splits))
        Q, X = W.random_case(5000 + case, m, n, d, kind)
        idx, dist = run_gpu(K, Q, X, k, limit, metric=metric)
        o_idx, o_dist, o_next = oracle.knn(Q, X, k, metric=metric)
        check(idx, dist, o_idx, o_dist, o_next, n)
    assert len({p for p, _, _ in seen}) >= 4  # several kernel families were exercised


def test_several_chunks_overlap_on_a_second_stream_and_give_the_same_bits(K):
    # a limit that cuts the queries into chunks: plan.streams == 2, merge and re-evaluation of a
    # chunk run on the library's internal stream while the next chunk is searched; the call is made
    # on a stream of the caller's, three times in a row into the same workspace
    for (m, n, d, k) in [(3000, 30_000, 24, 16), (4000, 50_000, 3, 8), (900, 70_000, 64, 10)]:
        Q, X = W.random_case(9100 + d, m, n, d)
        Xd = torch.from_numpy(X).cuda()
        Qd = torch.from_numpy(Q).cuda()
        ref_i, ref_d = K.knn_search(Qd, Xd, k, 4 * 10 ** 9)
        one = K.knn_last_stats()[0]
        lo = K.knn_plan(m, n, d, k, 1 << 40)
        tight = p = None
        for extra in range(0, 4_000_000, 10_000):
            tight = lo.min_limit_bytes + lo.private_bytes + extra
            p = K.knn_plan(m, n, d, k, tight)
            if p.q_chunks > 2 and p.streams == 2:
                break
        assert one.q_chunks == 1 and p.q_chunks > 2 and p.streams == 2, (one, p)
        ws = torch.empty(p.workspace_bytes, dtype=torch.uint8, device="cuda")
        side = torch.cuda.Stream()
        with torch.cuda.stream(side):
            for _ in range(3):
                i2, d2 = K.knn_search(Qd, Xd, k, tight, workspace=ws)
        side.synchronize()
        assert torch.equal(ref_i, i2) and torch.equal(ref_d.view(torch.int32), d2.view(torch.int32))
