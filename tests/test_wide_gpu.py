"""GPU parity tests of the wide path (d > 256, at least 16 queries and 65536 points, k <= 512, room for
the points rounded to bf16): through the C ABI against the CPU oracle on sampled rows, and bit for
bit against the split path, which the same call takes under a limit too small for the packed copy.
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


def both_paths(K, Qd, Xd, k, big=4 * 10 ** 9):
    """(idx, dist) on the wide path, after checking that the split path gives the same bits."""
    m, d = Qd.shape
    n = Xd.shape[0]
    p7 = K.knn_plan(m, n, d, k, big)
    assert p7.path == K.KNN_PATH_MFMA_WIDE, p7
    # a limit with room for the split path's largest chunk but not for a slab of the copy
    small = p7.min_limit_bytes + 8 * 10 ** 6
    p5 = K.knn_plan(m, n, d, k, small)
    assert p5.path == K.KNN_PATH_MFMA_SPLIT, p5
    i7, d7 = K.knn_search(Qd, Xd, k, big)
    torch.cuda.synchronize()
    plan, peak = K.knn_last_stats()
    assert plan.path == K.KNN_PATH_MFMA_WIDE and peak <= big
    i5, d5 = K.knn_search(Qd, Xd, k, small)
    torch.cuda.synchronize()
    same_i = torch.equal(i7, i5)
    same_d = torch.equal(d7.view(torch.int32), d5.view(torch.int32))
    if not (same_i and same_d):
        bad = (i7 != i5).any(dim=1).nonzero().flatten()
        say("   rows that differ between the paths:", bad[:10].tolist(), "of", int(bad.numel()))
    assert same_i and same_d
    return i7.cpu().numpy(), d7.cpu().numpy()


def against_oracle(oracle, Q, X, k, idx, dist, rows):
    o_idx, o_dist, o_next = oracle.knn(Q, X, k, rows=rows)
    stats = check(idx[rows], dist[rows], o_idx, o_dist, o_next, X.shape[0])
    say("   parity", stats)
    return stats


def make(seed, m, n, d, kind):
    rng = np.random.default_rng(2000 + seed)
    if kind == "image":  # the image-like rows of the d = 784 workload: 80 % zeros, else uniform in (0, 1]
        X = (1.0 - rng.random((n, d), dtype=np.float32)) * (rng.random((n, d), dtype=np.float32) < 0.2)
        Q = (1.0 - rng.random((m, d), dtype=np.float32)) * (rng.random((m, d), dtype=np.float32) < 0.2)
        return Q.astype(np.float32), X.astype(np.float32)
    if kind == "normal":
        return rng.standard_normal((m, d), dtype=np.float32), rng.standard_normal((n, d), dtype=np.float32)
    if kind == "uniform":
        return rng.random((m, d), dtype=np.float32), rng.random((n, d), dtype=np.float32)
    c = 2.0 * rng.standard_normal((40, d), dtype=np.float32)
    X = c[rng.integers(0, 40, n)] + rng.standard_normal((n, d), dtype=np.float32)
    Q = c[rng.integers(0, 40, m)] + rng.standard_normal((m, d), dtype=np.float32)
    return Q, X


# (seed, m, n, d, k, kind): odd and even stage counts per tile, ragged query tiles and point tiles,
# k below and above the 32 slots of a candidate buffer, the largest k the path takes
CASES = [
    (1, 2500, 70001, 784, 10, "image"),      # 49 chunks -> 50: 25 stages
    (2, 2100, 66000, 260, 5, "normal"),      # 17 chunks -> 18: 9 stages
    (3, 2300, 80000, 512, 100, "normal"),    # 32 chunks: 16 stages, first tiles overflow the buffers
    (4, 2049, 65613, 300, 1, "uniform"),     # k = 1, one query in the last tile's last wave
    (5, 2560, 70000, 272, 512, "normal"),    # k = 512
    (6, 3000, 90000, 400, 33, "clustered"),  # 25 chunks -> 26
    (7, 2048, 65536, 260, 128, "normal"),    # the smallest shape the path takes; k = the points of a tile
    (8, 2100, 66001, 264, 129, "uniform"),   # k above a tile's points: no bound from the first tile
    (9, 16, 70000, 784, 10, "image"),        # the fewest queries the path takes: one wave holds them all
    (10, 700, 131072, 300, 20, "normal"),    # two query tiles, 64 ranges
]


@pytest.mark.parametrize("seed,m,n,d,k,kind", CASES)
def test_wide_parity(K, oracle, seed, m, n, d, k, kind):
    say(f"wide case seed={seed} m={m} n={n} d={d} k={k} {kind}")
    Q, X = make(seed, m, n, d, kind)
    idx, dist = both_paths(K, torch.from_numpy(Q).cuda(), torch.from_numpy(X).cuda(), k)
    rows = np.unique(np.concatenate([np.arange(0, m, max(1, m // 16)), [m - 1]]))
    against_oracle(oracle, Q, X, k, idx, dist, rows)


def test_wide_plan_bounds(K):
    # what the path does not take goes to the split path
    big = 8 * 10 ** 9
    assert K.knn_plan(4000, 100000, 300, 513, big).path == K.KNN_PATH_MFMA_SPLIT   # k > 512
    assert K.knn_plan(15, 100000, 300, 10, big).path == K.KNN_PATH_MFMA_SPLIT      # few queries
    assert K.knn_plan(16, 100000, 300, 10, big).n_splits == 48                     # one query tile: ranges of at least 16 point tiles
    assert K.knn_plan(16, 1000000, 300, 10, big).n_splits == 64                    # at most 64
    assert K.knn_plan(4000, 65535, 300, 10, big).path == K.KNN_PATH_MFMA_SPLIT     # few points
    assert K.knn_plan(4000, 100000, 256, 10, big).path == K.KNN_PATH_MFMA_PACKED   # d <= 256
    assert K.knn_plan(4000, 100000, 300, 10, big, "cosine").path == K.KNN_PATH_MFMA_SPLIT
    p = K.knn_plan(4000, 100000, 300, 10, big)
    assert p.path == K.KNN_PATH_MFMA_WIDE and p.tile_q == 512 and p.slab_points == 100032
    assert p.workspace_bytes == p.norms_bytes + p.query_bytes + p.lists_bytes


def test_wide_worst_order_stream_overflows_the_buffers(K, oracle):
    # points sorted by decreasing distance from the queries' common neighbourhood: every tile
    # brings pairs under every threshold, so buffers overflow and whole tiles are evaluated
    say("wide worst-order case")
    rng = np.random.default_rng(78)
    n, d, m, k = 66000, 320, 2100, 8
    X = rng.standard_normal((n, d), dtype=np.float32)
    X = np.ascontiguousarray(X[np.argsort(-np.linalg.norm(X, axis=1))])
    Q = 0.01 * rng.standard_normal((m, d), dtype=np.float32)
    idx, dist = both_paths(K, torch.from_numpy(Q).cuda(), torch.from_numpy(X).cuda(), k)
    against_oracle(oracle, Q, X, k, idx, dist, np.arange(0, m, 131))


def test_wide_ties_go_to_the_lower_index(K):
    # every point appears four times, far apart in the stream: each query's result is whole
    # groups of equal distances, which must come out in index order
    say("wide duplicated-points case")
    rng = np.random.default_rng(6)
    base, d, m, k = 17000, 288, 2100, 12
    B = rng.standard_normal((base, d), dtype=np.float32)
    X = np.concatenate([B, B, B, B])
    Q = rng.standard_normal((m, d), dtype=np.float32)
    idx, dist = both_paths(K, torch.from_numpy(Q).cuda(), torch.from_numpy(X).cuda(), k)
    assert (idx[:, 0::4] + base == idx[:, 1::4]).all() and (idx[:, 1::4] + base == idx[:, 2::4]).all()
    assert (idx[:, 2::4] + base == idx[:, 3::4]).all() and (idx[:, 0::4] < base).all()
    assert (dist[:, 0::4] == dist[:, 3::4]).all()


def test_wide_strided_rows_unaligned_rows_and_query_chunks(K, oracle):
    say("wide strided / unaligned / chunked case")
    rng = np.random.default_rng(10)
    n, d, m, k = 70000, 300, 5000, 20
    Xs = torch.from_numpy(rng.standard_normal((n, 308), dtype=np.float32)).cuda()
    Qs = torch.from_numpy(rng.standard_normal((m, 304), dtype=np.float32)).cuda()
    Xd, Qd = Xs[:, :d], Qs[:, :d]
    big = 4 * 10 ** 9
    ref_i, ref_d = K.knn_search(Qd.contiguous(), Xd.contiguous(), k, big)
    i1, d1 = K.knn_search(Qd, Xd, k, big)  # strides 308 / 304 floats: still 16-byte aligned rows
    torch.cuda.synchronize()
    assert K.knn_last_stats()[0].path == K.KNN_PATH_MFMA_WIDE
    assert torch.equal(ref_i, i1) and torch.equal(ref_d.view(torch.int32), d1.view(torch.int32))
    # rows that are not 16-byte aligned: the same plan runs on the split kernel
    Xu = torch.from_numpy(rng.standard_normal((n, 301), dtype=np.float32)).cuda()
    Xu[:, :d] = Xd
    i3, d3 = K.knn_search(Qd, Xu[:, :d], k, big)
    torch.cuda.synchronize()
    assert K.knn_last_stats()[0].path == K.KNN_PATH_MFMA_WIDE
    assert torch.equal(ref_i, i3) and torch.equal(ref_d.view(torch.int32), d3.view(torch.int32))
    # a limit that cuts the queries into several chunks (two sets of lists, two streams)
    full = K.knn_plan(m, n, d, k, big)
    tight = full.norms_bytes + 2_600_000
    p = K.knn_plan(m, n, d, k, tight)
    assert p.path == K.KNN_PATH_MFMA_WIDE and p.q_chunks > 1, p
    i2, d2 = K.knn_search(Qd, Xd, k, tight)
    torch.cuda.synchronize()
    assert torch.equal(ref_i, i2) and torch.equal(ref_d.view(torch.int32), d2.view(torch.int32))
    X = Xd.contiguous().cpu().numpy()
    Q = Qd.contiguous().cpu().numpy()
    against_oracle(oracle, Q, X, k, ref_i.cpu().numpy(), ref_d.cpu().numpy(), np.arange(0, m, 211))


def test_wide_slabs_under_a_limit_without_room_for_the_whole_copy(K, oracle):
    # the bf16 copy of all points does not fit: the points are packed and searched slab after
    # slab into the same buffer, the lists carrying over; same bits as with the whole copy
    say("wide slabs case")
    rng = np.random.default_rng(32)
    n, d, m, k = 600_001, 272, 2500, 20
    X = rng.standard_normal((n, d), dtype=np.float32)
    Q = rng.standard_normal((m, d), dtype=np.float32)
    Xd, Qd = torch.from_numpy(X).cuda(), torch.from_numpy(Q).cuda()
    big = 4 * 10 ** 9
    full = K.knn_plan(m, n, d, k, big)
    assert full.path == K.KNN_PATH_MFMA_WIDE and full.slab_points >= n
    ref_i, ref_d = K.knn_search(Qd, Xd, k, big)
    seen = set()
    for frac in (0.6, 0.3):
        lim = int(full.norms_bytes * frac) + full.query_bytes + full.lists_bytes + 4 * 10 ** 6
        p = K.knn_plan(m, n, d, k, lim)
        assert p.path == K.KNN_PATH_MFMA_WIDE and 131072 <= p.slab_points < n and p.q_chunks == 1, p
        assert p.workspace_bytes <= lim
        seen.add(-(-n // p.slab_points))
        guard = 4096
        ws = torch.full((p.workspace_bytes + guard,), 0x3C, dtype=torch.uint8, device="cuda")
        i2, d2 = K.knn_search(Qd, Xd, k, lim, workspace=ws[:p.workspace_bytes])
        torch.cuda.synchronize()
        assert bool((ws[p.workspace_bytes:] == 0x3C).all())
        assert torch.equal(ref_i, i2) and torch.equal(ref_d.view(torch.int32), d2.view(torch.int32)), p
    assert len(seen) >= 2, seen
    against_oracle(oracle, Q, X, k, ref_i.cpu().numpy(), ref_d.cpu().numpy(), np.arange(0, m, 127))
