"""GPU parity tests of the packed path (8 < d <= 256, at least 64 queries - 2048 up to d = 16 - and 65536 points, room for the points
rounded to bf16): through the C ABI against the CPU oracle on sampled rows, and bit for bit
against the split path, which the same call takes under a limit too small for the packed copy.
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


def both_paths(K, Qd, Xd, k, big=4 * 10 ** 9, metric="l2"):
    """(idx, dist) on the packed path, after checking that the split path gives the same bits."""
    m, d = Qd.shape
    n = Xd.shape[0]
    p6 = K.knn_plan(m, n, d, k, big, metric)
    assert p6.path == K.KNN_PATH_MFMA_PACKED, p6
    small = K.knn_plan(m, n, d, k, 1 << 44, metric).min_limit_bytes + 10 ** 6
    p5 = K.knn_plan(m, n, d, k, small, metric)
    assert p5.path == K.KNN_PATH_MFMA_SPLIT, p5
    i6, d6 = K.knn_search(Qd, Xd, k, big, metric=metric)
    torch.cuda.synchronize()
    plan, peak = K.knn_last_stats()
    assert plan.path == K.KNN_PATH_MFMA_PACKED and peak <= big
    i5, d5 = K.knn_search(Qd, Xd, k, small, metric=metric)
    torch.cuda.synchronize()
    same_i = torch.equal(i6, i5)
    same_d = torch.equal(d6.view(torch.int32), d5.view(torch.int32))
    if not (same_i and same_d):
        bad = (i6 != i5).any(dim=1).nonzero().flatten()
        say("   rows that differ between the paths:", bad[:10].tolist(), "of", int(bad.numel()))
    assert same_i and same_d
    return i6.cpu().numpy(), d6.cpu().numpy()


def against_oracle(oracle, Q, X, k, idx, dist, rows, metric="l2"):
    o_idx, o_dist, o_next = oracle.knn(Q, X, k, rows=rows, metric=metric)
    stats = check(idx[rows], dist[rows], o_idx, o_dist, o_next, X.shape[0])
    say("   parity", stats)
    return stats


# (seed, m, n, d, k, kind): every instantiated chunk count, ragged query tiles, ragged last step
CASES = [
    (1, 2500, 70001, 128, 10, "normal"),     # 8 chunks, n not a multiple of 64
    (2, 2333, 131072, 32, 16, "normal"),     # 2 chunks
    (3, 2700, 90000, 48, 5, "uniform"),      # 3 chunks
    (4, 2513, 80000, 64, 100, "normal"),     # 4 chunks, k = 100
    (5, 2200, 66000, 80, 7, "normal"),       # 5 chunks
    (6, 3500, 100000, 96, 10, "clustered"),  # 6 chunks
    (7, 2900, 120000, 100, 10, "clustered"), # 7 chunks, the shape of the embedding rows
    (8, 2400, 70000, 144, 12, "normal"),     # 9 chunks -> 10
    (9, 2400, 70000, 192, 12, "normal"),     # 12 chunks
    (10, 2300, 70000, 200, 9, "normal"),     # 13 chunks -> 14
    (11, 2600, 75000, 256, 32, "normal"),    # 16 chunks
    (12, 2048, 65536, 20, 3, "normal"),      # the fewest points the path takes, d % 16 != 0
    (13, 64, 70000, 128, 10, "normal"),      # the fewest queries the path takes
    (14, 333, 80000, 256, 40, "clustered"),  # a few hundred queries, d = 256
    (15, 2500, 70000, 16, 10, "normal"),     # one chunk
    (16, 2048, 66000, 16, 33, "uniform"),    # one chunk, the fewest queries it takes
    (17, 2300, 90000, 12, 5, "clustered"),   # one chunk, a quarter of it padding
    (18, 2200, 70000, 64, 1024, "normal"),   # k above 789: eight waves per workgroup at d <= 128 too
    (19, 2100, 140000, 128, 300, "clustered"),  # a seed sample of 160 k = 48000 > n / 4 points: capped
]


def make(seed, m, n, d, kind):
    rng = np.random.default_rng(1000 + seed)
    if kind == "normal":
        X = rng.standard_normal((n, d), dtype=np.float32)
        Q = rng.standard_normal((m, d), dtype=np.float32)
    elif kind == "uniform":
        X = rng.random((n, d), dtype=np.float32)
        Q = rng.random((m, d), dtype=np.float32)
    else:
        c = 2.0 * rng.standard_normal((50, d), dtype=np.float32)
        X = c[rng.integers(0, 50, n)] + rng.standard_normal((n, d), dtype=np.float32)
        Q = c[rng.integers(0, 50, m)] + rng.standard_normal((m, d), dtype=np.float32)
    return Q, X


@pytest.mark.parametrize("seed,m,n,d,k,kind", CASES)
def test_packed_parity(K, oracle, seed, m, n, d, k, kind):
    say(f"packed case seed={seed} m={m} n={n} d={d} k={k} {kind}")
    Q, X = make(seed, m, n, d, kind)
    Xd = torch.from_numpy(X).cuda()
    Qd = torch.from_numpy(Q).cuda()
    idx, dist = both_paths(K, Qd, Xd, k)
    rows = np.unique(np.concatenate([np.arange(0, m, max(1, m // 24)), [m - 1]]))
    against_oracle(oracle, Q, X, k, idx, dist, rows)


# the cosine metric on the packed path: the copy holds the rows x / |x|
COSINE_CASES = [
    (31, 2500, 70001, 100, 10, "clustered"),  # the shape of the embedding rows, three waves per SIMD
    (32, 2300, 80000, 256, 32, "normal"),     # 16 chunks, two waves per SIMD
    (33, 2100, 90000, 16, 33, "normal"),      # one chunk
    (34, 300, 66000, 64, 7, "zeros"),         # zero rows among points and queries: distance 1
    (35, 2200, 70000, 40, 5, "scales"),       # row lengths over four orders of magnitude
]


@pytest.mark.parametrize("seed,m,n,d,k,kind", COSINE_CASES)
def test_packed_cosine_parity(K, oracle, seed, m, n, d, k, kind):
    say(f"packed cosine case seed={seed} m={m} n={n} d={d} k={k} {kind}")
    Q, X = make(seed, m, n, d, "clustered" if kind == "clustered" else "normal")
    rng = np.random.default_rng(seed)
    if kind == "zeros":
        X[::97] = 0
        Q[5] = 0
    if kind == "scales":
        X *= (10.0 ** rng.uniform(-2, 2, (n, 1))).astype(np.float32)
        Q *= (10.0 ** rng.uniform(-2, 2, (m, 1))).astype(np.float32)
    idx, dist = both_paths(K, torch.from_numpy(Q).cuda(), torch.from_numpy(X).cuda(), k, metric="cosine")
    rows = np.unique(np.concatenate([np.arange(0, m, max(1, m // 24)), [5, m - 1]]))
    against_oracle(oracle, Q, X, k, idx, dist, rows, metric="cosine")


def test_packed_worst_order_stream_overflows_the_buffers(K, oracle):
    # points sorted by decreasing distance from the queries' common neighbourhood: every step
    # brings pairs under every threshold, so the buffers overflow and steps are made good
    say("packed worst-order case")
    rng = np.random.default_rng(77)
    n, d, m, k = 70000, 32, 2300, 8
    X = rng.standard_normal((n, d), dtype=np.float32)
    order = np.argsort(-np.linalg.norm(X, axis=1))
    X = np.ascontiguousarray(X[order])
    Q = 0.01 * rng.standard_normal((m, d), dtype=np.float32)
    Xd = torch.from_numpy(X).cuda()
    Qd = torch.from_numpy(Q).cuda()
    idx, dist = both_paths(K, Qd, Xd, k)
    against_oracle(oracle, Q, X, k, idx, dist, np.arange(0, m, 97))


def test_packed_ties_go_to_the_lower_index(K):
    # every point appears four times, far apart in the stream: each query's result is whole
    # groups of equal distances, which must come out in index order
    say("packed duplicated-points case")
    rng = np.random.default_rng(5)
    base, d, m, k = 20000, 64, 2200, 12
    B = rng.standard_normal((base, d), dtype=np.float32)
    X = np.concatenate([B, B, B, B])
    Q = rng.standard_normal((m, d), dtype=np.float32)
    idx, dist = both_paths(K, torch.from_numpy(Q).cuda(), torch.from_numpy(X).cuda(), k)
    assert (idx[:, 0::4] + base == idx[:, 1::4]).all() and (idx[:, 1::4] + base == idx[:, 2::4]).all()
    assert (idx[:, 2::4] + base == idx[:, 3::4]).all() and (idx[:, 0::4] < base).all()
    assert (dist[:, 0::4] == dist[:, 3::4]).all()


def test_packed_strided_rows_and_query_chunks(K, oracle):
    # rows with a stride larger than d (still 16-byte aligned), and a limit that cuts the
    # queries into several chunks on the packed path
    say("packed strided / chunked case")
    rng = np.random.default_rng(9)
    n, d, m, k = 80000, 40, 3000, 20
    Xs = torch.from_numpy(rng.standard_normal((n, 48), dtype=np.float32)).cuda()
    Qs = torch.from_numpy(rng.standard_normal((m, 44), dtype=np.float32)).cuda()
    Xd, Qd = Xs[:, :d], Qs[:, :d]
    ref_i, ref_d = K.knn_search(Qd.contiguous(), Xd.contiguous(), k, 4 * 10 ** 9)
    i1, d1 = K.knn_search(Qd, Xd, k, 4 * 10 ** 9)
    torch.cuda.synchronize()
    assert K.knn_last_stats()[0].path == K.KNN_PATH_MFMA_PACKED
    assert torch.equal(ref_i, i1) and torch.equal(ref_d.view(torch.int32), d1.view(torch.int32))
    lo = K.knn_plan(m, n, d, k, 4 * 10 ** 9)
    tight = lo.norms_bytes + 1_200_000
    p = K.knn_plan(m, n, d, k, tight)
    assert p.path == K.KNN_PATH_MFMA_PACKED and p.q_chunks > 1, p
    i2, d2 = K.knn_search(Qd, Xd, k, tight)
    torch.cuda.synchronize()
    assert torch.equal(ref_i, i2) and torch.equal(ref_d.view(torch.int32), d2.view(torch.int32))
    X = Xd.contiguous().cpu().numpy()
    Q = Qd.contiguous().cpu().numpy()
    against_oracle(oracle, Q, X, k, ref_i.cpu().numpy(), ref_d.cpu().numpy(), np.arange(0, m, 97))


def test_packed_unaligned_rows_fall_back_to_the_split_kernel(K, oracle):
    # d % 4 != 0: the plan is the packed one, the call runs the split kernel inside its workspace
    say("packed plan, unaligned rows")
    rng = np.random.default_rng(11)
    n, d, m, k = 70000, 30, 2150, 6
    X = rng.standard_normal((n, d), dtype=np.float32)
    Q = rng.standard_normal((m, d), dtype=np.float32)
    idx, dist = both_paths(K, torch.from_numpy(Q).cuda(), torch.from_numpy(X).cuda(), k)
    against_oracle(oracle, Q, X, k, idx, dist, np.arange(0, m, 89))


def test_packed_slabs_under_a_limit_without_room_for_the_whole_copy(K, oracle):
    # the bf16 copy of all points does not fit: the points are packed and searched slab after slab
    # into the same buffer, the lists carrying over; same bits as with the whole copy and as the
    # split path
    say("packed slabs case")
    rng = np.random.default_rng(31)
    n, d, m, k = 600_001, 40, 2500, 20
    X = rng.standard_normal((n, d), dtype=np.float32)
    Q = rng.standard_normal((m, d), dtype=np.float32)
    Xd, Qd = torch.from_numpy(X).cuda(), torch.from_numpy(Q).cuda()
    full = K.knn_plan(m, n, d, k, 4 * 10 ** 9)
    assert full.path == K.KNN_PATH_MFMA_PACKED and full.slab_points >= n
    ref_i, ref_d = K.knn_search(Qd, Xd, k, 4 * 10 ** 9)
    seen = set()
    for frac in (0.6, 0.3):
        lim = int(full.norms_bytes * frac) + full.query_bytes + full.lists_bytes + 4 * 10 ** 6
        p = K.knn_plan(m, n, d, k, lim)
        assert p.path == K.KNN_PATH_MFMA_PACKED and 131072 <= p.slab_points < n and p.q_chunks == 1, p
        assert p.workspace_bytes <= lim
        seen.add(-(-n // p.slab_points))
        guard = 4096
        ws = torch.full((p.workspace_bytes + guard,), 0x3C, dtype=torch.uint8, device="cuda")
        i2, d2 = K.knn_search(Qd, Xd, k, lim, workspace=ws[:p.workspace_bytes])
        torch.cuda.synchronize()
        assert bool((ws[p.workspace_bytes:] == 0x3C).all())
        assert torch.equal(ref_i, i2) and torch.equal(ref_d.view(torch.int32), d2.view(torch.int32)), p
    assert len(seen) >= 2, seen  # different slab counts, one of them with a short last slab
    against_oracle(oracle, Q, X, k, ref_i.cpu().numpy(), ref_d.cpu().numpy(), np.arange(0, m, 101))
