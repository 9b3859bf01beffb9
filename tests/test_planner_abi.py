"""CPU-only tests: the C-ABI library loads, exports every declared symbol, and the host
planner's arithmetic holds (no GPU call is made)."""
import ctypes
import os
import re

import pytest

import paper_2206_14148_amd as K

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    names = set()
    for header in ("knn.h", "kmv.h", "sgpr.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b((?:knn|kmv|sgpr)_[a-z0-9_]+)\s*\(", text))
    return sorted(names)


def test_library_loads_and_exports_every_declared_symbol():
    lib = K.load()
    names = declared_symbols()
    assert set(names) == set(K.EXPORTED_SYMBOLS)
    for name in names:
        assert getattr(lib, name) is not None
    raw = ctypes.CDLL(K.library_path())
    for name in names:
        getattr(raw, name)  # AttributeError if missing


def test_worked_example_from_the_paper_appendix():
    # golden fixture: 1GB threshold, rows of 1e6 fp64 entries -> 125 rows
    path = os.path.join(ROOT, "tests", "golden", "planner_worked_example.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    assert rows
    for limit_text, entries, width, expected in rows:
        limit = K.knn_parse_size(limit_text)
        assert limit == 10 ** 9
        assert K.knn_chunk_rows(limit, int(entries) * int(width)) == int(expected)


@pytest.mark.parametrize("text,val", [("64MB", 64 * 10 ** 6), ("1GB", 10 ** 9), ("500MB", 5 * 10 ** 8),
                                      ("2kb", 2000), ("123", 123), ("7B", 7), ("3TB", 3 * 10 ** 12),
                                      (" 8GB ", 8 * 10 ** 9)])
def test_parse_size_decimal(text, val):
    assert K.knn_parse_size(text) == val


@pytest.mark.parametrize("text", ["", "GB", "1.5GB", "1GiB", "-1MB", "1 GB x", "99999999999999999999999"])
def test_parse_size_rejects(text):
    with pytest.raises(K.KnnError):
        K.knn_parse_size(text)


def test_chunk_rows_floor():
    assert K.knn_chunk_rows(999, 1000) == 0
    assert K.knn_chunk_rows(1000, 1000) == 1
    assert K.knn_chunk_rows(1999, 1000) == 1
    assert K.knn_chunk_rows(5, 0) == 0


# (m, n, d, k, limit, path): d <= 8 with room for the packed points takes the low-d matrix-core
# filter; 8 < d <= 256 with room for the points rounded to bf16 (32 bytes per point and 16
# coordinates: 2.56 GB at d = 128, n = 1e7; 1.02 GB at d = 256, n = 2e6) or of a slab of them (at
# least 65536 points) the packed path
CONFIGS = [
    (1_000, 10_000, 16, 10, 64 * 10 ** 6, K.KNN_PATH_MFMA_SPLIT),
    (1_000_000, 1_000_000, 3, 16, 10 ** 9, K.KNN_PATH_LOWD_BF16),
    (10_000, 1_000_000, 784, 10, 2 * 10 ** 9, K.KNN_PATH_MFMA_WIDE),
    (100_000, 10_000_000, 128, 100, 8 * 10 ** 9, K.KNN_PATH_MFMA_PACKED),
    (50_000, 2_000_000, 256, 32, 128 * 10 ** 6, K.KNN_PATH_MFMA_PACKED),  # slabs of the copy
    (50_000, 2_000_000, 256, 32, 10 ** 9, K.KNN_PATH_MFMA_PACKED),        # two slabs
    (50_000, 2_000_000, 256, 32, 8 * 10 ** 9, K.KNN_PATH_MFMA_PACKED),
    (50_000, 2_000_000, 256, 32, 64 * 10 ** 9, K.KNN_PATH_MFMA_PACKED),
]


@pytest.mark.parametrize("m,n,d,k,limit,want", CONFIGS)
def test_every_baseline_config_has_a_plan_under_its_limit(m, n, d, k, limit, want):
    p = K.knn_plan(m, n, d, k, limit)
    assert p.workspace_bytes <= limit
    assert p.workspace_bytes == p.norms_bytes + p.query_bytes + p.lists_bytes
    assert p.path == want
    assert p.q_chunks * p.chunk_rows >= m
    assert p.chunk_rows == m or p.chunk_rows % p.tile_q == 0
    # every concurrently live list is counted: rows x ranges x k x (key + index)
    assert p.lists_bytes >= p.chunk_rows * p.n_splits * k * 8
    assert K.knn_workspace_bytes(m, n, d, k, limit) == p.workspace_bytes


def test_min_limit_is_exact_boundary():
    for (m, n, d, k) in [(1000, 10000, 16, 10), (5000, 20000, 3, 16), (7, 50, 4, 50), (100000, 10 ** 7, 128, 100)]:
        p = K.knn_plan(m, n, d, k, 1 << 40)
        lo = p.min_limit_bytes
        q = K.knn_plan(m, n, d, k, lo)
        assert q.workspace_bytes <= lo and q.n_splits == 1
        with pytest.raises(K.KnnError) as ei:
            K.knn_plan(m, n, d, k, lo - 1)
        assert ei.value.status == K.KNN_ERR_MEM_LIMIT_TOO_SMALL
        assert ei.value.min_limit_bytes == lo


def test_small_limits_cut_queries_into_chunks_and_never_exceed_the_limit():
    m, n, d, k = 50_000, 2_000_000, 256, 32
    prev_lists = prev_path = None
    for limit in [8_400_000, 8_700_000, 9_000_000, 12_000_000, 20_000_000, 50_000_000, 128_000_000, 10 ** 9]:
        p = K.knn_plan(m, n, d, k, limit)
        assert p.workspace_bytes <= limit
        assert p.chunk_rows >= p.tile_q or p.chunk_rows == m
        # more memory never means fewer (query, range) lists in flight; the chunk count itself
        # may go up when the plan trades rows for ranges (more workgroups per launch)
        # (with several chunks two sets of lists are live, one being merged while the other is
        # filled: plan.streams == 2)
        # (compared between plans of one kernel family: with room for a slab of the bf16 copy the
        # plan changes to the packed path, which takes all queries in one chunk of few ranges)
        if prev_lists is not None and p.path == prev_path:
            assert p.chunk_rows * p.n_splits * p.streams >= prev_lists
        prev_lists = p.chunk_rows * p.n_splits * p.streams
        prev_path = p.path
        assert p.streams == (2 if p.q_chunks > 1 and p.lists_bytes >= 4 * p.tile_q * p.n_splits * k * 4 else 1)
    tight = K.knn_plan(m, n, d, k, 8_400_000)
    assert tight.q_chunks > 1
    one = K.knn_plan(m, n, d, k, 10 ** 9)
    assert one.q_chunks == 1 and one.streams == 1
    # two streams: both sets of lists are counted
    two = K.knn_plan(m, n, d, k, 20_000_000)
    assert two.q_chunks > 1 and two.streams == 2
    assert two.lists_bytes == 2 * 2 * ((two.chunk_rows * two.n_splits * k * 4 + 255) // 256 * 256)
    assert two.workspace_bytes == two.norms_bytes + two.query_bytes + two.lists_bytes <= 20_000_000


def test_low_d_falls_back_to_the_vector_path_when_packed_points_do_not_fit():
    m, n, d, k = 100_000, 1_000_000, 3, 16
    roomy = K.knn_plan(m, n, d, k, 10 ** 9)
    assert roomy.path == K.KNN_PATH_LOWD_BF16 and roomy.norms_bytes >= 32 * n
    mid = K.knn_plan(m, n, d, k, 25 * 10 ** 6)  # 16 bytes per point fit, 32 do not
    assert mid.path == K.KNN_PATH_LOWD_MFMA and 16 * n <= mid.norms_bytes < 32 * n
    assert mid.workspace_bytes <= 25 * 10 ** 6
    tight = K.knn_plan(m, n, d, k, 10 ** 7)  # 16 MB of packed points do not fit in 10 MB
    assert tight.path == K.KNN_PATH_LOWD and tight.norms_bytes == 0
    assert tight.workspace_bytes <= 10 ** 7
    # d in 4..8: bf16 filter (32 bytes per point up to d = 4, 64 above) or the vector kernel
    assert K.knn_plan(m, n, 4, k, 10 ** 9).norms_bytes == 256 + 32 * n
    assert K.knn_plan(m, n, 8, k, 10 ** 9).path == K.KNN_PATH_LOWD_BF16
    assert K.knn_plan(m, n, 8, k, 10 ** 9).norms_bytes == 256 + 64 * n
    assert K.knn_plan(m, n, 8, k, 60 * 10 ** 6).path == K.KNN_PATH_LOWD
    assert K.knn_plan(m, n, 9, k, 10 ** 9).path == K.KNN_PATH_MFMA_PACKED  # (one chunk: from 2048 queries)
    assert K.knn_plan(2047, n, 9, k, 10 ** 9).path == K.KNN_PATH_MFMA_SPLIT
    assert K.knn_plan(m, n, 9, k, 30 * 10 ** 6).slab_points < n  # a slab of the copy
    assert K.knn_plan(m, n, 9, k, 12 * 10 ** 6).path == K.KNN_PATH_MFMA_SPLIT  # no room for one
    # the cosine metric: the packed path at any d <= 256 (the whole copy, and n more words), else path 5
    for dc in (9, 3):
        pc = K.knn_plan(m, n, dc, k, 10 ** 9, metric="cosine")
        assert pc.path == K.KNN_PATH_MFMA_PACKED and pc.slab_points == n
        assert pc.norms_bytes == 2 * (4 * n) + 256 + 32 * n
        assert K.knn_plan(m, n, dc, k, 30 * 10 ** 6, metric="cosine").path == K.KNN_PATH_MFMA_SPLIT
        assert K.knn_plan(2047, n, dc, k, 10 ** 9, metric="cosine").path == K.KNN_PATH_MFMA_SPLIT


def test_threshold_seed_grid_is_sized_from_n_and_k_and_paid_for_under_the_limit():
    # path 4, d <= 3: G cells per axis, the largest G with G^d <= min(2 n / (3 k), 32768); the
    # cell starts (G^d + 1 words), the fill cursors (G^d words) and the points in cell order
    # (16 bytes each), 256-aligned each, follow the packed points inside norms_bytes
    def up(v):
        return (v + 255) // 256 * 256

    def seed_bytes(n, cells):
        return up(4 * (cells + 1)) + up(4 * cells) + up(16 * n)

    for n, d, k, G in [(1_000_000, 3, 16, 32), (1_000_000, 2, 16, 181), (750_000, 1, 16, 31250),
                       (10_000_000, 1, 1, 32768), (10_000_000, 3, 1, 32), (10_000_000, 2, 1, 181),
                       (9000, 3, 12, 7), (40_000, 3, 200, 5), (500, 3, 16, 2)]:
        p = K.knn_plan(1000, n, d, k, 10 ** 10)
        assert p.path == K.KNN_PATH_LOWD_BF16 and p.seed_cells == G, (n, d, k, p.seed_cells)
        assert G ** d <= min(2 * n // (3 * k), 32768) < (G + 1) ** d or G ** d <= 32768 < (G + 1) ** d
        assert p.norms_bytes == 256 + up(32 * n) + seed_bytes(n, G ** d)
        assert p.workspace_bytes <= 10 ** 10
    # fewer than two cells per axis, or d > 3: no grid
    assert K.knn_plan(1000, 100, 3, 16, 10 ** 9).seed_cells == 0
    assert K.knn_plan(1000, 1_000_000, 4, 16, 10 ** 9).seed_cells == 0
    # room for the packed points and one tile of lists but not for the grid: same path, no grid
    # (the kernel's private segment, at most 64 bytes per lane x 64 lanes x 16 waves x 256 compute
    # units, counts against the limit as well)
    n, d, k = 1_000_000, 3, 16
    priv = 64 * 64 * 16 * 256
    packed = 256 + 32 * n
    tile_lists = 2 * ((256 * k * 4 + 255) // 256 * 256)
    assert K.knn_plan(1000, n, d, k, packed + priv + tile_lists - 1).path != K.KNN_PATH_LOWD_BF16
    bare = K.knn_plan(1000, n, d, k, packed + priv + tile_lists)
    assert bare.path == K.KNN_PATH_LOWD_BF16 and bare.seed_cells == 0 and bare.norms_bytes == packed
    assert bare.private_bytes == priv and bare.workspace_bytes + priv <= packed + priv + tile_lists
    assert K.knn_plan(1000, n, d, k, packed + priv + tile_lists + seed_bytes(n, 32 ** 3) - 1).seed_cells == 0
    full = K.knn_plan(1000, n, d, k, packed + priv + tile_lists + seed_bytes(n, 32 ** 3))
    assert full.seed_cells == 32
    assert full.workspace_bytes + full.private_bytes <= packed + priv + tile_lists + seed_bytes(n, 32 ** 3)


def test_split_paths_account_for_the_per_query_data_and_use_every_byte_they_can():
    # paths 5 and 6 (d > 8, squared-Euclidean): per query 32 bytes per 16 coordinates of bf16 B
    # operands, a squared norm and a shared-threshold word, each array 256-aligned; the chunk is
    # the longest multiple of the query tile that fits with them.  Path 6 (8 < d <= 256, at least 64 queries - 2048 up to d = 16 -,
    # 65536 points and four times the smallest sample its first thresholds come from) adds the points rounded to bf16, 32 bytes
    # per point and 16 coordinates (the chunk count padded to an even one above 8), and pads the
    # norms to a multiple of 64 points; its query tile is 32 x the query sets of a workgroup.
    import random
    rnd = random.Random(20240611)

    def up(v):
        return (v + 255) // 256 * 256

    seen = set()
    for _ in range(400):
        d = rnd.choice([9, 16, 17, 100, 128, 129, 144, 256, 784, 2000])
        k = rnd.choice([1, 7, 32, 100, 1024])
        n = rnd.randrange(k, 3_000_000)
        m = rnd.choice([1, 255, 256, 257, 5000, 123_457])
        lo = K.knn_plan(m, n, d, k, 1 << 44).min_limit_bytes
        limit = lo + rnd.choice([0, 1, 255, 256, 4096, 10 ** 6, 10 ** 8, 10 ** 10])
        p = K.knn_plan(m, n, d, k, limit)
        nch = (d + 15) // 16
        seen.add(p.path)
        if p.path == K.KNN_PATH_MFMA_PACKED:
            seed_min = (max(8192, 8 * k) + 63) // 64 * 64
            seed = max(seed_min, min(160 * k, 65536, n // 4) // 64 * 64)
            assert 8 < d <= 256 and m >= (2048 if d <= 16 else 64) and n >= 65536 and n >= 4 * seed_min and p.seed_points == seed
            nch_p = nch if nch <= 8 else (nch + 1) // 2 * 2
            # three waves per SIMD where their registers allow and their merge scratch takes at most half the LDS
            waves = 12 if nch_p <= 8 and 12 * (128 + 2 * k) * 4 <= 80 * 1024 else 8
            n64 = (n + 63) // 64 * 64
            # the copy holds all points, or a slab of them (a multiple of 8192 points, at least 65536)
            assert p.slab_points == n64 or (p.slab_points % 8192 == 0 and 131072 <= p.slab_points < n64 and p.q_chunks == 1)
            assert p.norms_bytes == up(4 * n64) + 256 + up(p.slab_points * nch_p * 32)
            assert p.tile_q % 32 == 0 and 64 <= p.tile_q <= 512 and p.tile_x == 64
            # the workgroup's LDS: B operands, candidate buffers and state, merge scratch, control
            sets = p.tile_q // 32
            assert sets * nch_p * 1024 + sets * 32 * (32 * 4 + 28) + waves * (128 + 2 * k) * 4 + waves * 256 + 256 \
                <= 160 * 1024
        elif p.path == K.KNN_PATH_MFMA_WIDE:
            # d > 256, k <= 512: the copy as on path 6, tiles of 512 queries x 128 points, at most 64
            # ranges; the queries' B operands in operand order (rows rounded up to 64, chunk count
            # to an even one)
            assert d > 256 and k <= 512 and m >= 16 and n >= 65536 and p.seed_points == 0
            nch_p = (nch + 1) // 2 * 2
            n64 = (n + 63) // 64 * 64
            assert p.slab_points == n64 or (p.slab_points % 8192 == 0 and 131072 <= p.slab_points < n64 and p.q_chunks == 1)
            assert p.norms_bytes == up(4 * n64) + 256 + up(p.slab_points * nch_p * 32)
            assert p.tile_q == 512 and p.tile_x == 128 and 1 <= p.n_splits <= 64
            # the workgroup's LDS: stage buffers, norms, candidate buffers, state, control, merge scratch
            assert 16384 + 1024 + 512 * 32 * 4 + 7 * 512 * 4 + 64 + 8 * (128 + 2 * k) * 4 <= 160 * 1024
        else:
            assert p.path == K.KNN_PATH_MFMA_SPLIT and p.tile_q == 256
            assert p.norms_bytes == up(4 * n) + 256
        tile = p.tile_q
        wide = p.path == K.KNN_PATH_MFMA_WIDE

        def operand_bytes(rows):
            return up((rows + 63) // 64 * 64 * ((nch + 1) // 2 * 2) * 32) if wide else up(rows * nch * 32)

        # paths 6 and 7 also keep one word per query and point range (the ranges bound each other)
        ranged = p.path in (K.KNN_PATH_MFMA_PACKED, K.KNN_PATH_MFMA_WIDE)
        per_range = up(p.chunk_rows * p.n_splits * 4) if ranged else 0
        assert p.query_bytes == operand_bytes(p.chunk_rows) + 2 * up(p.chunk_rows * 4) + per_range
        assert p.lists_bytes == p.streams * 2 * up(p.chunk_rows * p.n_splits * k * 4)
        assert p.streams == 1 or p.q_chunks > 1
        assert p.workspace_bytes == p.norms_bytes + p.query_bytes + p.lists_bytes <= limit
        assert p.chunk_rows == m or p.chunk_rows % tile == 0
        assert p.q_chunks == -(-m // p.chunk_rows)
        if p.chunk_rows < m and p.chunk_rows < (1 << 22):  # a longer chunk would not have fitted
            r = p.chunk_rows + tile
            more = operand_bytes(r) + 2 * up(r * 4) + p.streams * 2 * up(r * p.n_splits * k * 4) + \
                (up(r * p.n_splits * 4) if ranged else 0)
            assert p.norms_bytes + more > limit
        with pytest.raises(K.KnnError):
            K.knn_plan(m, n, d, k, lo - 1)
    assert seen == {K.KNN_PATH_MFMA_SPLIT, K.KNN_PATH_MFMA_PACKED, K.KNN_PATH_MFMA_WIDE}


def test_l1_path_accounts_for_the_transposed_queries():
    # L1 metric, any d: besides the lists a chunk holds its queries transposed in blocks of 64
    # rows, 16 bytes per row and 4 coordinates; nothing per point
    import random
    rnd = random.Random(20240612)

    def up(v):
        return (v + 255) // 256 * 256

    def qbytes(rows, d):
        return up(-(-rows // 64) * 64 * -(-d // 4) * 16)

    for _ in range(300):
        d = rnd.choice([1, 3, 4, 5, 16, 17, 100, 128, 784, 2001])
        k = rnd.choice([1, 7, 32, 100, 1024])
        n = rnd.randrange(k, 3_000_000)
        m = rnd.choice([1, 63, 64, 65, 255, 256, 257, 5000, 123_457])
        lo = K.knn_plan(m, n, d, k, 1 << 44, metric="l1").min_limit_bytes
        limit = lo + rnd.choice([0, 1, 255, 256, 4096, 10 ** 6, 10 ** 8, 10 ** 10])
        p = K.knn_plan(m, n, d, k, limit, metric="l1")
        assert p.path == K.KNN_PATH_L1 and p.tile_q == 256
        assert p.norms_bytes == 0
        assert p.query_bytes == qbytes(p.chunk_rows, d)
        assert p.lists_bytes == p.streams * 2 * up(p.chunk_rows * p.n_splits * k * 4)
        assert p.workspace_bytes == p.query_bytes + p.lists_bytes <= limit
        assert p.chunk_rows == m or p.chunk_rows % 256 == 0
        assert p.q_chunks == -(-m // p.chunk_rows)
        if p.chunk_rows < m and p.chunk_rows < (1 << 22):  # a longer chunk would not have fitted
            r = p.chunk_rows + 256
            assert qbytes(r, d) + p.streams * 2 * up(r * p.n_splits * k * 4) > limit
        with pytest.raises(K.KnnError):
            K.knn_plan(m, n, d, k, lo - 1, metric="l1")


def test_plan_argument_errors():
    bad = [(-1, 10, 3, 1), (5, 0, 3, 1), (5, 10, 0, 1), (5, 10, 3, 0), (5, 10, 3, 11)]
    for m, n, d, k in bad:
        with pytest.raises(K.KnnError) as ei:
            K.knn_plan(m, n, d, k, 10 ** 9)
        assert ei.value.status == K.KNN_ERR_INVALID_ARG
    with pytest.raises(K.KnnError) as ei:
        K.knn_plan(5, 1 << 31, 3, 1, 10 ** 12)
    assert ei.value.status == K.KNN_ERR_UNSUPPORTED
    with pytest.raises(K.KnnError) as ei:
        K.knn_plan(5, (1 << 31) - 65535, 3, 1, 10 ** 12)
    assert ei.value.status == K.KNN_ERR_UNSUPPORTED
    assert K.knn_plan(5, (1 << 31) - 65536, 3, 1, 10 ** 12).n == (1 << 31) - 65536
    with pytest.raises(K.KnnError) as ei:
        K.knn_plan(5, 5000, 3, K.KNN_MAX_K + 1, 10 ** 12)
    assert ei.value.status == K.KNN_ERR_UNSUPPORTED
    p = K.knn_plan(0, 10, 3, 2, 0)  # no queries: empty plan, nothing needed
    assert p.q_chunks == 0 and p.workspace_bytes == 0


def test_status_strings_are_distinct():
    texts = {K.knn_status_string(s) for s in range(6)}
    assert len(texts) == 6


def test_host_entry_points_reject_bad_arguments_without_a_gpu():
    # knn_search validates before it touches HIP: these return synchronously on any machine
    st = K.knn_search_raw(0, 3, 0, 3, 5, 10, 3, 11, 10 ** 9, 0, 0, 0, 0, 0)  # k > n
    assert st == K.KNN_ERR_INVALID_ARG
    st = K.knn_search_raw(0, 3, 0, 3, 5, 10, 3, 2, 10 ** 9, 0, 0, 0, 0, 0)  # null X
    assert st == K.KNN_ERR_INVALID_ARG
    st = K.knn_search_raw(256, 2, 256, 3, 5, 10, 3, 2, 10 ** 9, 256, 1 << 20, 256, 256, 0)  # ldq < d
    assert st == K.KNN_ERR_INVALID_ARG
    st = K.knn_search_raw(256, 3, 256, 3, 5, 10, 3, 2, 16, 256, 1 << 20, 256, 256, 0)  # limit too small
    assert st == K.KNN_ERR_MEM_LIMIT_TOO_SMALL
    st = K.knn_search_raw(256, 3, 256, 3, 5, 10, 3, 2, 10 ** 9, 256, 8, 256, 256, 0)  # workspace too small
    assert st == K.KNN_ERR_WORKSPACE_TOO_SMALL
    st = K.knn_search_raw(256, 3, 256, 3, 5, 10, 3, 2, 10 ** 9, 257, 1 << 20, 256, 256, 0)  # misaligned ws
    assert st == K.KNN_ERR_INVALID_ARG
    st = K.knn_search_raw(0, 3, 256, 3, 0, 10, 3, 2, 0, 0, 0, 0, 0, 0)  # m == 0: nothing to do
    assert st == K.KNN_OK
