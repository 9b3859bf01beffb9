"""CPU-only tests of sgpr_plan (include/sgpr.h): host arithmetic, no GPU call."""
import pytest

import paper_2206_14148_amd as K
import workloads as W


def up(v):
    return (v + 255) // 256 * 256


def test_chunk_is_what_the_limit_holds_capped_at_4096_columns():
    p = K.sgpr_plan(10_000, 434_874, 3, W.GB)
    assert (p.chunk_cols, p.chunk_ld, p.col_groups) == (4096, 4096, 1)
    assert p.n_chunks == -(-434_874 // 4096)
    assert p.workspace_bytes == up(10_000 * 4096 * 4) <= W.GB
    # a limit that holds 1000 columns of m fp32 values: chunks of 992 (multiple of 16)
    p = K.sgpr_plan(10_000, 434_874, 3, 10_000 * 4 * 1000)
    assert p.chunk_cols == 992 and p.workspace_bytes <= 10_000 * 4 * 1000
    assert p.min_limit_bytes == up(10_000 * 16 * 4)
    assert K.sgpr_plan(10_000, 434_874, 3, p.min_limit_bytes).chunk_cols == 16
    with pytest.raises(K.KnnError) as ei:
        K.sgpr_plan(10_000, 434_874, 3, p.min_limit_bytes - 1)
    assert ei.value.status == K.KNN_ERR_MEM_LIMIT_TOO_SMALL and ei.value.min_limit_bytes == p.min_limit_bytes


def test_few_tiles_buy_column_groups_when_the_limit_has_room():
    m, n = 4000, 2_049_280
    roomy = K.sgpr_plan(m, n, 11, W.GB)
    assert roomy.col_groups == 4  # 528 tiles x 4 groups >= 2048 workgroups
    assert roomy.workspace_bytes == up(m * 4096 * 4) + 3 * up(m * m * 8) <= W.GB
    tight = K.sgpr_plan(m, n, 11, 100 * W.MB)  # the chunk fits, a copy of A (128 MB) does not
    assert tight.col_groups == 1 and tight.workspace_bytes <= 100 * W.MB
    two = K.sgpr_plan(m, n, 11, up(m * 4096 * 4) + up(m * m * 8))
    assert two.col_groups == 2
    # a group keeps at least 256 columns
    assert K.sgpr_plan(300, 5000, 3, 300 * 4 * 512).col_groups == 1


def test_small_and_empty_data_and_errors():
    p = K.sgpr_plan(50, 10, 2, W.MB)
    assert (p.chunk_cols, p.chunk_ld, p.n_chunks) == (10, 16, 1)
    p = K.sgpr_plan(50, 0, 2, W.MB)
    assert p.n_chunks == 0
    for bad in ((0, 10, 2), (5, -1, 2), (5, 10, 0)):
        with pytest.raises(K.KnnError) as ei:
            K.sgpr_plan(*bad, W.MB)
        assert ei.value.status == K.KNN_ERR_INVALID_ARG
    with pytest.raises(K.KnnError) as ei:
        K.sgpr_plan((1 << 17) + 1, 10, 2, 10 ** 12)
    assert ei.value.status == K.KNN_ERR_UNSUPPORTED
