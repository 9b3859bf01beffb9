"""The entry point that allocates nothing, knn_search_static, against knn_search: same kernels,
the workspace in the library's static device buffer instead of the caller's.  Two calls in a row
on the same GPU, the second with a smaller input, each compared bit for bit with knn_search."""
import ctypes

import numpy as np
import pytest

import paper_2206_14148_amd as K
import workloads as W

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu


def _run_pair(m, n, d, k, seed):
    rng = np.random.default_rng(seed)
    X = torch.from_numpy(rng.standard_normal((n, d), dtype=np.float32)).to("cuda:0")
    Q = torch.from_numpy(rng.standard_normal((m, d), dtype=np.float32)).to("cuda:0")
    ref_idx, ref_dist = K.knn_search(Q, X, k, K.KNN_STATIC_SCRATCH_BYTES)
    torch.cuda.synchronize()
    # outputs are the caller's; poisoned so that an entry point that wrote nothing would show
    idx = torch.full((m, k), -7, dtype=torch.int32, device="cuda:0")
    dist = torch.full((m, k), float("nan"), dtype=torch.float32, device="cuda:0")
    stream = torch.cuda.current_stream().cuda_stream
    st = K.load().knn_search_static(Q.data_ptr(), Q.stride(0), X.data_ptr(), X.stride(0), m, n, d, k,
                                    idx.data_ptr(), dist.data_ptr(), stream)
    assert st == K.KNN_OK, K.knn_status_string(st)
    torch.cuda.synchronize()
    assert torch.equal(idx, ref_idx)
    assert torch.equal(dist.view(torch.int32), ref_dist.view(torch.int32))
    plan, peak = K.knn_last_stats()
    assert 0 < peak <= K.KNN_STATIC_SCRATCH_BYTES
    return plan


def test_static_scratch_matches_knn_search_twice_second_smaller():
    # matrix-core path, several point ranges; then a smaller input that leaves most of the buffer
    # holding the first call's lists and norms
    p1 = _run_pair(1500, 40000, 48, 24, 1)
    p2 = _run_pair(300, 9000, 48, 10, 2)
    assert p1.path == K.KNN_PATH_MFMA_SPLIT and p2.path == K.KNN_PATH_MFMA_SPLIT
    # the low-d path with its grid of counters, twice as well
    _run_pair(5000, 60000, 3, 16, 3)
    _run_pair(700, 8000, 3, 5, 4)


def test_static_scratch_rejects_what_does_not_fit():
    lib = K.load()
    n = 20_000_000  # 4 n bytes of norms alone exceed the buffer; nothing is dereferenced
    one = torch.zeros(16, dtype=torch.float32, device="cuda:0")
    out_i = torch.full((1, 1), -7, dtype=torch.int32, device="cuda:0")
    out_d = torch.zeros((1, 1), dtype=torch.float32, device="cuda:0")
    st = lib.knn_search_static(one.data_ptr(), 16, one.data_ptr(), 16, 1, n, 16, 1,
                               out_i.data_ptr(), out_d.data_ptr(), None)
    assert st == K.KNN_ERR_STATIC_SCRATCH_TOO_SMALL
    assert "static scratch" in K.knn_status_string(st)
    torch.cuda.synchronize()
    assert int(out_i[0, 0]) == -7
