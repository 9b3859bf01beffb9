"""GPU parity tests of the SGPR accumulations (paper section 5.3): A = K_uf K_fu and b = K_uf y
from the HIP path, called through the C ABI, against the fp64 CPU oracle.

Tolerance (eps = 2^-24): a K_uf entry with exponent -a has relative error <= a (d+4) eps + 2 eps
(fp32 difference-form distance, hardware exp2, one multiply by the variance); a product of two
of them twice that; a sum of C products in fp32 on the matrix cores at most C eps of the sum,
C = the chunk length; sums over chunks are fp64.  All terms of an entry of A are positive, so
  |A_ij - oracle| <= A_ij (1e-5 + (d+4) eps (a_i + a_j)_max + C eps) + tiny,
with the exponents bounded through the largest squared distance of the case, and
  |b_i - oracle|  <= sum_t |K_it y_t| (1e-5 + (d+4) eps a_max) + tiny   (64-lane fp64 sums).
"""
import sys

import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

EPS = 2.0 ** -24


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def K():
    import paper_2206_14148_amd as K
    assert torch.cuda.is_available(), "these tests need the GPU"
    K.load()
    return K


def a_max(U, X, lengthscale):
    """Largest exponent magnitude of the case, from the bounding boxes of U and X."""
    lo = np.minimum(U.min(0), X.min(0)).astype(np.float64)
    hi = np.maximum(U.max(0), X.max(0)).astype(np.float64)
    return 0.5 * ((hi - lo) ** 2).sum() / lengthscale ** 2


def run_gpu(K, U, X, y, variance, lengthscale, limit):
    A, b = K.sgpr_accumulate(torch.from_numpy(U).cuda(), torch.from_numpy(X).cuda(),
                             torch.from_numpy(y).cuda(), variance, lengthscale, limit)
    torch.cuda.synchronize()
    return A.cpu().numpy(), b.cpu().numpy()


def parity(K, oracle, U, X, y, variance, lengthscale, limit=64 * W.MB):
    m, d = U.shape
    plan = K.sgpr_plan(m, X.shape[0], d, limit)
    assert plan.workspace_bytes <= limit
    A, b = run_gpu(K, U, X, y, variance, lengthscale, limit)
    assert A.shape == (m, m) and b.shape == (m,) and np.isfinite(A).all() and np.isfinite(b).all()
    assert np.array_equal(A, A.T)
    rA, rb = oracle.sgpr_accumulate(U, X, y, variance, lengthscale)
    am = a_max(U, X, lengthscale)
    tolA = rA * (1e-5 + 2 * (d + 4) * EPS * am + plan.chunk_cols * EPS) + 1e-36 * variance ** 2 * X.shape[0]
    mag = oracle.kmv(U, X, np.abs(y), variance, lengthscale)
    tolb = mag * (1e-5 + (d + 4) * EPS * am) + 1e-37 * variance * np.abs(y).sum()
    eA, eb = np.abs(A - rA), np.abs(b - rb)
    say(f"   sgpr parity m={m} n={X.shape[0]} chunks={plan.n_chunks}x{plan.chunk_cols}: "
        f"max errA/tol={float((eA / tolA).max()):.3g} rel={float((eA / np.maximum(rA, 1e-300)).max()):.3g} "
        f"max errb/tol={float((eb / tolb).max()):.3g}")
    assert (eA <= tolA).all() and (eb <= tolb).all()
    return A, b


# (seed, m, n, d, variance, lengthscale, limit)
SMALL = [
    (0, 1, 1, 1, 1.0, 1.0, 64 * W.MB),          # smallest possible call
    (1, 5, 100, 1, 1.0, 1.0, 64 * W.MB),
    (2, 128, 16, 2, 2.5, 0.7, 64 * W.MB),       # one tile, one K step
    (3, 129, 777, 3, 0.3, 1.5, 64 * W.MB),      # ragged tile pair, ragged columns
    (4, 300, 5003, 11, 1.0, 3.0, 64 * W.MB),    # two chunks of 4096 / 907 columns, six tile pairs
    (5, 257, 1000, 4, 1.0, 2.0, 257 * 64 + 255),  # the smallest limit: chunks of 16 columns
    (6, 200, 3000, 3, 1.7, 1.0, 200 * 4 * 100),   # chunks of 96 columns
    (7, 513, 2048, 2, 1.0, 1.0, 64 * W.MB),     # 15 tile pairs
]


@pytest.mark.parametrize("case", SMALL, ids=lambda c: "s%d_m%d_n%d_d%d" % c[:4])
def test_small_cases_match_oracle(K, oracle, case):
    seed, m, n, d, variance, lengthscale, limit = case
    say("case", case)
    U, X, y = W.random_sgpr_case(seed, m, n, d)
    parity(K, oracle, U, X, y, variance, lengthscale, limit)


def test_inducing_points_among_the_data(K, oracle):
    # the usual initialisation: U = first m data points, so K_uf has exact ones (times variance)
    _, X, y = W.random_sgpr_case(20, 1, 2500, 3)
    parity(K, oracle, X[:150].copy(), X, y, 1.2, 0.9)


def test_limits_give_the_same_sums_up_to_rounding(K, oracle):
    U, X, y = W.random_sgpr_case(21, 260, 6000, 3)
    A1, b1 = parity(K, oracle, U, X, y, 1.0, 1.0, 64 * W.MB)
    A2, b2 = parity(K, oracle, U, X, y, 1.0, 1.0, 260 * 4 * 512)   # chunks of 512 columns
    assert np.allclose(A1, A2, rtol=1e-4) and np.allclose(b1, b2, rtol=1e-4, atol=1e-4)
    A3, b3 = run_gpu(K, U, X, y, 1.0, 1.0, 64 * W.MB)
    assert np.array_equal(A1, A3) and np.array_equal(b1, b3)   # a fixed order of summation


def test_strides_guard_bytes_and_empty_data(K, oracle):
    U, X, y = W.random_sgpr_case(22, 140, 1500, 5)
    m, d = U.shape
    Uw = torch.full((m, d + 3), 9.0, device="cuda")
    Xw = torch.full((1500, d + 1), -9.0, device="cuda")
    Uw[:, :d] = torch.from_numpy(U).cuda()
    Xw[:, :d] = torch.from_numpy(X).cuda()
    plan = K.sgpr_plan(m, 1500, d, 64 * W.MB)
    buf = torch.full((plan.workspace_bytes + 4096,), 0xA5, dtype=torch.uint8, device="cuda")
    Abig = torch.full((m, m + 7), 5.0, dtype=torch.float64, device="cuda")
    b = torch.empty(m, dtype=torch.float64, device="cuda")
    K.sgpr_accumulate(Uw[:, :d], Xw[:, :d], torch.from_numpy(y).cuda(), 1.0, 2.0, 64 * W.MB,
                      workspace=buf[:plan.workspace_bytes], out=(Abig[:, :m], b))
    torch.cuda.synchronize()
    assert (buf[plan.workspace_bytes:] == 0xA5).all()
    assert (Abig[:, m:] == 5.0).all()
    rA, rb = oracle.sgpr_accumulate(U, X, y, 1.0, 2.0)
    assert np.allclose(Abig[:, :m].cpu().numpy(), rA, rtol=1e-4)
    assert np.allclose(b.cpu().numpy(), rb, rtol=1e-4, atol=1e-4)
    A0, b0 = K.sgpr_accumulate(torch.from_numpy(U).cuda(), torch.empty((0, d), device="cuda"),
                               torch.empty((0,), device="cuda"), 1.0, 2.0, 64 * W.MB)
    torch.cuda.synchronize()
    assert (A0 == 0).all() and (b0 == 0).all()


def test_errors(K):
    U, X, y = (torch.from_numpy(a).cuda() for a in W.random_sgpr_case(23, 100, 500, 3))
    with pytest.raises(K.KnnError) as ei:
        K.sgpr_accumulate(U, X, y, 1.0, 1.0, 100 * 64 - 1)
    assert ei.value.status == K.KNN_ERR_MEM_LIMIT_TOO_SMALL and ei.value.min_limit_bytes == 6400
    with pytest.raises(K.KnnError) as ei:
        K.sgpr_accumulate(U, X, y, 1.0, 0.0, W.MB)
    assert ei.value.status == K.KNN_ERR_INVALID_ARG
    with pytest.raises(K.KnnError) as ei:
        K.sgpr_accumulate(U, X, y[:-1], 1.0, 1.0, W.MB)
    assert ei.value.status == K.KNN_ERR_INVALID_ARG
    plan = K.sgpr_plan(100, 500, 3, W.MB)
    with pytest.raises(K.KnnError) as ei:
        K.sgpr_accumulate(U, X, y, 1.0, 1.0, W.MB,
                          workspace=torch.empty(plan.workspace_bytes - 256, dtype=torch.uint8, device="cuda"))
    assert ei.value.status == K.KNN_ERR_WORKSPACE_TOO_SMALL


@pytest.mark.parametrize("key", ["sgpr1", "sgpr2"])
def test_full_size_sampled_entries(K, oracle, key):
    # the benchmark's launch configuration; sampled entries of A and b against the oracle
    w = W.SGPR_WORKLOADS[key]
    say("full size", w)
    U, X, y = W.make_sgpr(w)
    A, b = K.sgpr_accumulate(torch.from_numpy(U).cuda(), torch.from_numpy(X).cuda(),
                             torch.from_numpy(y).cuda(), w.variance, w.lengthscale, w.mem_limit)
    torch.cuda.synchronize()
    g = np.random.Generator(np.random.PCG64(8))
    ii = np.concatenate([g.integers(0, w.m, 40), [0, w.m - 1, w.m - 1, 127, 128]])
    jj = np.concatenate([g.integers(0, w.m, 40), [0, w.m - 1, 0, 128, 127]])
    ref = oracle.sgpr_entries(U, X, ii, jj, w.variance, w.lengthscale)
    got = A[torch.from_numpy(ii).cuda(), torch.from_numpy(jj).cuda()].cpu().numpy()
    got_t = A[torch.from_numpy(jj).cuda(), torch.from_numpy(ii).cuda()].cpu().numpy()
    rel = np.abs(got - ref) / ref
    say(f"   sampled entries: max rel err {rel.max():.3g}")
    plan = K.sgpr_plan(w.m, w.n, w.d, w.mem_limit)
    assert (rel <= 1e-5 + 2 * (w.d + 4) * EPS * a_max(U, X, w.lengthscale) + plan.chunk_cols * EPS).all()
    assert np.array_equal(got, got_t)
    rows = np.sort(g.choice(w.m, 16, replace=False))
    rb = oracle.kmv(U, X, y, w.variance, w.lengthscale, rows=rows)
    mag = oracle.kmv(U, X, np.abs(y), w.variance, w.lengthscale, rows=rows)
    assert (np.abs(b.cpu().numpy()[rows] - rb) <= 2e-5 * mag).all()
