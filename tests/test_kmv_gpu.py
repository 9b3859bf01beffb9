"""GPU parity tests of the kernel matrix-vector product (paper section 5.1): the HIP path,
called through the C ABI, against the fp64 CPU oracle.

Tolerance (derived from the kernels' arithmetic, eps = 2^-24):
  low-d path    the fp32 squared distance has relative error <= (d+2) eps, the scaled exponent
                (d+4) eps, so a kernel entry with exponent -a has relative error
                <= a (d+4) eps + 2 eps (hardware exp2: 1 ulp); a 64-term fp32 sum adds at most
                64 eps of the sum of magnitudes.
  matrix-core   the exponent comes from the expansion of section 4.1, so its ABSOLUTE error is
                <= (d+4) eps c (|x_i| + |z_j|)^2 with c = 1 / (2 l^2).
Hence  |y_i - oracle_i| <= sum_j |K_ij v_j| * (4e-6 + (d+4) eps * e_ij),  e_ij = a_ij or
c (|x_i|+|z_j|)^2, plus 1e-37 * variance * sum|v| for entries below the smallest normal fp32.

The all-fp64 entry point does what the oracle does in the same precision with other roundings
(fused multiply-adds, another exp): with eps = 2^-53 an entry differs by <= a (d+4) eps + 2 eps
relative on each side and a running sum of m terms by <= m eps of the sum of magnitudes on each
side:  |y_i - oracle_i| <= 2 sum_j |K_ij v_j| * ((m + 8) eps + (d+4) eps a_ij).
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


def tolerance(X, Z, v, variance, lengthscale, rows, mfma):
    """Per-row bound from the docstring, evaluated pair by pair in fp64 (rows: row subset)."""
    Xr = X[rows].astype(np.float64)
    Zd = Z.astype(np.float64)
    d = X.shape[1]
    tol = np.empty(len(rows))
    c = 0.5 / lengthscale ** 2
    zn = np.sqrt((Zd * Zd).sum(1))
    for t in range(len(rows)):
        a = c * ((Xr[t][None, :] - Zd) ** 2).sum(1)
        mag = variance * np.exp(-a) * np.abs(v)
        e = c * (np.sqrt((Xr[t] * Xr[t]).sum()) + zn) ** 2 if mfma else a
        tol[t] = (mag * (4e-6 + (d + 4) * EPS * e)).sum() + 1e-37 * variance * np.abs(v).sum()
    return tol


def run_gpu(K, X, Z, v, variance, lengthscale, limit, z_is_x=False):
    Xd = torch.from_numpy(X).cuda()
    Zd = Xd if z_is_x else torch.from_numpy(Z).cuda()
    vd = torch.from_numpy(v).cuda()
    y = K.kmv_apply(Xd, Zd, vd, variance, lengthscale, limit)
    torch.cuda.synchronize()
    return y.cpu().numpy()


def parity(K, oracle, X, Z, v, variance, lengthscale, limit=64 * W.MB, rows=None, z_is_x=False):
    y = run_gpu(K, X, Z, v, variance, lengthscale, limit, z_is_x)
    assert y.shape == (X.shape[0],) and y.dtype == np.float64
    assert np.isfinite(y).all()
    sel = np.arange(X.shape[0]) if rows is None else np.asarray(rows)
    ref = oracle.kmv(X, Z, v, variance, lengthscale, rows=None if rows is None else sel)
    tol = tolerance(X, Z, v, variance, lengthscale, sel, X.shape[1] > 8)
    err = np.abs(y[sel] - ref)
    worst = float((err / np.maximum(tol, 1e-300)).max()) if len(sel) else 0.0
    say(f"   kmv parity rows={len(sel)} max err/tol={worst:.3g} max|err|={err.max() if len(sel) else 0:.3g}")
    assert (err <= tol).all(), f"worst err/tol {worst}"
    return y


# (seed, n, m, d, variance, lengthscale, spread)
SMALL = [
    (0, 1, 1, 1, 1.0, 1.0, 1.0),        # smallest possible call
    (1, 700, 1513, 1, 1.0, 1.0, 1.0),   # the appendix case (1-D inputs), ragged both ways
    (2, 257, 64, 2, 2.5, 0.7, 1.0),     # exactly one group of points
    (3, 256, 63, 3, 0.3, 1.5, 1.0),     # tail only
    (4, 513, 1000, 4, 1.0, 2.0, 1.0),
    (5, 300, 777, 5, 1.0, 2.0, 1.0),
    (6, 300, 777, 6, 1.0, 2.5, 1.0),
    (7, 300, 777, 7, 1.0, 2.5, 1.0),
    (8, 300, 777, 8, 1.0, 3.0, 1.0),
    (9, 300, 1000, 9, 1.0, 3.0, 1.0),     # first matrix-core dimension, unaligned rows
    (10, 129, 128, 16, 1.0, 4.0, 1.0),    # one K chunk, one tile of points, ragged rows
    (11, 260, 1111, 20, 1.7, 4.0, 1.0),   # aligned, d not a multiple of the K chunk
    (12, 260, 1111, 33, 1.0, 6.0, 1.0),   # unaligned
    (13, 140, 700, 300, 1.0, 17.0, 1.0),  # many K chunks
    (14, 500, 900, 3, 1.0, 0.05, 1.0),    # short lengthscale: almost all entries underflow
    (15, 500, 900, 12, 1.0, 100.0, 1.0),  # long lengthscale: K close to all ones
    (16, 400, 800, 2, 1.0, 1.0, 30.0),    # large coordinates
    (17, 400, 800, 24, 1.0, 40.0, 10.0),  # large coordinates on the expansion path
    (18, 200, 900, 48, 1.0, 7.0, 1.0),    # three K chunks of rows kept in registers, aligned
    (19, 200, 900, 64, 1.0, 8.0, 1.0),    # four: the last dimension with resident rows
    (20, 130, 500, 65, 1.0, 8.0, 1.0),    # first dimension whose rows stream through LDS
    (21, 150, 700, 100, 1.0, 10.0, 1.0),  # streamed rows, odd number of chunks, aligned
]


@pytest.mark.parametrize("case", SMALL, ids=lambda c: "s%d_n%d_m%d_d%d" % c[:4])
def test_small_cases_match_oracle(K, oracle, case):
    seed, n, m, d, variance, lengthscale, spread = case
    say("case", case)
    X, Z, v = W.random_kmv_case(seed, n, m, d, spread)
    parity(K, oracle, X, Z, v, variance, lengthscale)


@pytest.mark.parametrize("d", [2, 16])
def test_point_ranges_and_limit(K, oracle, d):
    # few rows, many points: the point axis is cut into ranges; a tight limit forbids that
    n, m = 300, 40000
    say("ranges d", d)
    X, Z, v = W.random_kmv_case(30 + d, n, m, d)
    ls = 1.0 if d == 2 else 4.0
    roomy = K.kmv_plan(n, m, d, 64 * W.MB)
    assert roomy.n_splits > 1 and roomy.workspace_bytes <= 64 * W.MB
    tight_limit = roomy.norms_bytes + 8 * n  # no room for two ranges of partial sums
    tight = K.kmv_plan(n, m, d, tight_limit)
    assert tight.n_splits == 1 and tight.workspace_bytes <= tight_limit
    y1 = parity(K, oracle, X, Z, v, 1.0, ls, limit=64 * W.MB)
    y2 = parity(K, oracle, X, Z, v, 1.0, ls, limit=tight_limit)
    assert np.allclose(y1, y2, rtol=1e-4, atol=1e-4)


def test_square_kernel_matrix_is_symmetric_in_use(K, oracle):
    # Z aliases X (the n x n matrix of section 5.1): u.(K v) == v.(K u)
    X, _, v = W.random_kmv_case(40, 900, 900, 3)
    u = W.random_kmv_case(41, 1, 900, 1)[2]
    yv = parity(K, oracle, X, X, v, 1.3, 0.8, z_is_x=True)
    yu = parity(K, oracle, X, X, u, 1.3, 0.8, z_is_x=True)
    lhs, rhs = float(u.astype(np.float64) @ yv), float(v.astype(np.float64) @ yu)
    assert abs(lhs - rhs) <= 1e-5 * (np.abs(u) @ np.abs(yv) + np.abs(v) @ np.abs(yu))


def test_tiny_lengthscale_gives_variance_times_v(K):
    X, _, v = W.random_kmv_case(42, 600, 600, 2)
    y = run_gpu(K, X, X, v, 2.0, 1e-4, 64 * W.MB, z_is_x=True)
    assert np.allclose(y, 2.0 * v.astype(np.float64), rtol=1e-6, atol=1e-30)


def test_zero_variance_and_empty_sides(K):
    X, Z, v = W.random_kmv_case(43, 300, 500, 3)
    assert (run_gpu(K, X, Z, v, 0.0, 1.0, 64 * W.MB) == 0).all()
    Xd = torch.from_numpy(X).cuda()
    y = K.kmv_apply(Xd, torch.empty((0, 3), device="cuda"), torch.empty((0,), device="cuda"),
                    1.0, 1.0, 64 * W.MB, out=torch.full((300,), 7.0, dtype=torch.float64, device="cuda"))
    torch.cuda.synchronize()
    assert (y.cpu().numpy() == 0).all()
    y = K.kmv_apply(torch.empty((0, 3), device="cuda"), Xd, torch.zeros(300, device="cuda"),
                    1.0, 1.0, 64 * W.MB)
    torch.cuda.synchronize()
    assert y.shape == (0,)


@pytest.mark.parametrize("d", [3, 20])
def test_strided_rows_and_determinism(K, oracle, d):
    n, m = 333, 2222
    X, Z, v = W.random_kmv_case(50 + d, n, m, d)
    Xw = torch.full((n, d + 5), 99.0, device="cuda")
    Zw = torch.full((m, d + 3), -99.0, device="cuda")
    Xw[:, :d] = torch.from_numpy(X).cuda()
    Zw[:, :d] = torch.from_numpy(Z).cuda()
    vd = torch.from_numpy(v).cuda()
    ls = 1.0 if d == 3 else 4.0
    y1 = K.kmv_apply(Xw[:, :d], Zw[:, :d], vd, 1.0, ls, 64 * W.MB)
    y2 = K.kmv_apply(Xw[:, :d], Zw[:, :d], vd, 1.0, ls, 64 * W.MB)
    y3 = K.kmv_apply(torch.from_numpy(X).cuda(), torch.from_numpy(Z).cuda(), vd, 1.0, ls, 64 * W.MB)
    torch.cuda.synchronize()
    assert torch.equal(y1, y2)
    ref = oracle.kmv(X, Z, v, 1.0, ls)
    tol = tolerance(X, Z, v, 1.0, ls, np.arange(n), d > 8)
    assert (np.abs(y1.cpu().numpy() - ref) <= tol).all()
    assert (np.abs(y3.cpu().numpy() - ref) <= tol).all()


def test_workspace_stays_inside_its_bytes(K):
    n, m, d = 300, 40000, 16
    X, Z, v = W.random_kmv_case(60, n, m, d)
    plan = K.kmv_plan(n, m, d, 64 * W.MB)
    assert plan.n_splits > 1
    guard = 4096
    buf = torch.full((plan.workspace_bytes + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    K.kmv_apply(torch.from_numpy(X).cuda(), torch.from_numpy(Z).cuda(), torch.from_numpy(v).cuda(),
                1.0, 4.0, 64 * W.MB, workspace=buf[:plan.workspace_bytes])
    torch.cuda.synchronize()
    assert (buf[plan.workspace_bytes:] == 0xA5).all()


def test_errors(K):
    X, Z, v = W.random_kmv_case(61, 100, 5000, 16)
    Xd, Zd, vd = (torch.from_numpy(a).cuda() for a in (X, Z, v))
    with pytest.raises(K.KnnError) as ei:
        K.kmv_apply(Xd, Zd, vd, 1.0, 0.0, 64 * W.MB)
    assert ei.value.status == K.KNN_ERR_INVALID_ARG
    with pytest.raises(K.KnnError) as ei:
        K.kmv_apply(Xd, Zd, vd, -1.0, 1.0, 64 * W.MB)
    assert ei.value.status == K.KNN_ERR_INVALID_ARG
    with pytest.raises(K.KnnError) as ei:
        K.kmv_apply(Xd, Zd, vd, 1.0, 1.0, 1000)  # the scaled norms of Z alone need 20 KB
    assert ei.value.status == K.KNN_ERR_MEM_LIMIT_TOO_SMALL
    plan = K.kmv_plan(100, 5000, 16, 64 * W.MB)
    small = torch.empty(plan.workspace_bytes - 256, dtype=torch.uint8, device="cuda")
    y = torch.empty(100, dtype=torch.float64, device="cuda")
    st = K.kmv_apply_raw(Xd.data_ptr(), 16, Zd.data_ptr(), 16, vd.data_ptr(), 100, 5000, 16, 1.0,
                         1.0, 64 * W.MB, small.data_ptr(), small.numel(), y.data_ptr(), 0)
    assert st == K.KNN_ERR_WORKSPACE_TOO_SMALL
    st = K.kmv_apply_raw(Xd.data_ptr(), 8, Zd.data_ptr(), 16, vd.data_ptr(), 100, 5000, 16, 1.0,
                         1.0, 64 * W.MB, small.data_ptr(), small.numel(), y.data_ptr(), 0)
    assert st == K.KNN_ERR_INVALID_ARG


@pytest.mark.parametrize("key,count", [("kmv1", 24), ("kmv2", 24)])
def test_full_size_sampled_rows(K, oracle, key, count):
    # the benchmark's launch configuration; sampled rows against the oracle
    w = W.KMV_WORKLOADS[key]
    say("full size", w)
    X, Z, v = W.make_kmv(w)
    rows = np.sort(np.random.Generator(np.random.PCG64(5)).choice(w.n, count, replace=False))
    parity(K, oracle, X, Z, v, w.variance, w.lengthscale, limit=w.mem_limit, rows=rows,
           z_is_x=w.z_is_x)


# ---------------------------------------------------------------------------------------
# all-fp64 entry point (kmv_apply_f64), against the fp64-input oracle
# ---------------------------------------------------------------------------------------
EPS64 = 2.0 ** -53


def parity_f64(K, oracle, X, Z, v, variance, lengthscale, limit=64 * W.MB, rows=None, z_is_x=False):
    Xd = torch.from_numpy(X).cuda()
    Zd = Xd if z_is_x else torch.from_numpy(Z).cuda()
    y = K.kmv_apply(Xd, Zd, torch.from_numpy(v).cuda(), variance, lengthscale, limit)
    torch.cuda.synchronize()
    y = y.cpu().numpy()
    assert y.shape == (X.shape[0],) and y.dtype == np.float64 and np.isfinite(y).all()
    sel = np.arange(X.shape[0]) if rows is None else np.asarray(rows)
    ref = oracle.kmv_f64(X, Z, v, variance, lengthscale, rows=None if rows is None else sel)
    m, d = Z.shape
    c = 0.5 / lengthscale ** 2
    tol = np.empty(len(sel))
    for t, i in enumerate(sel):
        a = c * ((X[i][None, :] - Z) ** 2).sum(1)
        mag = variance * np.exp(-a) * np.abs(v)
        tol[t] = 2 * (mag * ((m + 8) * EPS64 + (d + 4) * EPS64 * a)).sum() + 1e-300
    err = np.abs(y[sel] - ref)
    worst = float((err / tol).max()) if len(sel) else 0.0
    say(f"   kmv f64 parity rows={len(sel)} max err/tol={worst:.3g} max|err|={err.max() if len(sel) else 0:.3g}")
    assert (err <= tol).all(), f"worst err/tol {worst}"
    return y


# (seed, n, m, d, variance, lengthscale, spread)
SMALL_F64 = [
    (100, 1, 1, 1, 1.0, 1.0, 1.0),
    (101, 700, 1513, 1, 1.0, 1.0, 1.0),    # the appendix case, ragged both ways
    (102, 257, 66, 3, 2.5, 0.7, 1.0),
    (103, 300, 777, 8, 1.0, 3.0, 1.0),     # last register-resident dimension
    (104, 300, 1003, 9, 1.0, 3.0, 1.0),    # chunked rows: two chunks and one column, point tail
    (105, 260, 1111, 11, 1.7, 4.0, 1.0),   # three tail columns
    (106, 260, 1112, 20, 1.0, 4.0, 1.0),   # whole chunks, whole point groups
    (107, 140, 700, 300, 1.0, 17.0, 1.0),
    (108, 400, 800, 2, 1.0, 1.0, 1e4),     # coordinates far from the origin
]


@pytest.mark.parametrize("case", SMALL_F64, ids=lambda c: "s%d_n%d_m%d_d%d" % c[:4])
def test_f64_small_cases_match_oracle(K, oracle, case):
    seed, n, m, d, variance, lengthscale, spread = case
    say("f64 case", case)
    X, Z, v = W.random_kmv_case(seed, n, m, d, spread, dtype="f64")
    parity_f64(K, oracle, X, Z, v, variance, lengthscale)


@pytest.mark.parametrize("d", [2, 16])
def test_f64_point_ranges_strides_and_guard(K, oracle, d):
    n, m = 300, 40000
    X, Z, v = W.random_kmv_case(120 + d, n, m, d, dtype="f64")
    ls = 1.0 if d == 2 else 4.0
    plan = K.kmv_plan(n, m, d, 64 * W.MB, "f64")
    assert plan.n_splits > 1 and plan.norms_bytes == 0
    assert K.kmv_plan(n, m, d, 8 * n, "f64").n_splits == 1
    y1 = parity_f64(K, oracle, X, Z, v, 1.0, ls)
    y2 = parity_f64(K, oracle, X, Z, v, 1.0, ls, limit=8 * n)
    assert np.allclose(y1, y2, rtol=1e-12, atol=1e-12)
    # strided rows, caller-owned workspace with guard bytes behind it
    Xw = torch.full((n, d + 3), 9.0, dtype=torch.float64, device="cuda")
    Zw = torch.full((m, d + 1), -9.0, dtype=torch.float64, device="cuda")
    Xw[:, :d] = torch.from_numpy(X).cuda()
    Zw[:, :d] = torch.from_numpy(Z).cuda()
    buf = torch.full((plan.workspace_bytes + 4096,), 0xA5, dtype=torch.uint8, device="cuda")
    y3 = K.kmv_apply(Xw[:, :d], Zw[:, :d], torch.from_numpy(v).cuda(), 1.0, ls, 64 * W.MB,
                     workspace=buf[:plan.workspace_bytes])
    torch.cuda.synchronize()
    assert np.array_equal(y3.cpu().numpy(), y1)
    assert (buf[plan.workspace_bytes:] == 0xA5).all()


def test_f64_resolves_what_fp32_cannot(K, oracle):
    # points 1e-9 apart around 1.0, lengthscale 1e-9: in fp32 they would coincide
    X = 1.0 + 1e-9 * np.arange(500, dtype=np.float64).reshape(-1, 1)
    v = np.random.Generator(np.random.PCG64(3)).standard_normal(500)
    y = parity_f64(K, oracle, X, X, v, 1.0, 1e-9, z_is_x=True)
    assert not np.allclose(y, v.sum(), rtol=1e-3)  # far from the all-ones matrix fp32 would see


def test_f64_empty_sides_and_errors(K):
    X = torch.zeros((300, 3), dtype=torch.float64, device="cuda")
    y = K.kmv_apply(X, torch.empty((0, 3), dtype=torch.float64, device="cuda"),
                    torch.empty((0,), dtype=torch.float64, device="cuda"), 1.0, 1.0, 64 * W.MB,
                    out=torch.full((300,), 7.0, dtype=torch.float64, device="cuda"))
    torch.cuda.synchronize()
    assert (y.cpu().numpy() == 0).all()
    with pytest.raises(K.KnnError) as ei:
        K.kmv_apply(X, X, torch.zeros(300, dtype=torch.float32, device="cuda"), 1.0, 1.0, 64 * W.MB)
    assert ei.value.status == K.KNN_ERR_INVALID_ARG  # mixed precisions
    with pytest.raises(K.KnnError) as ei:
        K.kmv_apply(X, X, torch.zeros(300, dtype=torch.float64, device="cuda"), 1.0, -2.0, 64 * W.MB)
    assert ei.value.status == K.KNN_ERR_INVALID_ARG


def test_f64_full_size_sampled_rows(K, oracle):
    w = W.KMV_WORKLOADS["kmv3"]
    say("full size", w)
    X, Z, v = W.make_kmv(w)
    rows = np.sort(np.random.Generator(np.random.PCG64(6)).choice(w.n, 16, replace=False))
    parity_f64(K, oracle, X, Z, v, w.variance, w.lengthscale, limit=w.mem_limit, rows=rows,
               z_is_x=True)
