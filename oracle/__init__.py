"""ctypes front end of the CPU oracle (oracle/knn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
cpu_baseline leg of bench.py.  The GPU package never imports this module and
this module never imports the GPU package.

The oracle evaluates the plain definition of brute-force kNN (paper section
5.2) with naive difference-form squared distances in fp64 (section 4.1) and a
(distance, index) lexicographic order.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "knn_oracle.c")
_LIB = os.path.join(_HERE, "liboracle_knn.so")

_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, no fast-math, no FMA contraction)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        fp = ctypes.POINTER(ctypes.c_float)
        i64p = ctypes.POINTER(ctypes.c_int64)
        dp = ctypes.POINTER(ctypes.c_double)
        common = [fp, ctypes.c_int64, fp, ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                  ctypes.c_int32, i64p, ctypes.c_int64, i64p, dp, dp]
        lib.oracle_knn.argtypes = common + [ctypes.c_int32]
        lib.oracle_knn.restype = ctypes.c_int
        lib.oracle_knn_fullsort.argtypes = common
        lib.oracle_knn_fullsort.restype = ctypes.c_int
        lib.oracle_knn_metric.argtypes = common + [ctypes.c_int32, ctypes.c_int32]
        lib.oracle_knn_metric.restype = ctypes.c_int
        lib.oracle_knn_fullsort_metric.argtypes = common + [ctypes.c_int32]
        lib.oracle_knn_fullsort_metric.restype = ctypes.c_int
        lib.oracle_cosdist.argtypes = [fp, fp, ctypes.c_int32]
        lib.oracle_cosdist.restype = ctypes.c_double
        lib.oracle_l1dist.argtypes = [fp, fp, ctypes.c_int32]
        lib.oracle_l1dist.restype = ctypes.c_double
        lib.oracle_sqdist.argtypes = [fp, fp, ctypes.c_int32]
        lib.oracle_sqdist.restype = ctypes.c_double
        lib.oracle_sqdist_expanded.argtypes = [fp, fp, ctypes.c_int32]
        lib.oracle_sqdist_expanded.restype = ctypes.c_double
        lib.oracle_kmv.argtypes = [fp, ctypes.c_int64, fp, ctypes.c_int64, fp, ctypes.c_int64,
                                   ctypes.c_int64, ctypes.c_int32, ctypes.c_double, ctypes.c_double,
                                   i64p, ctypes.c_int64, dp, ctypes.c_int32]
        lib.oracle_kmv.restype = ctypes.c_int
        lib.oracle_kmv_f64.argtypes = [dp, ctypes.c_int64, dp, ctypes.c_int64, dp, ctypes.c_int64,
                                       ctypes.c_int64, ctypes.c_int32, ctypes.c_double,
                                       ctypes.c_double, i64p, ctypes.c_int64, dp, ctypes.c_int32]
        lib.oracle_kmv_f64.restype = ctypes.c_int
        lib.oracle_sgpr_accumulate.argtypes = [fp, ctypes.c_int64, fp, ctypes.c_int64, fp,
                                               ctypes.c_int64, ctypes.c_int64, ctypes.c_int32,
                                               ctypes.c_double, ctypes.c_double, dp, dp,
                                               ctypes.c_int32]
        lib.oracle_sgpr_accumulate.restype = ctypes.c_int
        lib.oracle_sgpr_entries.argtypes = [fp, ctypes.c_int64, fp, ctypes.c_int64, ctypes.c_int64,
                                            ctypes.c_int64, ctypes.c_int32, ctypes.c_double,
                                            ctypes.c_double, i64p, i64p, ctypes.c_int64, dp,
                                            ctypes.c_int32]
        lib.oracle_sgpr_entries.restype = ctypes.c_int
        lib.oracle_threads_used.argtypes = [ctypes.c_int32]
        lib.oracle_threads_used.restype = ctypes.c_int32
        _lib = lib
    return _lib


def default_threads() -> int:
    try:
        return max(1, len(os.sched_getaffinity(0)))
    except AttributeError:  # pragma: no cover
        return max(1, os.cpu_count() or 1)


def threads_used(nthreads: int | None = None) -> int:
    return int(_load().oracle_threads_used(int(nthreads or default_threads())))


def _as_f32_2d(a) -> np.ndarray:
    a = np.ascontiguousarray(a, dtype=np.float32)
    if a.ndim != 2:
        raise ValueError("expected a 2-D array")
    return a


def _run(fn, Q, X, k, rows, extra):
    Q = _as_f32_2d(Q)
    X = _as_f32_2d(X)
    if Q.shape[1] != X.shape[1]:
        raise ValueError("Q and X differ in dimension")
    n, d = X.shape
    if rows is None:
        rows_arr = None
        nrows = Q.shape[0]
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        nrows = rows_arr.shape[0]
        if nrows and (rows_arr.min() < 0 or rows_arr.max() >= Q.shape[0]):
            raise ValueError("row index out of range")
    idx = np.empty((nrows, k), dtype=np.int64)
    dist = np.empty((nrows, k), dtype=np.float64)
    nxt = np.empty((nrows,), dtype=np.float64)
    fp = ctypes.POINTER(ctypes.c_float)
    i64p = ctypes.POINTER(ctypes.c_int64)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = fn(Q.ctypes.data_as(fp), Q.shape[1], X.ctypes.data_as(fp), d, n, d, int(k),
            rows_arr.ctypes.data_as(i64p) if rows_arr is not None else None, nrows,
            idx.ctypes.data_as(i64p), dist.ctypes.data_as(dp), nxt.ctypes.data_as(dp), *extra)
    if rc != 0:
        raise ValueError("oracle rejected its arguments (need 1 <= k <= n, d >= 1)")
    return idx, dist, nxt


METRICS = {"l2": 0, "cosine": 1, "l1": 2}


def knn(Q, X, k, rows=None, nthreads: int | None = None, metric: str = "l2"):
    """Heap-selection oracle.  Returns (idx int64[r,k], dist fp64[r,k], next fp64[r])."""
    return _run(_load().oracle_knn_metric, Q, X, k, rows,
                (int(nthreads or default_threads()), METRICS[metric]))


def knn_fullsort(Q, X, k, rows=None, metric: str = "l2"):
    """Definition written out: all distances, one full sort, first k."""
    return _run(_load().oracle_knn_fullsort_metric, Q, X, k, rows, (METRICS[metric],))


def cosdist(q, x) -> float:
    q = np.ascontiguousarray(q, dtype=np.float32).ravel()
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    fp = ctypes.POINTER(ctypes.c_float)
    return float(_load().oracle_cosdist(q.ctypes.data_as(fp), x.ctypes.data_as(fp), q.shape[0]))


def l1dist(q, x) -> float:
    q = np.ascontiguousarray(q, dtype=np.float32).ravel()
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    fp = ctypes.POINTER(ctypes.c_float)
    return float(_load().oracle_l1dist(q.ctypes.data_as(fp), x.ctypes.data_as(fp), q.shape[0]))


def sqdist(q, x) -> float:
    q = np.ascontiguousarray(q, dtype=np.float32).ravel()
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    fp = ctypes.POINTER(ctypes.c_float)
    return float(_load().oracle_sqdist(q.ctypes.data_as(fp), x.ctypes.data_as(fp), q.shape[0]))


def sqdist_expanded(q, x) -> float:
    q = np.ascontiguousarray(q, dtype=np.float32).ravel()
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    fp = ctypes.POINTER(ctypes.c_float)
    return float(_load().oracle_sqdist_expanded(q.ctypes.data_as(fp), x.ctypes.data_as(fp),
                                                q.shape[0]))


def sqdist_pairs(Q, X, qi, xj, metric: str = "l2") -> np.ndarray:
    """fp64 distance of the listed (query, point) pairs."""
    Q = _as_f32_2d(Q)
    X = _as_f32_2d(X)
    qi = np.asarray(qi, dtype=np.int64).ravel()
    xj = np.asarray(xj, dtype=np.int64).ravel()
    out = np.empty(qi.shape[0], dtype=np.float64)
    lib = _load()
    fp = ctypes.POINTER(ctypes.c_float)
    d = Q.shape[1]
    qb = Q.ctypes.data
    xb = X.ctypes.data
    fn = {"cosine": lib.oracle_cosdist, "l1": lib.oracle_l1dist}.get(metric, lib.oracle_sqdist)
    for p in range(qi.shape[0]):
        out[p] = fn(ctypes.cast(qb + 4 * d * int(qi[p]), fp),
                                   ctypes.cast(xb + 4 * d * int(xj[p]), fp), d)
    return out


def kmv(X, Z, v, variance: float, lengthscale: float, rows=None, nthreads: int | None = None):
    """y = K(X, Z) v for the squared-exponential kernel, fp64 (paper section 5.1)."""
    X = _as_f32_2d(X)
    Z = _as_f32_2d(Z)
    v = np.ascontiguousarray(v, dtype=np.float32).ravel()
    if X.shape[1] != Z.shape[1] or v.shape[0] != Z.shape[0]:
        raise ValueError("shape mismatch")
    if rows is None:
        rows_arr, nrows = None, X.shape[0]
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        nrows = rows_arr.shape[0]
    y = np.empty(nrows, dtype=np.float64)
    fp = ctypes.POINTER(ctypes.c_float)
    i64p = ctypes.POINTER(ctypes.c_int64)
    rc = _load().oracle_kmv(X.ctypes.data_as(fp), X.shape[1], Z.ctypes.data_as(fp), Z.shape[1],
                            v.ctypes.data_as(fp), X.shape[0], Z.shape[0], X.shape[1],
                            float(variance), float(lengthscale),
                            rows_arr.ctypes.data_as(i64p) if rows_arr is not None else None, nrows,
                            y.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                            int(nthreads or default_threads()))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return y


def kmv_f64(X, Z, v, variance: float, lengthscale: float, rows=None, nthreads: int | None = None):
    """The same product on fp64 inputs, all in fp64 (the precision of paper section 5.1)."""
    X = np.ascontiguousarray(X, dtype=np.float64)
    Z = np.ascontiguousarray(Z, dtype=np.float64)
    v = np.ascontiguousarray(v, dtype=np.float64).ravel()
    if X.ndim != 2 or Z.ndim != 2 or X.shape[1] != Z.shape[1] or v.shape[0] != Z.shape[0]:
        raise ValueError("shape mismatch")
    if rows is None:
        rows_arr, nrows = None, X.shape[0]
    else:
        rows_arr = np.ascontiguousarray(rows, dtype=np.int64)
        nrows = rows_arr.shape[0]
    y = np.empty(nrows, dtype=np.float64)
    dp = ctypes.POINTER(ctypes.c_double)
    i64p = ctypes.POINTER(ctypes.c_int64)
    rc = _load().oracle_kmv_f64(X.ctypes.data_as(dp), X.shape[1], Z.ctypes.data_as(dp), Z.shape[1],
                                v.ctypes.data_as(dp), X.shape[0], Z.shape[0], X.shape[1],
                                float(variance), float(lengthscale),
                                rows_arr.ctypes.data_as(i64p) if rows_arr is not None else None,
                                nrows, y.ctypes.data_as(dp), int(nthreads or default_threads()))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return y


def sgpr_accumulate(U, X, y, variance: float, lengthscale: float, nthreads: int | None = None):
    """A = K_uf K_fu (fp64 [m,m]) and b = K_uf y (fp64 [m]) of paper section 5.3, the definition
    written out with K_uf stored whole: small cases only."""
    U = _as_f32_2d(U)
    X = _as_f32_2d(X)
    y = np.ascontiguousarray(y, dtype=np.float32).ravel()
    if U.shape[1] != X.shape[1] or y.shape[0] != X.shape[0]:
        raise ValueError("shape mismatch")
    m = U.shape[0]
    A = np.empty((m, m), dtype=np.float64)
    b = np.empty((m,), dtype=np.float64)
    fp = ctypes.POINTER(ctypes.c_float)
    dp = ctypes.POINTER(ctypes.c_double)
    rc = _load().oracle_sgpr_accumulate(U.ctypes.data_as(fp), U.shape[1], X.ctypes.data_as(fp),
                                        X.shape[1], y.ctypes.data_as(fp), m, X.shape[0], U.shape[1],
                                        float(variance), float(lengthscale), A.ctypes.data_as(dp),
                                        b.ctypes.data_as(dp), int(nthreads or default_threads()))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return A, b


def sgpr_entries(U, X, ii, jj, variance: float, lengthscale: float, nthreads: int | None = None):
    """The entries A[ii[p], jj[p]] of K_uf K_fu, each summed directly over the data."""
    U = _as_f32_2d(U)
    X = _as_f32_2d(X)
    ii = np.ascontiguousarray(ii, dtype=np.int64).ravel()
    jj = np.ascontiguousarray(jj, dtype=np.int64).ravel()
    if U.shape[1] != X.shape[1] or ii.shape != jj.shape:
        raise ValueError("shape mismatch")
    if ii.size and (min(ii.min(), jj.min()) < 0 or max(ii.max(), jj.max()) >= U.shape[0]):
        raise ValueError("entry out of range")
    out = np.empty(ii.shape[0], dtype=np.float64)
    fp = ctypes.POINTER(ctypes.c_float)
    i64p = ctypes.POINTER(ctypes.c_int64)
    rc = _load().oracle_sgpr_entries(U.ctypes.data_as(fp), U.shape[1], X.ctypes.data_as(fp),
                                     X.shape[1], U.shape[0], X.shape[0], U.shape[1], float(variance),
                                     float(lengthscale), ii.ctypes.data_as(i64p),
                                     jj.ctypes.data_as(i64p), ii.shape[0],
                                     out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
                                     int(nthreads or default_threads()))
    if rc != 0:
        raise ValueError("oracle rejected its arguments")
    return out
