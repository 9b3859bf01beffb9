"""Seeded synthetic inputs shaped like the paper's kNN workloads.

This module only draws random numbers (numpy PCG64) and names sizes.  It holds
none of the method's arithmetic: no distances, no norms, no selection.  Both the
CPU oracle's callers and the GPU path's callers take their inputs from here so
that the two sides see identical bits.

The five workloads follow the paper's experiment grid (section 5.2 and the
appendix table: random data with n in {1e4, 1e6, 1e7} and d in {3, 10, 100},
image vectors with d = 784, word-embedding-like vectors with d in 50..200) and
the memory-limit sweep of section 5.1 / figure 1.  The image and embedding data
sets themselves are not available; value distributions of the same structure
(sparse non-negative pixels, clustered embeddings) stand in for them.
"""
from __future__ import annotations

from dataclasses import dataclass, replace

import numpy as np

SEED_BASE = 220614148
MB = 10 ** 6  # decimal units: the paper's worked example has 125e6 fp64 values = "1GB"
GB = 10 ** 9


@dataclass(frozen=True)
class Workload:
    cfg: int
    name: str
    m: int
    n: int
    d: int
    k: int
    mem_limit: int
    kind: str            # value distribution
    q_is_x: bool = False  # queries are the data points themselves (kNN graph)
    sweep: tuple = ()     # extra memory limits (config 5)
    metric: str = "l2"    # "l2" (squared Euclidean), "cosine" or "l1"

    @property
    def pairs(self) -> int:
        return self.m * self.n


WORKLOADS = {
    1: Workload(1, "c1_random_d16", 1_000, 10_000, 16, 10, 64 * MB, "normal"),
    2: Workload(2, "c2_pointcloud_d3", 1_000_000, 1_000_000, 3, 16, 1 * GB, "uniform", q_is_x=True),
    3: Workload(3, "c3_imagelike_d784", 10_000, 1_000_000, 784, 10, 2 * GB, "sparse"),
    4: Workload(4, "c4_clustered_d128", 100_000, 10_000_000, 128, 100, 8 * GB, "gmm"),
    5: Workload(5, "c5_memsweep_d256", 50_000, 2_000_000, 256, 32, 1 * GB, "normal",
                sweep=(128 * MB, 1 * GB, 8 * GB, 64 * GB)),
    # the cosine rows of the paper's table: word embeddings with n = 1,183,514 and d in
    # {50, 100, 200}, m = 1e4 queries; the same clustered mixture stands in for them
    6: Workload(6, "c6_cosine_d100", 10_000, 1_183_514, 100, 10, 1 * GB, "gmm", metric="cosine"),
    # the L1 rows of the table: random data, n = 1e6, d = 100, m = 1e4 queries
    7: Workload(7, "c7_l1_d100", 10_000, 1_000_000, 100, 10, 1 * GB, "normal", metric="l1"),
}


def scaled(cfg: int, m: int | None = None, n: int | None = None, **kw) -> Workload:
    """Same distribution and d as config `cfg`, other sizes."""
    w = WORKLOADS[cfg]
    if w.q_is_x:
        size = n if n is not None else (m if m is not None else w.n)
        m = n = size
    else:
        m = w.m if m is None else m
        n = w.n if n is None else n
    return replace(w, m=m, n=n, **kw)


def _rng(cfg: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(SEED_BASE + 1000 * cfg + stream))


_CHUNK = 1 << 22  # values drawn per call, bounds temporary memory


def _fill_normal(rng, out):
    flat = out.reshape(-1)
    for s in range(0, flat.size, _CHUNK):
        e = min(flat.size, s + _CHUNK)
        rng.standard_normal(e - s, dtype=np.float32, out=flat[s:e])


def _fill_uniform(rng, out):
    flat = out.reshape(-1)
    for s in range(0, flat.size, _CHUNK):
        e = min(flat.size, s + _CHUNK)
        rng.random(e - s, dtype=np.float32, out=flat[s:e])


def _fill_sparse(rng, out):
    """Entry is 0 with probability 0.8, else uniform in (0, 1]."""
    flat = out.reshape(-1)
    for s in range(0, flat.size, _CHUNK):
        e = min(flat.size, s + _CHUNK)
        keep = rng.random(e - s, dtype=np.float32) < np.float32(0.2)
        val = np.float32(1.0) - rng.random(e - s, dtype=np.float32)
        flat[s:e] = np.where(keep, val, np.float32(0.0))


def _fill_gmm(rng, out, centres):
    """Uniform mixture weights; point = centre + unit isotropic noise."""
    rows = out.shape[0]
    step = max(1, _CHUNK // out.shape[1])
    for s in range(0, rows, step):
        e = min(rows, s + step)
        lab = rng.integers(0, centres.shape[0], size=e - s)
        noise = rng.standard_normal((e - s, out.shape[1]), dtype=np.float32)
        out[s:e] = centres[lab] + noise


def gmm_centres(cfg: int, d: int, comps: int = 1000) -> np.ndarray:
    """Component centres ~ N(0, 4 I), i.e. standard deviation 2 per coordinate."""
    c = _rng(cfg, 2).standard_normal((comps, d), dtype=np.float32)
    return (np.float32(2.0) * c).astype(np.float32)


def make(w: Workload):
    """Returns (Q, X) as C-contiguous float32 arrays; Q is X itself when q_is_x."""
    X = np.empty((w.n, w.d), dtype=np.float32)
    if w.kind == "normal":
        _fill_normal(_rng(w.cfg, 0), X)
    elif w.kind == "uniform":
        _fill_uniform(_rng(w.cfg, 0), X)
    elif w.kind == "sparse":
        _fill_sparse(_rng(w.cfg, 0), X)
    elif w.kind == "gmm":
        centres = gmm_centres(w.cfg, w.d)
        _fill_gmm(_rng(w.cfg, 0), X, centres)
    else:
        raise ValueError(w.kind)
    if w.q_is_x:
        return X, X
    Q = np.empty((w.m, w.d), dtype=np.float32)
    if w.kind == "normal":
        _fill_normal(_rng(w.cfg, 1), Q)
    elif w.kind == "uniform":
        _fill_uniform(_rng(w.cfg, 1), Q)
    elif w.kind == "sparse":
        _fill_sparse(_rng(w.cfg, 1), Q)
    else:
        _fill_gmm(_rng(w.cfg, 1), Q, centres)
    return Q, X


def sample_rows(w: Workload, count: int) -> np.ndarray:
    """Seeded subset of query rows (sorted, distinct) for row-level checks."""
    count = min(count, w.m)
    r = _rng(w.cfg, 3).choice(w.m, size=count, replace=False)
    return np.sort(r).astype(np.int64)


def random_case(seed: int, m: int, n: int, d: int, kind: str = "normal"):
    """Small free-form case for the edge-case tests."""
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 7_000_000 + seed))
    if kind == "normal":
        X = rng.standard_normal((n, d), dtype=np.float32)
        Q = rng.standard_normal((m, d), dtype=np.float32)
    elif kind == "uniform":
        X = rng.random((n, d), dtype=np.float32)
        Q = rng.random((m, d), dtype=np.float32)
    elif kind == "grid":  # many exact ties: small integer coordinates
        X = rng.integers(0, 4, size=(n, d)).astype(np.float32)
        Q = rng.integers(0, 4, size=(m, d)).astype(np.float32)
    else:
        raise ValueError(kind)
    return Q, X


# ---------------------------------------------------------------------------------------------
# Kernel matrix-vector product (paper section 5.1): y = K v with an n x n squared-exponential
# kernel matrix.  The appendix names 1-dimensional inputs of size 1e6 and the kernel's library
# defaults (variance 1, lengthscale 1); it does not say how the inputs are distributed, so
# they are standard normal here.
# ---------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class KmvWorkload:
    name: str
    n: int               # rows of X = rows of K
    m: int               # rows of Z = columns of K = length of v
    d: int
    variance: float
    lengthscale: float
    mem_limit: int
    z_is_x: bool = True  # square kernel matrix of one point set
    stream: int = 0
    dtype: str = "f32"   # "f64": fp64 inputs for the all-fp64 entry point (the paper's precision)

    @property
    def pairs(self) -> int:
        return self.n * self.m


KMV_WORKLOADS = {
    "kmv1": KmvWorkload("kmv1_d1", 1_000_000, 1_000_000, 1, 1.0, 1.0, 1 * GB),
    # a multi-dimensional input set on the matrix-core path, lengthscale of the order sqrt(d)
    "kmv2": KmvWorkload("kmv2_d32", 200_000, 200_000, 32, 1.0, 6.0, 1 * GB, stream=1),
    # the appendix case in the precision the paper evaluates it in
    "kmv3": KmvWorkload("kmv3_d1_f64", 1_000_000, 1_000_000, 1, 1.0, 1.0, 1 * GB, stream=2,
                        dtype="f64"),
}


def scaled_kmv(key: str, n: int | None = None, m: int | None = None, **kw) -> KmvWorkload:
    w = KMV_WORKLOADS[key]
    if w.z_is_x and "z_is_x" not in kw:
        size = n if n is not None else (m if m is not None else w.n)
        n = m = size
    else:
        n = w.n if n is None else n
        m = w.m if m is None else m
    return replace(w, n=n, m=m, **kw)


def make_kmv(w: KmvWorkload):
    """Returns (X, Z, v): [n,d], [m,d] (X itself when z_is_x) and [m], float32 or float64."""
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 9_000_000 + w.stream))
    if w.dtype == "f64":
        X = rng.standard_normal((w.n, w.d))
        Z = X if w.z_is_x else rng.standard_normal((w.m, w.d))
        return X, Z, rng.standard_normal(w.m)
    X = np.empty((w.n, w.d), dtype=np.float32)
    _fill_normal(rng, X)
    if w.z_is_x:
        Z = X
    else:
        Z = np.empty((w.m, w.d), dtype=np.float32)
        _fill_normal(rng, Z)
    v = np.empty((w.m,), dtype=np.float32)
    _fill_normal(rng, v)
    return X, Z, v


def random_kmv_case(seed: int, n: int, m: int, d: int, spread: float = 1.0, dtype: str = "f32"):
    """Small free-form case: normal points with the given spread, normal v."""
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 8_000_000 + seed))
    if dtype == "f64":
        return (spread * rng.standard_normal((n, d)), spread * rng.standard_normal((m, d)),
                rng.standard_normal(m))
    X = (np.float32(spread) * rng.standard_normal((n, d), dtype=np.float32)).astype(np.float32)
    Z = (np.float32(spread) * rng.standard_normal((m, d), dtype=np.float32)).astype(np.float32)
    v = rng.standard_normal((m,), dtype=np.float32)
    return X, Z, v


# ---------------------------------------------------------------------------------------------
# SGPR accumulations (paper section 5.3): A = K_uf K_fu, b = K_uf y.  The paper runs on two
# regression data sets (n = 434,874 with d = 3, scaled to 1e4 inducing points; n = 2,049,280
# with d = 11, up to 4000 inducing points in its table); the data sets are not available, so
# standardised features are drawn as N(0, 1), the inducing points are the first m data
# points (the usual initialisation) and the targets are N(0, 1).
# ---------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class SgprWorkload:
    name: str
    m: int   # inducing points
    n: int   # data points
    d: int
    variance: float
    lengthscale: float
    mem_limit: int
    stream: int = 0

    @property
    def flops(self) -> int:
        """Multiply-adds of the lower triangle of A, counted as 2 flops each."""
        return self.n * self.m * (self.m + 1)


SGPR_WORKLOADS = {
    "sgpr1": SgprWorkload("sgpr1_road_d3_m10000", 10_000, 434_874, 3, 1.0, 1.0, 1 * GB),
    "sgpr2": SgprWorkload("sgpr2_electric_d11_m4000", 4_000, 2_049_280, 11, 1.0, 3.0, 1 * GB, stream=1),
}


def make_sgpr(w: SgprWorkload):
    """Returns (U, X, y): float32 [m,d] (a copy of the first m data points), [n,d], [n]."""
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 10_000_000 + w.stream))
    X = np.empty((w.n, w.d), dtype=np.float32)
    _fill_normal(rng, X)
    y = np.empty((w.n,), dtype=np.float32)
    _fill_normal(rng, y)
    return X[:w.m].copy(), X, y


def random_sgpr_case(seed: int, m: int, n: int, d: int):
    rng = np.random.Generator(np.random.PCG64(SEED_BASE + 11_000_000 + seed))
    U = rng.standard_normal((m, d), dtype=np.float32)
    X = rng.standard_normal((n, d), dtype=np.float32)
    y = rng.standard_normal((n,), dtype=np.float32)
    return U, X, y
