"""ctypes binding of libknn_mi355x.so: argument marshalling only.

Every step of the search runs in the library's HIP kernels; PyTorch is used for device
memory (inputs, outputs, the workspace) and for the current stream, nothing else.  There is
no CPU fallback: a missing library raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

from . import build as _build

KNN_OK = 0
KNN_ERR_INVALID_ARG = 1
KNN_ERR_MEM_LIMIT_TOO_SMALL = 2
KNN_ERR_WORKSPACE_TOO_SMALL = 3
KNN_ERR_UNSUPPORTED = 4
KNN_ERR_HIP = 5
KNN_ERR_STATIC_SCRATCH_TOO_SMALL = 6
KNN_STATIC_SCRATCH_BYTES = 33554432
KNN_MAX_K = 1024
KNN_PATH_LOWD = 0
KNN_PATH_LOWD_MFMA = 2
KNN_PATH_LOWD_BF16 = 4
KNN_PATH_MFMA_SPLIT = 5
KNN_PATH_MFMA_PACKED = 6
KNN_PATH_MFMA_WIDE = 7
KNN_METRIC_L2SQ = 0
KNN_METRIC_COSINE = 1
KNN_METRIC_L1 = 2
KNN_PATH_L1 = 3
METRICS = {"l2": KNN_METRIC_L2SQ, "cosine": KNN_METRIC_COSINE, "l1": KNN_METRIC_L1}

EXPORTED_SYMBOLS = (
    "knn_plan", "knn_workspace_bytes", "knn_search", "knn_last_stats", "knn_status_string",
    "knn_parse_size", "knn_chunk_rows", "knn_last_hip_error", "knn_profile_enable",
    "knn_profile_read", "knn_plan_metric", "knn_search_metric",
    "kmv_plan", "kmv_apply", "kmv_plan_f64", "kmv_apply_f64",
    "knn_plan_host_x", "knn_search_host_x", "sgpr_plan", "sgpr_accumulate",
    "knn_search_static", "knn_measure_mfma_peak",
)
KMV_PATH_LOWD = 0
KMV_PATH_MFMA = 1
KMV_PATH_VALU = 2


class KmvPlanStruct(ctypes.Structure):
    _fields_ = [
        ("n", ctypes.c_int64), ("m", ctypes.c_int64),
        ("d", ctypes.c_int32), ("path", ctypes.c_int32),
        ("tile_rows", ctypes.c_int32), ("n_splits", ctypes.c_int32),
        ("norms_bytes", ctypes.c_int64), ("partials_bytes", ctypes.c_int64),
        ("workspace_bytes", ctypes.c_int64), ("min_limit_bytes", ctypes.c_int64),
    ]


class SgprPlanStruct(ctypes.Structure):
    _fields_ = [
        ("m", ctypes.c_int64), ("n", ctypes.c_int64),
        ("d", ctypes.c_int32), ("col_groups", ctypes.c_int32),
        ("chunk_cols", ctypes.c_int64), ("n_chunks", ctypes.c_int64), ("chunk_ld", ctypes.c_int64),
        ("workspace_bytes", ctypes.c_uint64), ("min_limit_bytes", ctypes.c_uint64),
    ]


@dataclass(frozen=True)
class SgprPlan:
    m: int
    n: int
    d: int
    col_groups: int
    chunk_cols: int
    n_chunks: int
    chunk_ld: int
    workspace_bytes: int
    min_limit_bytes: int


@dataclass(frozen=True)
class KmvPlan:
    n: int
    m: int
    d: int
    path: int
    tile_rows: int
    n_splits: int
    norms_bytes: int
    partials_bytes: int
    workspace_bytes: int
    min_limit_bytes: int


class PlanStruct(ctypes.Structure):
    _fields_ = [
        ("m", ctypes.c_int64), ("n", ctypes.c_int64),
        ("d", ctypes.c_int32), ("k", ctypes.c_int32),
        ("path", ctypes.c_int32), ("tile_q", ctypes.c_int32),
        ("tile_x", ctypes.c_int32), ("n_splits", ctypes.c_int32),
        ("chunk_rows", ctypes.c_int64), ("q_chunks", ctypes.c_int64),
        ("streams", ctypes.c_int32), ("seed_points", ctypes.c_int32),
        ("metric", ctypes.c_int32), ("seed_cells", ctypes.c_int32),
        ("norms_bytes", ctypes.c_uint64), ("query_bytes", ctypes.c_uint64),
        ("lists_bytes", ctypes.c_uint64),
        ("workspace_bytes", ctypes.c_uint64), ("min_limit_bytes", ctypes.c_uint64),
        ("private_bytes", ctypes.c_uint64), ("slab_points", ctypes.c_int64),
    ]


class HostPlanStruct(ctypes.Structure):
    _fields_ = [
        ("m", ctypes.c_int64), ("n", ctypes.c_int64),
        ("d", ctypes.c_int32), ("k", ctypes.c_int32),
        ("metric", ctypes.c_int32), ("reserved", ctypes.c_int32),
        ("block_rows", ctypes.c_int64), ("n_blocks", ctypes.c_int64),
        ("staging_bytes", ctypes.c_uint64), ("block_out_bytes", ctypes.c_uint64),
        ("inner_limit_bytes", ctypes.c_uint64), ("workspace_bytes", ctypes.c_uint64),
        ("min_limit_bytes", ctypes.c_uint64), ("inner", PlanStruct),
    ]


@dataclass(frozen=True)
class HostPlan:
    m: int
    n: int
    d: int
    k: int
    metric: int
    block_rows: int
    n_blocks: int
    staging_bytes: int
    block_out_bytes: int
    inner_limit_bytes: int
    workspace_bytes: int
    min_limit_bytes: int
    inner: "Plan"


@dataclass(frozen=True)
class Plan:
    m: int
    n: int
    d: int
    k: int
    path: int
    tile_q: int
    tile_x: int
    n_splits: int
    chunk_rows: int
    q_chunks: int
    streams: int
    seed_points: int
    metric: int
    seed_cells: int
    norms_bytes: int
    query_bytes: int
    lists_bytes: int
    workspace_bytes: int
    min_limit_bytes: int
    private_bytes: int = 0
    slab_points: int = 0


class KnnError(RuntimeError):
    def __init__(self, status: int, message: str, min_limit_bytes: int = 0):
        super().__init__(f"knn status {status}: {message}")
        self.status = status
        self.min_limit_bytes = min_limit_bytes


_lib = None


def library_path() -> str:
    return _build.LIB_PATH


def load():
    """Loads the built library; builds it first only if it does not exist at all."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB_PATH):
        _build.build()
    # The tensors this binding passes are torch's, so the HIP runtime inside torch has to be the
    # one this library binds to: loaded first, its libamdhip64 satisfies the library's dependency.
    # (The other way round the process holds two runtimes, and the one the library got sees no
    # device.)  Planning needs neither.
    try:
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = ctypes.CDLL(_build.LIB_PATH)
    i64, i32, u64, vp = ctypes.c_int64, ctypes.c_int32, ctypes.c_uint64, ctypes.c_void_p
    lib.knn_plan.argtypes = [i64, i64, i32, i32, u64, ctypes.POINTER(PlanStruct)]
    lib.knn_plan.restype = ctypes.c_int
    lib.knn_plan_metric.argtypes = [i64, i64, i32, i32, ctypes.c_int, u64, ctypes.POINTER(PlanStruct)]
    lib.knn_plan_metric.restype = ctypes.c_int
    lib.knn_search_metric.argtypes = [vp, i64, vp, i64, i64, i64, i32, i32, ctypes.c_int, u64, vp, u64,
                                      vp, vp, vp]
    lib.knn_search_metric.restype = ctypes.c_int
    lib.knn_workspace_bytes.argtypes = [i64, i64, i32, i32, u64]
    lib.knn_workspace_bytes.restype = u64
    lib.knn_search.argtypes = [vp, i64, vp, i64, i64, i64, i32, i32, u64, vp, u64, vp, vp, vp]
    lib.knn_search.restype = ctypes.c_int
    lib.knn_search_static.argtypes = [vp, i64, vp, i64, i64, i64, i32, i32, vp, vp, vp]
    lib.knn_search_static.restype = ctypes.c_int
    lib.knn_measure_mfma_peak.argtypes = [i32, vp, u64, vp, ctypes.POINTER(ctypes.c_float)]
    lib.knn_measure_mfma_peak.restype = ctypes.c_int
    lib.knn_last_stats.argtypes = [ctypes.POINTER(PlanStruct), ctypes.POINTER(u64)]
    lib.knn_last_stats.restype = ctypes.c_int
    lib.knn_status_string.argtypes = [ctypes.c_int]
    lib.knn_status_string.restype = ctypes.c_char_p
    lib.knn_parse_size.argtypes = [ctypes.c_char_p, ctypes.POINTER(u64)]
    lib.knn_parse_size.restype = ctypes.c_int
    lib.knn_chunk_rows.argtypes = [u64, u64]
    lib.knn_chunk_rows.restype = i64
    lib.knn_profile_enable.argtypes = [i32]
    lib.knn_profile_enable.restype = ctypes.c_int
    lib.knn_profile_read.argtypes = [ctypes.POINTER(ctypes.c_float)] * 3 + [ctypes.POINTER(i64)]
    lib.knn_profile_read.restype = ctypes.c_int
    lib.knn_last_hip_error.argtypes = []
    lib.knn_last_hip_error.restype = ctypes.c_char_p
    lib.knn_plan_host_x.argtypes = [i64, i64, i32, i32, ctypes.c_int, u64,
                                    ctypes.POINTER(HostPlanStruct)]
    lib.knn_plan_host_x.restype = ctypes.c_int
    lib.knn_search_host_x.argtypes = lib.knn_search_metric.argtypes
    lib.knn_search_host_x.restype = ctypes.c_int
    lib.sgpr_plan.argtypes = [i64, i64, i32, u64, ctypes.POINTER(SgprPlanStruct)]
    lib.sgpr_plan.restype = ctypes.c_int
    lib.sgpr_accumulate.argtypes = [vp, i64, vp, i64, vp, i64, i64, i32, ctypes.c_double,
                                    ctypes.c_double, u64, vp, u64, vp, i64, vp, vp]
    lib.sgpr_accumulate.restype = ctypes.c_int
    lib.kmv_plan.argtypes = [i64, i64, i32, i64, ctypes.POINTER(KmvPlanStruct)]
    lib.kmv_plan.restype = ctypes.c_int
    lib.kmv_apply.argtypes = [vp, i64, vp, i64, vp, i64, i64, i32, ctypes.c_double, ctypes.c_double,
                              i64, vp, i64, vp, vp]
    lib.kmv_apply.restype = ctypes.c_int
    lib.kmv_plan_f64.argtypes = lib.kmv_plan.argtypes
    lib.kmv_plan_f64.restype = ctypes.c_int
    lib.kmv_apply_f64.argtypes = lib.kmv_apply.argtypes
    lib.kmv_apply_f64.restype = ctypes.c_int
    _lib = lib
    return lib


def knn_status_string(status: int) -> str:
    return load().knn_status_string(int(status)).decode()


def _plan_from_struct(ps: PlanStruct) -> Plan:
    return Plan(ps.m, ps.n, ps.d, ps.k, ps.path, ps.tile_q, ps.tile_x, ps.n_splits,
                ps.chunk_rows, ps.q_chunks, ps.streams, ps.seed_points, ps.metric, ps.seed_cells,
                ps.norms_bytes, ps.query_bytes, ps.lists_bytes,
                ps.workspace_bytes, ps.min_limit_bytes, ps.private_bytes, ps.slab_points)


def knn_plan(m: int, n: int, d: int, k: int, mem_limit_bytes: int, metric: str = "l2") -> Plan:
    ps = PlanStruct()
    st = load().knn_plan_metric(m, n, d, k, METRICS[metric], mem_limit_bytes, ctypes.byref(ps))
    if st != KNN_OK:
        raise KnnError(st, knn_status_string(st), int(ps.min_limit_bytes))
    return _plan_from_struct(ps)


def knn_workspace_bytes(m: int, n: int, d: int, k: int, mem_limit_bytes: int) -> int:
    return int(load().knn_workspace_bytes(m, n, d, k, mem_limit_bytes))


def knn_parse_size(text: str) -> int:
    out = ctypes.c_uint64(0)
    st = load().knn_parse_size(text.encode(), ctypes.byref(out))
    if st != KNN_OK:
        raise KnnError(st, f"cannot parse size {text!r}")
    return int(out.value)


def knn_chunk_rows(limit_bytes: int, row_bytes: int) -> int:
    return int(load().knn_chunk_rows(limit_bytes, row_bytes))


def knn_last_stats():
    ps = PlanStruct()
    peak = ctypes.c_uint64(0)
    st = load().knn_last_stats(ctypes.byref(ps), ctypes.byref(peak))
    if st != KNN_OK:
        raise KnnError(st, "no successful knn_search on this thread yet")
    return _plan_from_struct(ps), int(peak.value)


def knn_profile_enable(on: bool) -> None:
    load().knn_profile_enable(1 if on else 0)


def knn_profile_read():
    """(norms_ms, search_ms, refine_ms, search_launches) summed since the last read."""
    a, b, c = ctypes.c_float(0), ctypes.c_float(0), ctypes.c_float(0)
    launches = ctypes.c_int64(0)
    st = load().knn_profile_read(ctypes.byref(a), ctypes.byref(b), ctypes.byref(c),
                                 ctypes.byref(launches))
    if st != KNN_OK:
        raise KnnError(st, knn_status_string(st))
    return float(a.value), float(b.value), float(c.value), int(launches.value)


def knn_search_raw(q_ptr, ldq, x_ptr, ldx, m, n, d, k, mem_limit_bytes, ws_ptr, ws_bytes,
                   idx_ptr, dist_ptr, stream_ptr, metric: int = KNN_METRIC_L2SQ) -> int:
    """Direct call, raw integers for pointers; returns the status code."""
    if metric == KNN_METRIC_L2SQ:
        return int(load().knn_search(q_ptr, ldq, x_ptr, ldx, m, n, d, k, mem_limit_bytes, ws_ptr,
                                     ws_bytes, idx_ptr, dist_ptr, stream_ptr))
    return int(load().knn_search_metric(q_ptr, ldq, x_ptr, ldx, m, n, d, k, metric,
                                        mem_limit_bytes, ws_ptr, ws_bytes, idx_ptr, dist_ptr,
                                        stream_ptr))


def knn_search(Q, X, k: int, mem_limit_bytes: int, workspace=None, out=None, metric: str = "l2"):
    """knn_search(Q[m,d], X[n,d], k, mem_limit_bytes) -> (idx int32[m,k], dist fp32[m,k]).

    metric: "l2" (squared Euclidean), "cosine" (cosine distance) or "l1".
    Q and X are fp32 CUDA(HIP) tensors, row-major (a row stride larger than d is allowed).
    The workspace (a uint8 tensor of plan.workspace_bytes) is allocated here unless given.
    Work is enqueued on torch's current stream; no synchronisation is done.
    """
    import torch

    if not (Q.is_cuda and X.is_cuda):
        raise KnnError(KNN_ERR_INVALID_ARG, "Q and X must be device tensors (no CPU path exists)")
    if Q.dtype != torch.float32 or X.dtype != torch.float32 or Q.dim() != 2 or X.dim() != 2:
        raise KnnError(KNN_ERR_INVALID_ARG, "Q and X must be 2-D float32")
    if Q.shape[1] != X.shape[1] or Q.stride(1) != 1 or X.stride(1) != 1:
        raise KnnError(KNN_ERR_INVALID_ARG, "Q and X must share d and have unit column stride")
    m, d = Q.shape
    n = X.shape[0]
    plan = knn_plan(m, n, d, k, mem_limit_bytes, metric)
    if workspace is None:
        workspace = torch.empty(max(int(plan.workspace_bytes), 256), dtype=torch.uint8,
                                device=Q.device)
    if out is None:
        idx = torch.empty((m, k), dtype=torch.int32, device=Q.device)
        dist = torch.empty((m, k), dtype=torch.float32, device=Q.device)
    else:
        idx, dist = _check_out(out, m, k, Q.device)
    stream = torch.cuda.current_stream(Q.device).cuda_stream
    ldq = Q.stride(0) if m > 1 else max(d, Q.stride(0))
    ldx = X.stride(0) if n > 1 else max(d, X.stride(0))
    st = knn_search_raw(Q.data_ptr(), ldq, X.data_ptr(), ldx, m, n, d, k, mem_limit_bytes,
                        workspace.data_ptr(), workspace.numel(), idx.data_ptr(),
                        dist.data_ptr(), stream, METRICS[metric])
    if st != KNN_OK:
        detail = knn_status_string(st)
        if st == KNN_ERR_HIP:
            detail += " (" + load().knn_last_hip_error().decode() + ")"
        raise KnnError(st, detail)
    return idx, dist


def knn_measure_mfma_peak(dtype: str = "bf16") -> float:
    """TFLOP/s of a kernel of nothing but MFMAs on the current device ("bf16" or "f32")."""
    import torch

    scratch = torch.empty(1 << 20, dtype=torch.uint8, device="cuda")
    out = ctypes.c_float(0)
    st = int(load().knn_measure_mfma_peak({"bf16": 0, "f32": 1}[dtype], scratch.data_ptr(), scratch.numel(),
                                          torch.cuda.current_stream().cuda_stream, ctypes.byref(out)))
    if st != KNN_OK:
        raise KnnError(st, knn_status_string(st))
    return float(out.value)


def _check_out(out, m: int, k: int, device):
    """The kernels write m*k int32 / fp32 values through raw pointers: the tensors must be that."""
    import torch

    idx, dist = out
    for t, dt in ((idx, torch.int32), (dist, torch.float32)):
        if not t.is_cuda or t.device != device or t.dtype != dt or tuple(t.shape) != (m, k) or \
                not t.is_contiguous():
            raise KnnError(KNN_ERR_INVALID_ARG,
                           "out must be (int32[m,k], float32[m,k]), contiguous, on the device of Q")
    return idx, dist


def knn_search_static(Q, X, k: int, out=None):
    """knn_search through the library's static scratch buffer: the call allocates nothing on the
    library side (the outputs are the caller's: pass `out` to allocate nothing here either).
    Squared-Euclidean metric; the shape must fit KNN_STATIC_SCRATCH_BYTES."""
    import torch

    if not (Q.is_cuda and X.is_cuda):
        raise KnnError(KNN_ERR_INVALID_ARG, "Q and X must be device tensors (no CPU path exists)")
    if Q.dtype != torch.float32 or X.dtype != torch.float32 or Q.dim() != 2 or X.dim() != 2:
        raise KnnError(KNN_ERR_INVALID_ARG, "Q and X must be 2-D float32")
    if Q.shape[1] != X.shape[1] or Q.stride(1) != 1 or X.stride(1) != 1:
        raise KnnError(KNN_ERR_INVALID_ARG, "Q and X must share d and have unit column stride")
    m, d = Q.shape
    n = X.shape[0]
    if out is None:
        idx = torch.empty((m, k), dtype=torch.int32, device=Q.device)
        dist = torch.empty((m, k), dtype=torch.float32, device=Q.device)
    else:
        idx, dist = _check_out(out, m, k, Q.device)
    stream = torch.cuda.current_stream(Q.device).cuda_stream
    ldq = Q.stride(0) if m > 1 else max(d, Q.stride(0))
    ldx = X.stride(0) if n > 1 else max(d, X.stride(0))
    st = int(load().knn_search_static(Q.data_ptr(), ldq, X.data_ptr(), ldx, m, n, d, k,
                                      idx.data_ptr(), dist.data_ptr(), stream))
    if st != KNN_OK:
        detail = knn_status_string(st)
        if st == KNN_ERR_HIP:
            detail += " (" + load().knn_last_hip_error().decode() + ")"
        raise KnnError(st, detail)
    return idx, dist


def kmv_plan(n: int, m: int, d: int, mem_limit_bytes: int, dtype: str = "f32") -> KmvPlan:
    """dtype "f32": the plan of kmv_apply on fp32 points; "f64": of the all-fp64 entry point."""
    ps = KmvPlanStruct()
    fn = {"f32": load().kmv_plan, "f64": load().kmv_plan_f64}[dtype]
    st = int(fn(n, m, d, mem_limit_bytes, ctypes.byref(ps)))
    if st != KNN_OK:
        raise KnnError(st, knn_status_string(st) + f" (needs at least {ps.min_limit_bytes} bytes)"
                       if st == KNN_ERR_MEM_LIMIT_TOO_SMALL else knn_status_string(st))
    return KmvPlan(*(getattr(ps, f[0]) for f in KmvPlanStruct._fields_))


def kmv_apply_raw(x_ptr, ldx, z_ptr, ldz, v_ptr, n, m, d, variance, lengthscale, mem_limit_bytes,
                  ws_ptr, ws_bytes, y_ptr, stream_ptr, dtype: str = "f32") -> int:
    """Direct call, raw integers for pointers; returns the status code."""
    fn = {"f32": load().kmv_apply, "f64": load().kmv_apply_f64}[dtype]
    return int(fn(x_ptr, ldx, z_ptr, ldz, v_ptr, n, m, d, float(variance),
                  float(lengthscale), mem_limit_bytes, ws_ptr, ws_bytes, y_ptr, stream_ptr))


def kmv_apply(X, Z, v, variance: float, lengthscale: float, mem_limit_bytes: int, workspace=None,
              out=None):
    """kmv_apply(X[n,d], Z[m,d], v[m], variance, lengthscale, mem_limit_bytes) -> y fp64[n].

    y = K(X, Z) v with the squared-exponential kernel.  X, Z, v are device tensors, all fp32
    or all fp64 (the all-fp64 entry point then runs); rows may be strided.  The workspace (uint8, plan.workspace_bytes) is allocated here unless
    given.  Work is enqueued on torch's current stream; no synchronisation is done.
    """
    import torch

    if not (X.is_cuda and Z.is_cuda and v.is_cuda):
        raise KnnError(KNN_ERR_INVALID_ARG, "X, Z and v must be device tensors (no CPU path exists)")
    if X.dtype not in (torch.float32, torch.float64) or Z.dtype != X.dtype or v.dtype != X.dtype:
        raise KnnError(KNN_ERR_INVALID_ARG, "X, Z and v must be all float32 or all float64")
    dtype = "f32" if X.dtype == torch.float32 else "f64"
    if X.dim() != 2 or Z.dim() != 2 or v.dim() != 1 or X.shape[1] != Z.shape[1]:
        raise KnnError(KNN_ERR_INVALID_ARG, "X and Z must be 2-D with the same d, v 1-D")
    if v.shape[0] != Z.shape[0] or X.stride(1) != 1 or Z.stride(1) != 1 or \
            (v.shape[0] > 1 and v.stride(0) != 1):
        raise KnnError(KNN_ERR_INVALID_ARG, "v must have m contiguous entries; unit column strides")
    n, d = X.shape
    m = Z.shape[0]
    plan = kmv_plan(n, m, d, mem_limit_bytes, dtype)
    if workspace is None:
        workspace = torch.empty(max(int(plan.workspace_bytes), 256), dtype=torch.uint8,
                                device=X.device)
    y = out if out is not None else torch.empty((n,), dtype=torch.float64, device=X.device)
    stream = torch.cuda.current_stream(X.device).cuda_stream
    ldx = X.stride(0) if n > 1 else max(d, X.stride(0))
    ldz = Z.stride(0) if m > 1 else max(d, Z.stride(0))
    st = kmv_apply_raw(X.data_ptr(), ldx, Z.data_ptr(), ldz, v.data_ptr(), n, m, d, variance,
                       lengthscale, mem_limit_bytes, workspace.data_ptr(), workspace.numel(),
                       y.data_ptr(), stream, dtype)
    if st != KNN_OK:
        detail = knn_status_string(st)
        if st == KNN_ERR_HIP:
            detail += " (" + load().knn_last_hip_error().decode() + ")"
        raise KnnError(st, detail)
    return y


def knn_plan_host_x(m: int, n: int, d: int, k: int, mem_limit_bytes: int,
                    metric: str = "l2") -> HostPlan:
    ps = HostPlanStruct()
    st = int(load().knn_plan_host_x(m, n, d, k, METRICS[metric], mem_limit_bytes, ctypes.byref(ps)))
    if st != KNN_OK:
        raise KnnError(st, knn_status_string(st), int(ps.min_limit_bytes))
    vals = {f[0]: getattr(ps, f[0]) for f in HostPlanStruct._fields_ if f[0] not in ("reserved", "inner")}
    return HostPlan(inner=_plan_from_struct(ps.inner), **vals)


def knn_search_host_x(Q, X_host, k: int, mem_limit_bytes: int, workspace=None, out=None,
                      metric: str = "l2"):
    """knn_search with the data points in HOST memory, streamed through the workspace.

    Q: fp32 device tensor [m, d].  X_host: fp32 [n, d] in host memory - a CPU torch tensor
    (pinned memory lets the copies overlap the search) or a C-contiguous numpy array; it must
    stay alive and unchanged until the stream has been synchronised.
    """
    import numpy as np
    import torch

    if isinstance(X_host, np.ndarray):
        if X_host.dtype != np.float32 or X_host.ndim != 2 or not X_host.flags.c_contiguous:
            raise KnnError(KNN_ERR_INVALID_ARG, "X_host must be a C-contiguous 2-D float32 array")
        x_ptr, n, d, ldx = X_host.ctypes.data, X_host.shape[0], X_host.shape[1], X_host.shape[1]
    else:
        if X_host.is_cuda or X_host.dtype != torch.float32 or X_host.dim() != 2 or \
                X_host.stride(1) != 1:
            raise KnnError(KNN_ERR_INVALID_ARG, "X_host must be a 2-D float32 CPU tensor")
        n, d = X_host.shape
        x_ptr = X_host.data_ptr()
        ldx = X_host.stride(0) if n > 1 else max(d, X_host.stride(0))
    if not Q.is_cuda or Q.dtype != torch.float32 or Q.dim() != 2 or Q.shape[1] != d or \
            Q.stride(1) != 1:
        raise KnnError(KNN_ERR_INVALID_ARG, "Q must be a 2-D float32 device tensor with X's d")
    m = Q.shape[0]
    plan = knn_plan_host_x(m, n, d, k, mem_limit_bytes, metric)
    if workspace is None:
        workspace = torch.empty(max(int(plan.workspace_bytes), 256), dtype=torch.uint8,
                                device=Q.device)
    if out is None:
        idx = torch.empty((m, k), dtype=torch.int32, device=Q.device)
        dist = torch.empty((m, k), dtype=torch.float32, device=Q.device)
    else:
        idx, dist = _check_out(out, m, k, Q.device)
    stream = torch.cuda.current_stream(Q.device).cuda_stream
    ldq = Q.stride(0) if m > 1 else max(d, Q.stride(0))
    st = int(load().knn_search_host_x(Q.data_ptr(), ldq, x_ptr, ldx, m, n, d, k, METRICS[metric],
                                      mem_limit_bytes, workspace.data_ptr(), workspace.numel(),
                                      idx.data_ptr(), dist.data_ptr(), stream))
    if st != KNN_OK:
        detail = knn_status_string(st)
        if st == KNN_ERR_HIP:
            detail += " (" + load().knn_last_hip_error().decode() + ")"
        raise KnnError(st, detail)
    return idx, dist


def sgpr_plan(m: int, n: int, d: int, mem_limit_bytes: int) -> SgprPlan:
    ps = SgprPlanStruct()
    st = int(load().sgpr_plan(m, n, d, mem_limit_bytes, ctypes.byref(ps)))
    if st != KNN_OK:
        raise KnnError(st, knn_status_string(st), int(ps.min_limit_bytes))
    return SgprPlan(ps.m, ps.n, ps.d, ps.col_groups, ps.chunk_cols, ps.n_chunks, ps.chunk_ld,
                    ps.workspace_bytes, ps.min_limit_bytes)


def sgpr_accumulate(U, X, y, variance: float, lengthscale: float, mem_limit_bytes: int,
                    workspace=None, out=None):
    """sgpr_accumulate(U[m,d], X[n,d], y[n], ...) -> (A fp64[m,m], b fp64[m]).

    A = K_uf K_fu and b = K_uf y for the squared-exponential kernel between the inducing points
    U and the data X.  fp32 device tensors in, fp64 device tensors out; the workspace (uint8,
    plan.workspace_bytes) is allocated here unless given.  Work is enqueued on torch's current
    stream; no synchronisation is done.
    """
    import torch

    for t, nd in ((U, 2), (X, 2), (y, 1)):
        if not t.is_cuda or t.dtype != torch.float32 or t.dim() != nd:
            raise KnnError(KNN_ERR_INVALID_ARG, "U, X (2-D) and y (1-D) must be float32 device tensors")
    if U.shape[1] != X.shape[1] or y.shape[0] != X.shape[0] or U.stride(1) != 1 or \
            X.stride(1) != 1 or (y.shape[0] > 1 and y.stride(0) != 1):
        raise KnnError(KNN_ERR_INVALID_ARG, "shapes or strides do not fit")
    m, d = U.shape
    n = X.shape[0]
    plan = sgpr_plan(m, n, d, mem_limit_bytes)
    if workspace is None:
        workspace = torch.empty(max(int(plan.workspace_bytes), 256), dtype=torch.uint8,
                                device=U.device)
    if out is None:
        A = torch.empty((m, m), dtype=torch.float64, device=U.device)
        b = torch.empty((m,), dtype=torch.float64, device=U.device)
    else:
        A, b = out
    stream = torch.cuda.current_stream(U.device).cuda_stream
    ldu = U.stride(0) if m > 1 else max(d, U.stride(0))
    ldx = X.stride(0) if n > 1 else max(d, X.stride(0))
    st = int(load().sgpr_accumulate(U.data_ptr(), ldu, X.data_ptr(), ldx, y.data_ptr(), m, n, d,
                                    float(variance), float(lengthscale), mem_limit_bytes,
                                    workspace.data_ptr(), workspace.numel(), A.data_ptr(),
                                    A.stride(0) if m > 1 else m, b.data_ptr(), stream))
    if st != KNN_OK:
        detail = knn_status_string(st)
        if st == KNN_ERR_HIP:
            detail += " (" + load().knn_last_hip_error().decode() + ")"
        raise KnnError(st, detail)
    return A, b
