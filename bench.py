#!/usr/bin/env python3
"""Benchmark of the whole kNN hot path on one MI355X.

A "step" is one knn_search call (norms, tiled distances + running top-k, merge, exact
re-evaluation) over one synthetic workload whose inputs are already resident in HBM.
Default (--workload all): the five kNN configurations, one after the other.  The top-level
record is the largest one, c4 (m = 1e5 queries, n = 1e7 points, d = 128, k = 100, 8 GB limit);
c1, c2, c3 and c5 (with its sweep over four memory limits) follow as sub-records under
"configs", each with its own time, kernel times, roofline, oracle timing and parity.

Prints ONE JSON line: pairs/s for the whole job, the roofline of the dominant kernel
(measured live with HIP events on the launch stream), the matrix-core peak measured on the
same GPU, and the CPU oracle timed on the host cores on a bounded sample of the same workload
(reported baseline, also a parity check).
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.join(ROOT, "tests"))

# published MI355X peaks
PEAK_BF16_MATRIX_TFLOPS = 2500.0  # dense bf16 MFMA, MI355X published
PEAK_FP32_MATRIX_TFLOPS = 157.3
PEAK_FP32_VECTOR_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

# HBM-side bytes per launch of the dominant kernel from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs,
# scaled by the copy-kernel calibration stated in the profile.  They describe the default shape of
# a workload on the kernel named; a run with other sizes, another limit or another kernel reports
# null.  {workload: (kernel, bytes, profile)}
PROFILED_TRAFFIC = {
    "c1_random_d16": ("knn_split_kernel", 11.8e6, "profiles/knn_split_kernel_c1.md"),
    "c2_pointcloud_d3": ("knn_lowd_bf16_kernel", 211.4e9, "profiles/knn_lowd_bf16_kernel_c2.md"),
    "c3_imagelike_d784": ("knn_wide_kernel", 50.6e9, "profiles/knn_wide_kernel_c3.md"),
    "c4_clustered_d128": ("knn_packed_kernel", 435.6e9, "profiles/knn_packed_kernel_c4.md"),
    "c5_memsweep_d256": ("knn_packed_kernel", 15.2e9, "profiles/knn_packed_kernel_c5_1GB.md"),  # per launch, two a step
    "c6_cosine_d100": ("knn_packed_kernel", 8.37e9, "profiles/knn_packed_kernel_c6.md"),
    "c7_l1_d100": ("knn_l1_kernel", 25.8e9, "profiles/knn_l1_kernel_c7.md"),
    "kmv1_d1": ("kmv_lowd_kernel", 1.84e9, "profiles/kmv_lowd_kernel_kmv1.md"),
    "kmv2_d32": ("kmv_mfma_kernel", 1.47e9, "profiles/kmv_mfma_kernel_kmv2.md"),
    "kmv3_d1_f64": ("kmv_lowd_f64_kernel", 4.02e9, "profiles/kmv_lowd_f64_kernel_kmv3.md"),
    "sgpr1_road_d3_m10000": ("sgpr_syrk_kernel", 8.99e9, "profiles/sgpr_syrk_kernel_sgpr1.md"),
}


def profiled_traffic(name: str, kernel: str, default_shape: bool):
    """(bytes, source) of the committed counter profile, only where it describes this run."""
    rec = PROFILED_TRAFFIC.get(name)
    if rec is None or not default_shape or rec[0] != kernel:
        return None, None
    return rec[1], rec[2]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def bench_kmv(args) -> int:
    """--workload kmv1 / kmv2: one step = one kmv_apply call (y = K v, squared-exponential K)."""
    import numpy as np
    import torch

    import paper_2206_14148_amd as K
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    K.load()
    w = W.scaled_kmv(args.workload, n=args.n, m=args.m) if (args.n or args.m) \
        else W.KMV_WORKLOADS[args.workload]
    limit = K.knn_parse_size(args.mem_limit) if args.mem_limit else w.mem_limit
    t0 = time.time()
    X, Z, v = W.make_kmv(w)
    log(f"[bench] inputs {w.name}: n={w.n} m={w.m} d={w.d} generated in {time.time()-t0:.1f}s")
    dev = torch.device("cuda:0")
    Xd = torch.from_numpy(X).to(dev)
    Zd = Xd if w.z_is_x else torch.from_numpy(Z).to(dev)
    vd = torch.from_numpy(v).to(dev)
    plan = K.kmv_plan(w.n, w.m, w.d, limit, w.dtype)
    assert plan.workspace_bytes <= limit
    ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device=dev)
    y = torch.empty((w.n,), dtype=torch.float64, device=dev)
    path_name = {0: "lowd", 1: "mfma", 2: "valu"}[plan.path]
    okmv = (lambda *a, **k: __import__("oracle").kmv_f64(*a, **k)) if w.dtype == "f64" \
        else (lambda *a, **k: __import__("oracle").kmv(*a, **k))
    log(f"[bench] plan: path={path_name} ranges={plan.n_splits} workspace={plan.workspace_bytes} B "
        f"(limit {limit} B)")

    def step():
        K.kmv_apply(Xd, Zd, vd, w.variance, w.lengthscale, limit, workspace=ws, out=y)

    if args.calibrate_copy_mb > 0:
        src = torch.ones(args.calibrate_copy_mb * 250_000, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)  # one elementwise kernel: reads and writes calibrate_copy_mb MB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    K.knn_profile_enable(True)  # HIP events around the main kernel, on the launch stream
    K.knn_profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    _, main_ms, _, launches = K.knn_profile_read()
    K.knn_profile_enable(False)
    call_ms = main_ms / max(launches, 1)
    ms_per_step = elapsed * 1e3 / args.steps
    pairs = float(w.n) * float(w.m)
    value = pairs * args.steps / elapsed
    log(f"[bench] {ms_per_step:.2f} ms/step, {value:.3e} pairs/s; kernels per call {call_ms:.3f} ms")
    rate = pairs / (call_ms * 1e-3)
    if w.dtype == "f64":
        # per pair: d subtractions, d multiply-adds, the scaling, exp (a polynomial of about 25
        # fp64 operations in the math library, counted as one flop here) and the multiply-add
        fpp = 3 * w.d + 3
        roofline = {"bound": "alu", "kernel": "kmv_lowd_f64_kernel" if w.d <= 8 else "kmv_anyd_f64_kernel",
                    "achieved": rate * fpp / 1e12, "peak": 78.6, "unit": "TFLOP/s",
                    "frac": rate * fpp / 1e12 / 78.6, "traffic": None, "flops_per_pair": fpp}
    elif plan.path == K.KMV_PATH_LOWD:
        # per pair: d subtractions, d multiplications, d-1 additions, the scaling, exp2, and
        # the multiply-add with v
        fpp = 3 * w.d + 3
        # issue slots per pair on a 16-lane SIMD: 2d + 2 full-rate operations and one
        # half-rate exp2 (measured on this chip: 4 and 8 cycles per wave instruction)
        slots = 2 * w.d + 2 + 2
        roofline = {"bound": "alu", "kernel": "kmv_lowd_kernel", "achieved": rate * fpp / 1e12,
                    "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                    "frac": rate * fpp / 1e12 / PEAK_FP32_VECTOR_TFLOPS, "traffic": None,
                    "flops_per_pair": fpp,
                    "issue_frac": rate * slots / (256 * 4 * 16 * 2.4e9)}
    else:
        # the contraction runs as six bf16 MFMAs per 16 coordinates (three-piece splits of the
        # fp32 values): 12 bf16 flops per pair and padded coordinate, priced at the bf16 peak
        # headline: the method's own contraction, 2 d flops per pair, against the bf16 peak; the
        # twelve bf16 flops per pair and padded coordinate that the three-piece emulation really
        # issues are reported beside it as `issued_*`
        d_pad = (w.d + 15) // 16 * 16
        fpp = 2 * w.d
        roofline = {"bound": "mfma", "kernel": "kmv_mfma_kernel", "achieved": rate * fpp / 1e12,
                    "peak": PEAK_BF16_MATRIX_TFLOPS, "unit": "TFLOP/s",
                    "frac": rate * fpp / 1e12 / PEAK_BF16_MATRIX_TFLOPS, "traffic": None,
                    "flops_per_pair": fpp, "issued_flops_per_pair": 12 * d_pad,
                    "issued_tflops": rate * 12 * d_pad / 1e12,
                    "issued_frac": rate * 12 * d_pad / 1e12 / PEAK_BF16_MATRIX_TFLOPS}
    roofline["traffic"], roofline["traffic_source"] = profiled_traffic(
        w.name, roofline["kernel"], not (args.n or args.m or args.mem_limit))
    roofline["avg_launch_ms"] = call_ms

    cpu_baseline = None
    parity = None
    if args.cpu_seconds > 0:
        import oracle

        threads = oracle.threads_used()
        rng = np.random.Generator(np.random.PCG64(11))
        probe = np.sort(rng.choice(w.n, size=min(w.n, 4 * threads), replace=False))
        t0 = time.perf_counter()
        okmv(X, Z, v, w.variance, w.lengthscale, rows=probe)
        probe_rate = len(probe) / max(time.perf_counter() - t0, 1e-6)
        nrows = int(max(len(probe), min(w.n, probe_rate * args.cpu_seconds)))
        rows = np.sort(rng.choice(w.n, size=nrows, replace=False))
        t0 = time.perf_counter()
        ref = okmv(X, Z, v, w.variance, w.lengthscale, rows=rows)
        dt = time.perf_counter() - t0
        cpu_baseline = {"value": len(rows) * float(w.m) / dt, "unit": "pairs/s", "cores": threads,
                        "kind": "oracle",
                        "sample": f"{len(rows)} seeded rows of K x all {w.m} points of {w.name}, {dt:.1f} s"}
        got = y[torch.from_numpy(rows).to(dev)].cpu().numpy()
        mag = okmv(X, Z, np.abs(v), w.variance, w.lengthscale, rows=rows)
        rel = float((np.abs(got - ref) / np.maximum(mag, 1e-300)).max())
        parity = {"rows": len(rows), "max_abs_err_over_sum_of_magnitudes": rel}
        log(f"[bench] oracle: {cpu_baseline['value']:.3e} pairs/s on {threads} threads; parity {parity}")

    # the memory-limit sweep of the paper's figure 1 (section 5.1), on this product: same inputs,
    # a range of limits; the workspace stays under each of them
    sweep = []
    if not args.mem_limit:
        for lim in (0 if plan.path != K.KMV_PATH_MFMA else plan.norms_bytes, 10 ** 6, 10 ** 8, 10 ** 9, 32 * 10 ** 9):
            p2 = K.kmv_plan(w.n, w.m, w.d, lim, w.dtype)
            ws2 = torch.empty(max(p2.workspace_bytes, 256), dtype=torch.uint8, device=dev)
            y2 = torch.empty_like(y)
            K.kmv_apply(Xd, Zd, vd, w.variance, w.lengthscale, lim, workspace=ws2, out=y2)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.steps):
                K.kmv_apply(Xd, Zd, vd, w.variance, w.lengthscale, lim, workspace=ws2, out=y2)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / args.steps
            sweep.append({"mem_limit_bytes": lim, "workspace_bytes": p2.workspace_bytes,
                          "point_ranges": p2.n_splits, "ms_per_step": dt * 1e3,
                          "max_abs_diff": float((y2 - y).abs().max())})
            log(f"[bench] sweep limit={lim}: {dt*1e3:.1f} ms, workspace {p2.workspace_bytes} B, "
                f"ranges {p2.n_splits}")
            del ws2, y2

    out = {
        "metric": "kernel-matrix entries per second, y = K v with a squared-exponential kernel (n*m/s)",
        "value": value, "unit": "pairs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "n": w.n, "m": w.m, "d": w.d, "variance": w.variance,
                   "lengthscale": w.lengthscale, "mem_limit_bytes": limit,
                   "workspace_bytes": plan.workspace_bytes, "point_ranges": plan.n_splits,
                   "path": path_name},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "parity": parity,
    }
    if sweep:
        out["mem_limit_sweep"] = sweep
    print(json.dumps(out), flush=True)
    return 0


def bench_sgpr(args) -> int:
    """--workload sgpr1 / sgpr2: one step = one sgpr_accumulate call (A = K_uf K_fu, b = K_uf y)."""
    import numpy as np
    import torch

    import paper_2206_14148_amd as K
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    K.load()
    w = W.SGPR_WORKLOADS[args.workload]
    if args.m or args.n:
        from dataclasses import replace
        w = replace(w, m=args.m or w.m, n=args.n or w.n)
    limit = K.knn_parse_size(args.mem_limit) if args.mem_limit else w.mem_limit
    t0 = time.time()
    U, X, y = W.make_sgpr(w)
    log(f"[bench] inputs {w.name}: m={w.m} n={w.n} d={w.d} generated in {time.time()-t0:.1f}s")
    dev = torch.device("cuda:0")
    Ud, Xd, yd = (torch.from_numpy(a).to(dev) for a in (U, X, y))
    plan = K.sgpr_plan(w.m, w.n, w.d, limit)
    assert plan.workspace_bytes <= limit
    ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device=dev)
    A = torch.empty((w.m, w.m), dtype=torch.float64, device=dev)
    b = torch.empty((w.m,), dtype=torch.float64, device=dev)
    log(f"[bench] plan: {plan.n_chunks} chunks of {plan.chunk_cols} data points, "
        f"workspace={plan.workspace_bytes} B (limit {limit} B)")

    def step():
        K.sgpr_accumulate(Ud, Xd, yd, w.variance, w.lengthscale, limit, workspace=ws, out=(A, b))

    if args.calibrate_copy_mb > 0:
        src = torch.ones(args.calibrate_copy_mb * 250_000, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)  # one elementwise kernel: reads and writes calibrate_copy_mb MB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    K.knn_profile_enable(True)
    K.knn_profile_read()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    kuf_ms, syrk_ms, kufy_ms, launches = K.knn_profile_read()
    K.knn_profile_enable(False)
    ms_per_step = elapsed * 1e3 / args.steps
    pairs = float(w.m) * float(w.n)
    value = pairs * args.steps / elapsed
    log(f"[bench] {ms_per_step:.2f} ms/step, {value:.3e} kernel entries/s; kernels per step: K_uf chunks "
        f"{kuf_ms/args.steps:.2f} ms, chunk products {syrk_ms/args.steps:.2f} ms ({launches // max(args.steps, 1)} "
        f"launches), times y {kufy_ms/args.steps:.2f} ms")
    # dominant kernel: the chunk product.  Algorithmic flops: the lower triangle of A once,
    # n * m * (m + 1) for the whole job, spread over the launches.
    avg_launch_s = syrk_ms / max(launches, 1) * 1e-3
    flops_per_launch = float(w.flops) * args.steps / max(launches, 1)
    achieved = flops_per_launch / avg_launch_s / 1e12
    roofline = {"bound": "mfma", "kernel": "sgpr_syrk_kernel", "achieved": achieved,
                "peak": PEAK_FP32_MATRIX_TFLOPS, "unit": "TFLOP/s",
                "frac": achieved / PEAK_FP32_MATRIX_TFLOPS,
                "traffic": None, "flops_per_pair": w.m + 1, "avg_launch_ms": avg_launch_s * 1e3}
    roofline["traffic"], roofline["traffic_source"] = profiled_traffic(
        w.name, "sgpr_syrk_kernel", not (args.n or args.m or args.mem_limit))

    cpu_baseline = None
    parity = None
    if args.cpu_seconds > 0:
        import oracle

        threads = oracle.threads_used()
        g = np.random.Generator(np.random.PCG64(12))
        count = 4 * threads
        ii, jj = g.integers(0, w.m, count), g.integers(0, w.m, count)
        t0 = time.perf_counter()
        oracle.sgpr_entries(U, X, ii[:threads], jj[:threads], w.variance, w.lengthscale)
        per_entry = (time.perf_counter() - t0) / 1.0  # one entry per thread in parallel
        count = int(max(threads, min(4096, threads * args.cpu_seconds / max(per_entry, 1e-6))))
        ii, jj = g.integers(0, w.m, count), g.integers(0, w.m, count)
        t0 = time.perf_counter()
        ref = oracle.sgpr_entries(U, X, ii, jj, w.variance, w.lengthscale)
        dt = time.perf_counter() - t0
        # an entry of A costs the oracle 2 n kernel evaluations; its rate in the metric's unit
        # is the rate at which it would cover the m n entries of K_uf while summing the
        # (m + 1) / 2 products each of them takes part in
        entry_rate = count / dt
        cpu_baseline = {"value": entry_rate * w.n / ((w.m + 1) / 2.0), "unit": "pairs/s",
                        "cores": threads, "kind": "oracle",
                        "sample": f"{count} seeded entries of A, each summed over all {w.n} data points of "
                                  f"{w.name}, {dt:.1f} s; scaled by the m(m+1)/2 entries of the triangle"}
        got = A[torch.from_numpy(ii).to(dev), torch.from_numpy(jj).to(dev)].cpu().numpy()
        parity = {"entries": count, "max_rel_err": float((np.abs(got - ref) / ref).max())}
        log(f"[bench] oracle: {cpu_baseline['value']:.3e} pairs/s on {threads} threads; parity {parity}")

    out = {
        "metric": "kernel-matrix entries per second through A = K_uf K_fu and b = K_uf y (m*n/s)",
        "value": value, "unit": "pairs/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "m": w.m, "n": w.n, "d": w.d, "variance": w.variance,
                   "lengthscale": w.lengthscale, "mem_limit_bytes": limit,
                   "workspace_bytes": plan.workspace_bytes, "chunk_cols": plan.chunk_cols,
                   "n_chunks": plan.n_chunks},
        "kernel_ms_per_step": {"kuf": kuf_ms / args.steps, "syrk": syrk_ms / args.steps,
                               "kufy": kufy_ms / args.steps},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "parity": parity,
    }
    print(json.dumps(out), flush=True)
    return 0


PATH_NAMES = {0: "lowd", 2: "lowd_mfma", 3: "l1", 4: "lowd_bf16", 5: "mfma_split", 6: "mfma_packed", 7: "mfma_wide"}
# arithmetic the path computes in: what the matrix cores filter in, what the list keys are, what the
# returned distances are evaluated in
PATH_DTYPES = {0: "f32 keys / f64 refine", 3: "f32 keys / f64 refine",
               2: "f32 filter / f32 keys / f64 refine", 4: "bf16 filter / f32 keys / f64 refine",
               5: "bf16 filter / f32 keys / f64 refine", 6: "bf16 filter / f32 keys / f64 refine",
               7: "bf16 filter / f32 keys / f64 refine"}


def knn_record(w, limit, steps, warmup, cpu_seconds, peaks, default_shape, host_x=False,
               calibrate_copy_mb=0, sweep=True):
    """Times one kNN workload; returns the record (the top-level fields of a bench line)."""
    import numpy as np
    import torch

    import paper_2206_14148_amd as K
    import workloads as W

    t0 = time.time()
    Q, X = W.make(w)
    log(f"[bench] inputs {w.name}: m={w.m} n={w.n} d={w.d} k={w.k} generated in {time.time()-t0:.1f}s")
    dev = torch.device("cuda:0")
    Xd = torch.from_numpy(X).to(dev)
    Qd = Xd if w.q_is_x else torch.from_numpy(Q).to(dev)
    plan = K.knn_plan(w.m, w.n, w.d, w.k, limit, w.metric)
    assert plan.workspace_bytes <= limit
    ws = torch.empty(max(plan.workspace_bytes, 256), dtype=torch.uint8, device=dev)
    idx = torch.empty((w.m, w.k), dtype=torch.int32, device=dev)
    dist = torch.empty((w.m, w.k), dtype=torch.float32, device=dev)
    path_name = PATH_NAMES[plan.path]
    log(f"[bench] plan: path={path_name} chunks={plan.q_chunks} ranges={plan.n_splits} "
        f"tile={plan.tile_q} workspace={plan.workspace_bytes} B (limit {limit} B)")

    def step():
        K.knn_search(Qd, Xd, w.k, limit, workspace=ws, out=(idx, dist), metric=w.metric)

    if calibrate_copy_mb > 0:
        src = torch.ones(calibrate_copy_mb * 250_000, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        torch.mul(src, 1.0, out=dst)  # one elementwise kernel: reads and writes calibrate_copy_mb MB
        torch.cuda.synchronize()
        del src, dst
    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    K.knn_profile_enable(True)
    K.knn_profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        step()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prep_ms, search_ms, refine_ms, launches = K.knn_profile_read()
    K.knn_profile_enable(False)
    ms_per_step = elapsed * 1e3 / steps
    pairs = float(w.m) * float(w.n)
    value = pairs * steps / elapsed
    log(f"[bench] {w.name}: {ms_per_step:.2f} ms/step, {value:.3e} pairs/s; kernels per step: "
        f"preparation {prep_ms/steps:.3f} ms, search {search_ms/steps:.3f} ms "
        f"({launches // max(steps,1)} launch), merge+refine {refine_ms/steps:.3f} ms")

    # roofline of the dominant kernel, per launch
    avg_launch_s = (search_ms / max(launches, 1)) * 1e-3
    launches_per_step = max(launches, 1) / steps
    pairs_per_launch = float(w.m) * float(w.n) / launches_per_step
    hbm_equiv = (pairs_per_launch / avg_launch_s) * 8.0 / (PEAK_HBM_GBS * 1e9)
    if plan.path in (K.KNN_PATH_MFMA_SPLIT, K.KNN_PATH_MFMA_PACKED, K.KNN_PATH_MFMA_WIDE):
        # The -2 Q X^T contraction of the filter runs on bf16 roundings of the values: 2 d bf16
        # flops per pair on the matrix cores, with d rounded up to the 16 coordinates of an MFMA,
        # against the dense bf16 peak.
        kernel = {K.KNN_PATH_MFMA_SPLIT: "knn_split_kernel", K.KNN_PATH_MFMA_PACKED: "knn_packed_kernel",
                  K.KNN_PATH_MFMA_WIDE: "knn_wide_kernel"}[plan.path]
        d_pad = (w.d + 15) // 16 * 16
        achieved = 2.0 * d_pad * pairs_per_launch / avg_launch_s / 1e12
        roofline = {"bound": "mfma", "kernel": kernel, "achieved": achieved,
                    "peak": PEAK_BF16_MATRIX_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_BF16_MATRIX_TFLOPS, "flops_per_pair": 2 * d_pad}
        if peaks.get("bf16"):
            roofline["measured_peak"] = peaks["bf16"]
            roofline["frac_of_measured_peak"] = achieved / peaks["bf16"]
    elif plan.path == K.KNN_PATH_LOWD_MFMA:
        # filter contraction over K = 4: [x0 x1 x2 |x|^2] . [-2q0 -2q1 -2q2 1]
        achieved = 8.0 * pairs_per_launch / avg_launch_s / 1e12
        roofline = {"bound": "mfma", "kernel": "knn_lowd_mfma_kernel", "achieved": achieved,
                    "peak": PEAK_FP32_MATRIX_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_FP32_MATRIX_TFLOPS, "flops_per_pair": 8,
                    # what a design that stores the distance tile would move: 4 B out + 4 B in
                    "hbm_equiv_frac": hbm_equiv}
        if peaks.get("f32"):
            roofline["measured_peak"] = peaks["f32"]
            roofline["frac_of_measured_peak"] = achieved / peaks["f32"]
    elif plan.path == K.KNN_PATH_LOWD_BF16:
        # Bound: instruction issue of one wave.  Per 32 x 32 keys a wave issues one
        # v_mfma_f32_32x32x16_bf16 (8 passes = the slot of 8 vector instructions) and 9 vector
        # instructions (8 three-input minima, 1 compare): 17 slots x 64 lanes / 1024 pairs =
        # 1.0625 lane-operations per pair against 256 CUs x 4 SIMDs x 16 lanes x 2.4 GHz.  The
        # unit is issue slots of one lane, not flops.
        lane_ops = 17.0 * 64.0 / 1024.0
        peak = 256 * 4 * 16 * 2.4e9 / 1e12
        achieved = lane_ops * pairs_per_launch / avg_launch_s / 1e12
        roofline = {"bound": "alu", "kernel": "knn_lowd_bf16_kernel", "achieved": achieved,
                    "peak": peak, "unit": "Tlane-op/s", "frac": achieved / peak,
                    "unit_note": "issue slots of the vector ALU / matrix core port per lane and second",
                    "lane_ops_per_pair": lane_ops,
                    # the filter contraction alone: 2 x 16 bf16 flops per pair against 2.5 PFLOP/s
                    "mfma_bf16_frac": 32.0 * pairs_per_launch / avg_launch_s / 2.5e15,
                    # what a design that stores the distance tile would move: 4 B out + 4 B in
                    "hbm_equiv_frac": hbm_equiv}
    elif plan.path == K.KNN_PATH_L1:
        # d subtractions and d-1 additions per pair (the absolute value is an operand modifier)
        achieved = (2.0 * w.d - 1.0) * pairs_per_launch / avg_launch_s / 1e12
        roofline = {"bound": "alu", "kernel": "knn_l1_kernel", "achieved": achieved,
                    "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_FP32_VECTOR_TFLOPS, "flops_per_pair": 2 * w.d - 1}
    else:
        # difference form: d subtractions, d multiplications, d-1 additions per pair
        achieved = (3.0 * w.d - 1.0) * pairs_per_launch / avg_launch_s / 1e12
        roofline = {"bound": "alu", "kernel": "knn_lowd_kernel", "achieved": achieved,
                    "peak": PEAK_FP32_VECTOR_TFLOPS, "unit": "TFLOP/s",
                    "frac": achieved / PEAK_FP32_VECTOR_TFLOPS,
                    "flops_per_pair": 3 * w.d - 1, "hbm_equiv_frac": hbm_equiv}
    roofline["traffic"], roofline["traffic_source"] = profiled_traffic(w.name, roofline["kernel"],
                                                                       default_shape)
    roofline["avg_launch_ms"] = avg_launch_s * 1e3
    roofline["algorithmic_bytes"] = 4.0 * (w.m + w.n) * w.d + 8.0 * w.m * w.k

    cpu_baseline = None
    parity = None
    if cpu_seconds > 0:
        import oracle
        from parity import check

        threads = oracle.threads_used()
        probe_rows = W.sample_rows(w, min(w.m, 4 * threads))
        t0 = time.perf_counter()
        oracle.knn(Q, X, w.k, rows=probe_rows, metric=w.metric)
        probe_rate = len(probe_rows) / max(time.perf_counter() - t0, 1e-6)
        nrows = int(max(len(probe_rows), min(w.m, probe_rate * cpu_seconds)))
        rows = W.sample_rows(w, nrows)
        t0 = time.perf_counter()
        o_idx, o_dist, o_next = oracle.knn(Q, X, w.k, rows=rows, metric=w.metric)
        dt = time.perf_counter() - t0
        cpu_baseline = {"value": len(rows) * float(w.n) / dt, "unit": "pairs/s", "cores": threads,
                        "kind": "oracle",
                        "sample": f"{len(rows)} seeded query rows x all {w.n} points of {w.name}, {dt:.1f} s"}
        rows_t = torch.from_numpy(rows).to(dev)
        parity = check(idx[rows_t].cpu().numpy(), dist[rows_t].cpu().numpy(), o_idx, o_dist, o_next, w.n)
        log(f"[bench] oracle: {cpu_baseline['value']:.3e} pairs/s on {threads} threads; parity {parity}")

    # the memory-limit sweep of the sweep workload (config 5): same inputs, each of its limits, and
    # one limit small enough to cut the queries into several chunks
    sweep_out = None
    if w.sweep and sweep:
        sweep_out = []
        # (the smallest limit, in steps of a quarter above the minimum, that takes 2 to 8 chunks)
        small = K.knn_plan(w.m, w.n, w.d, w.k, 1 << 44, w.metric).min_limit_bytes
        for _ in range(40):
            if 2 <= K.knn_plan(w.m, w.n, w.d, w.k, small, w.metric).q_chunks <= 8:
                break
            small = small * 5 // 4
        for lim in (small,) + tuple(w.sweep):
            p2 = K.knn_plan(w.m, w.n, w.d, w.k, lim, w.metric)
            ws2 = torch.empty(max(p2.workspace_bytes, 256), dtype=torch.uint8, device=dev)
            i2 = torch.empty_like(idx)
            d2 = torch.empty_like(dist)
            K.knn_search(Qd, Xd, w.k, lim, workspace=ws2, out=(i2, d2))  # warm-up
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps):
                K.knn_search(Qd, Xd, w.k, lim, workspace=ws2, out=(i2, d2))
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / steps
            sweep_out.append({"mem_limit_bytes": lim, "workspace_bytes": p2.workspace_bytes,
                              "path": PATH_NAMES[p2.path], "q_chunks": p2.q_chunks,
                              "point_ranges": p2.n_splits, "ms_per_step": dt * 1e3,
                              "pairs_per_s": pairs / dt,
                              "same_result": bool(torch.equal(i2, idx) and torch.equal(d2, dist))})
            log(f"[bench] sweep limit={lim}: {dt*1e3:.1f} ms, {pairs/dt:.3e} pairs/s, path "
                f"{PATH_NAMES[p2.path]}, {p2.q_chunks} chunks, workspace {p2.workspace_bytes} B, "
                f"same result: {sweep_out[-1]['same_result']}")
            del ws2, i2, d2

    host_streamed = None
    if host_x:
        hp = K.knn_plan_host_x(w.m, w.n, w.d, w.k, limit, w.metric)
        Xp = torch.from_numpy(X).pin_memory()
        ws3 = torch.empty(max(hp.workspace_bytes, 256), dtype=torch.uint8, device=dev)
        i3 = torch.empty_like(idx)
        d3 = torch.empty_like(dist)
        K.knn_search_host_x(Qd, Xp, w.k, limit, workspace=ws3, out=(i3, d3), metric=w.metric)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            K.knn_search_host_x(Qd, Xp, w.k, limit, workspace=ws3, out=(i3, d3), metric=w.metric)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        host_streamed = {"ms_per_step": dt * 1e3, "pairs_per_s": pairs / dt,
                         "h2d_GB_per_s": X.nbytes / dt / 1e9, "x_bytes": X.nbytes,
                         "n_blocks": hp.n_blocks, "block_rows": hp.block_rows,
                         "workspace_bytes": hp.workspace_bytes,
                         "same_distances": bool(torch.equal(d3, dist)),
                         "same_indices_fraction": float((i3 == idx).float().mean())}
        log(f"[bench] host-streamed X: {dt*1e3:.1f} ms/step, {pairs/dt:.3e} pairs/s, "
            f"{X.nbytes/dt/1e9:.1f} GB/s over the host link, {hp.n_blocks} blocks of {hp.block_rows}")
        del ws3, i3, d3, Xp

    rec = {
        "metric": "query-point pairs per second, exact brute-force kNN (m*n/s)",
        "value": value, "unit": "pairs/s", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": PATH_DTYPES[plan.path], "data": "synthetic",
        "config": {"workload": w.name, "metric": w.metric, "m": w.m, "n": w.n, "d": w.d, "k": w.k,
                   "mem_limit_bytes": limit, "workspace_bytes": plan.workspace_bytes,
                   "q_chunks": plan.q_chunks, "point_ranges": plan.n_splits,
                   "queries_per_workgroup": plan.tile_q, "seed_points": plan.seed_points,
                   "path": path_name},
        "kernel_ms_per_step": {"preparation": prep_ms / steps, "search": search_ms / steps,
                               "merge_refine": refine_ms / steps},
        "roofline": roofline, "cpu_baseline": cpu_baseline, "parity": parity,
    }
    if sweep_out is not None:
        rec["mem_limit_sweep"] = sweep_out
    if host_streamed is not None:
        rec["host_streamed_x"] = host_streamed
    del Xd, Qd, ws, idx, dist
    torch.cuda.empty_cache()
    return rec


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="all",
                    help="all (default: c4 as the top-level record, c1, c2, c3, c5 as sub-records), or one of "
                         "c1..c7 (c6 cosine, c7 L1), kmv1 / kmv2 / kmv3 (the kernel matrix-vector product), "
                         "sgpr1 / sgpr2 (the SGPR accumulations)")
    ap.add_argument("--mem-limit", default=None, help="e.g. 128MB, 1GB (decimal); default: the workload's")
    ap.add_argument("--m", type=int, default=None, help="override the query count (testing)")
    ap.add_argument("--n", type=int, default=None, help="override the point count (testing)")
    ap.add_argument("--k", type=int, default=None, help="override the neighbour count (testing)")
    ap.add_argument("--cpu-seconds", type=float, default=12.0,
                    help="oracle time budget of the top-level record (sub-records get a third); 0 skips it")
    ap.add_argument("--host-x", action="store_true",
                    help="also time knn_search_host_x: the same search with X in pinned host memory, "
                         "streamed through staging buffers inside the limit (PCIe-inclusive; reported "
                         "beside the resident figure, never as `value`)")
    ap.add_argument("--calibrate-copy-mb", type=int, default=0,
                    help="also run one plain elementwise copy of this many MB (read + write) before "
                         "the timed region, as the known-size reference for rocprofv3 --pmc byte counters")
    ap.add_argument("--no-peak", action="store_true", help="skip the MFMA-only peak measurement")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU; run with --gpus 1 "
              "(more GPUs would each take a share of the query rows; that is not built)", file=sys.stderr)
        return 2

    if args.workload.startswith("kmv"):
        return bench_kmv(args)
    if args.workload.startswith("sgpr"):
        return bench_sgpr(args)

    import torch

    import paper_2206_14148_amd as K
    import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the HIP path has no CPU fallback", file=sys.stderr)
        return 2
    K.load()
    peaks = {}
    if not args.no_peak:
        peaks = {"bf16": K.knn_measure_mfma_peak("bf16"), "f32": K.knn_measure_mfma_peak("f32")}
        log(f"[bench] MFMA-only loops on this GPU: bf16 {peaks['bf16']:.0f} TFLOP/s "
            f"(published 2500), f32 {peaks['f32']:.1f} TFLOP/s (published 157.3)")

    def one(cfg: int, steps: int, cpu_seconds: float, overrides: bool):
        w = W.WORKLOADS[cfg]
        default_shape = True
        if overrides and (args.m or args.n):
            w = W.scaled(cfg, m=args.m, n=args.n)
            default_shape = False
        if overrides and args.k:
            w = W.scaled(cfg, m=w.m, n=w.n, k=args.k)
            default_shape = False
        limit = w.mem_limit
        if overrides and args.mem_limit:
            limit = K.knn_parse_size(args.mem_limit)
            default_shape = False
        return knn_record(w, limit, steps, args.warmup, cpu_seconds, peaks, default_shape,
                          host_x=args.host_x and overrides, calibrate_copy_mb=args.calibrate_copy_mb if overrides else 0,
                          sweep=not (overrides and args.mem_limit))

    if args.workload == "all":
        out = one(4, args.steps, args.cpu_seconds, False)
        out["configs"] = {}
        for cfg in (1, 2, 3, 5):
            out["configs"][f"c{cfg}"] = one(cfg, max(args.steps, 5), args.cpu_seconds / 3.0, False)
    else:
        out = one(int(args.workload.lstrip("c")), args.steps, args.cpu_seconds, True)
    if peaks:
        out["measured_mfma_peak_tflops"] = peaks
    print(json.dumps(out), flush=True)
    return 0


if __name__ == "__main__":
    sys.exit(main())
