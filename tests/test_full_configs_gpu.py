"""The five benchmark workloads at FULL size, in the launch configuration bench.py times,
checked on seeded sample rows that the oracle computes one by one (rows are independent,
so a row subset is exact row-level parity), plus properties that hold at any size."""
import sys
import time

import numpy as np
import pytest

import workloads as W
from parity import check

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")

# (the oracle does about 4e7 pairs/s at d = 784, 3e8 at d = 128, 1.2e8 at d = 256 on 16 threads:
# 10 to 15 seconds each for the three large shapes)
SAMPLE_ROWS = {1: 1000, 2: 2000, 3: 512, 4: 320, 5: 512, 6: 512, 7: 256}


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


@pytest.fixture(scope="module")
def K():
    import paper_2206_14148_amd as K
    assert torch.cuda.is_available()
    K.load()
    return K


@pytest.mark.parametrize("cfg", [1, 2, 3, 4, 5, 6, 7])
def test_full_size_workload(K, oracle, cfg):
    w = W.WORKLOADS[cfg]
    t0 = time.time()
    Q, X = W.make(w)
    say(f"\n{w.name}: m={w.m} n={w.n} d={w.d} k={w.k} generated in {time.time()-t0:.1f}s")
    Xd = torch.from_numpy(X).cuda()
    Qd = Xd if w.q_is_x else torch.from_numpy(Q).cuda()
    limits = w.sweep if w.sweep else (w.mem_limit,)
    results = []
    for limit in limits:
        plan = K.knn_plan(w.m, w.n, w.d, w.k, limit, w.metric)
        assert plan.workspace_bytes <= limit
        guard = 4096
        ws = torch.full((plan.workspace_bytes + guard,), 0x5A, dtype=torch.uint8, device="cuda")
        torch.cuda.synchronize()
        t0 = time.time()
        idx, dist = K.knn_search(Qd, Xd, w.k, limit, workspace=ws[: plan.workspace_bytes],
                                   metric=w.metric)
        torch.cuda.synchronize()
        dt = time.time() - t0
        assert bool((ws[plan.workspace_bytes:] == 0x5A).all()), "wrote past the planned workspace"
        _, peak = K.knn_last_stats()
        assert peak <= limit
        say(f"   limit={limit:>12d} B  workspace={plan.workspace_bytes} B  chunks={plan.q_chunks} "
            f"ranges={plan.n_splits}  {dt*1e3:.1f} ms  {w.m*w.n/dt:.3e} pairs/s")
        results.append((idx, dist))
        del ws
    for idx, dist in results[1:]:  # the limit must not change the answer
        assert torch.equal(idx, results[0][0]) and torch.equal(dist, results[0][1])
    idx, dist = results[0]

    # properties that hold at any size
    assert bool((dist[:, 1:] >= dist[:, :-1]).all())
    assert bool((dist >= 0).all())
    assert int(idx.min()) >= 0 and int(idx.max()) < w.n
    if w.q_is_x:
        assert bool((idx[:, 0] == torch.arange(w.m, device="cuda", dtype=torch.int32)).all())
        assert bool((dist[:, 0] == 0).all())

    rows = W.sample_rows(w, SAMPLE_ROWS[cfg])
    t0 = time.time()
    o_idx, o_dist, o_next = oracle.knn(Q, X, w.k, rows=rows, metric=w.metric)
    say(f"   oracle on {len(rows)} rows: {time.time()-t0:.1f}s")
    rt = torch.from_numpy(rows).cuda()
    stats = check(idx[rt].cpu().numpy(), dist[rt].cpu().numpy(), o_idx, o_dist, o_next, w.n)
    say("   parity", stats)
    assert stats["strict_rows"] >= 0.95 * stats["rows"]
