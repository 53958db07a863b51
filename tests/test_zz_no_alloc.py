"""gd_update_ledger_static -- the entry point for callers that cannot allocate -- against
gd_update_ledger through the C ABI: same histories, two calls in a row (the second
shorter than the first), every read-out of the ledger equal bit for bit, and both equal
to the oracle's.  Collected last: a failure here hides no other test."""
import numpy as np
import pytest
import torch

import oracle
from gpu_harness import detector_for, oracle_params
from paper_2605_17879_amd.guard import GuardError
from test_gpu_ledger import compare_ledger, oracle_ledger, read_ledger, say
from workloads.histories import exceed_history, node_score_history

pytestmark = pytest.mark.gpu

CASES = [
    # R, M, W, k, first batch, second batch
    (1024, 4, 50, 40, 1200, 70),        # ten chunks, then a single one (no staged counts)
    (16384, 4, 100, 80, 900, 450),      # several chunks both times
    (65536, 8, 256, 200, 1100, 300),    # the benchmark's shape
]


@pytest.mark.parametrize("R,M,W,k,T1,T2", CASES)
def test_static_work_area_gives_the_same_ledger(R, M, W, k, T1, T2):
    say(f"case static ledger R={R} M={M} W={W} k={k} batches={[T1, T2]}")
    N, T = R // 8, T1 + T2
    p = oracle_params(R=R, M=M, W=W, k=k, primary=1 % M, min_signals=min(2, M), directions=(1,) * M)
    bursts = (max(2, W // 2), 3 * W + 5)
    exceed = exceed_history(R + T1, T, R, M, 0.03, burst_items=max(4, R // 50), burst_len=bursts,
                            gap_len=(1, 2 * W + 3), burst_metrics=M)
    node_mask = exceed_history(R + T1 + 1, T, N, M, 0.03, burst_items=max(3, N // 8), burst_len=bursts,
                               gap_len=(1, 2 * W + 3), burst_metrics=M)
    node_z = node_score_history(R + T2, T, N, scale=3.0)
    e, n, z = (torch.from_numpy(a).cuda() for a in (exceed, node_mask, node_z))
    horizon, limit, topk_k = 3 * W, 2, min(64, N)

    ref = detector_for(p)
    ref.alloc_ledger(max(T1, T2), recur_horizon=horizon, recur_limit=limit)
    new = detector_for(p)
    new.alloc_ledger(1, recur_horizon=horizon, recur_limit=limit)      # no work area of its own
    assert new.ledger_static_scratch_bytes() == 8 << 20
    t0 = 0
    for c in (T1, T2):
        batch = dict(exceed_mask=e[t0:t0 + c], node_mask=n[t0:t0 + c], node_z=z[t0:t0 + c])
        ref.update_ledger(batch, c)
        new.update_ledger_static(batch, c)
        t0 += c
        torch.cuda.synchronize()
        a, b = read_ledger(ref, topk_k), read_ledger(new, topk_k)
        for key in a:
            assert np.array_equal(a[key], b[key]), f"after {t0} steps: {key} differs between the two entry points"
    # and both are what the oracle says (sampled items at the largest size: every item is
    # independent of the others, and the oracle re-sums each window from scratch)
    ranks = nodes = None
    if R > 16384:
        rng = np.random.default_rng(3)
        ranks = np.unique(np.concatenate([[0, R - 1], rng.choice(R, 1022, replace=False)]))
        nodes = np.unique(np.concatenate([[0, N - 1], rng.choice(N, 510, replace=False)]))
    node_anom = oracle.combine(node_mask, p.primary, p.min_signals)
    want = oracle_ledger(p, exceed, node_mask, node_anom, node_z, 64.0, horizon, limit, topk_k,
                         ranks=ranks, nodes=nodes)
    compare_ledger(want, read_ledger(new, topk_k), f"static R{R}", ranks=ranks, nodes=nodes)
    assert (want["ranks"].first >= 0).any() and want["episodes"].any()
    ref.close()
    new.close()


def test_static_work_area_rejects_what_does_not_fit():
    R, M, W = 65536, 8, 256
    N = R // 8
    p = oracle_params(R=R, M=M, W=W, k=200, directions=(1,) * M)
    det = detector_for(p)
    det.alloc_ledger(1)
    T = 8000                                             # 8000 * 128 * 8 bytes of map alone: 7.8 MiB + counts
    e = torch.zeros((T, R), dtype=torch.uint8, device="cuda")
    n = torch.zeros((T, N), dtype=torch.uint8, device="cuda")
    z = torch.zeros((T, N), dtype=torch.float32, device="cuda")
    before = det.ledger.clone()
    with pytest.raises(GuardError) as err:
        det.update_ledger_static(dict(exceed_mask=e, node_mask=n, node_z=z), T)
    assert err.value.status == 1 and "static work area" in str(err.value)
    torch.cuda.synchronize()
    assert torch.equal(before, det.ledger), "a rejected call must launch nothing"
    det.update_ledger_static(dict(exceed_mask=e[:7000], node_mask=n[:7000], node_z=z[:7000]), 7000)   # fits
    torch.cuda.synchronize()
    det.close()
