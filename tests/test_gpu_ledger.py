"""GPU parity of the ledger (persistence per indicator, windowed score sum and its
ranking, recurrence of flag episodes) through the C ABI: every output bit for bit
against the oracle on the same seeded histories -- whole histories in one call, cut
into batches of any length, step by step, and at the benchmark's full size on
sampled ranks and nodes."""
import sys

import numpy as np
import pytest
import torch

import oracle
from gpu_harness import detector_for, gpu_score, compare_scores, oracle_params
from workloads import generate, workload
from workloads.histories import exceed_history, node_score_history

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def oracle_ledger(p, exceed, node_mask, node_anom_words, node_z, quant, horizon, limit, topk_k,
                  ranks=None, nodes=None):
    """What the ledger must hold after the whole history (optionally only for some
    ranks / nodes: every item is independent of the others)."""
    if ranks is not None:
        exceed = np.ascontiguousarray(exceed[:, ranks])
    r = oracle.metric_window(exceed, p.primary, p.min_signals, p.W, p.k)
    nm = node_mask if nodes is None else np.ascontiguousarray(node_mask[:, nodes])
    n = oracle.metric_window(nm, p.primary, p.min_signals, p.W, p.k)
    pn = oracle.window(p.N, node_anom_words, p.W, p.k, want_hist=True)
    flag_hist = (pn.count_hist >= p.k).astype(np.uint8)
    ep, tf = oracle.recurrence(flag_hist, horizon, limit)
    qsum = oracle.score_ring(node_z, p.W, quant)
    idx, key = oracle.topk_mean(pn.count, qsum, topk_k)
    return dict(ranks=r, nodes=n, ccount=pn.count, episodes=ep, terminal=tf, qsum=qsum, idx=idx, key=key)


def read_ledger(det, topk_k):
    f = det.alloc_ledger_flags()
    for v in f.values():
        v.view(torch.uint8).fill_(0xA5)
    det.ledger_flags(f)
    tk = det.alloc_topk(topk_k)
    det.topk_nodes_mean(topk_k, tk)
    torch.cuda.synchronize()
    g = {k: v.cpu().numpy() for k, v in f.items()}
    g["idx"] = tk["idx"].cpu().numpy()
    g["key"] = tk["key"].cpu().numpy().view(np.uint64)
    return g


def compare_ledger(want, g, label, ranks=None, nodes=None):
    rs = slice(None) if ranks is None else ranks
    ns = slice(None) if nodes is None else nodes
    assert np.array_equal(g["rank_pmask"][rs], want["ranks"].pmask), f"{label}: rank sustained masks"
    assert np.array_equal(g["rank_pflag"][rs], want["ranks"].flag), f"{label}: rank flags"
    assert np.array_equal(g["rank_pfirst"][rs], want["ranks"].first), f"{label}: rank first steps"
    assert np.array_equal(g["node_pmask"][ns], want["nodes"].pmask), f"{label}: node sustained masks"
    assert np.array_equal(g["node_pflag"][ns], want["nodes"].flag), f"{label}: node flags"
    assert np.array_equal(g["node_pfirst"][ns], want["nodes"].first), f"{label}: node first steps"
    assert np.array_equal(g["node_score_sum"], want["qsum"]), f"{label}: score sums"
    assert np.array_equal(g["node_episodes"], want["episodes"]), f"{label}: episodes"
    assert np.array_equal(g["node_terminal_first"], want["terminal"]), f"{label}: terminal steps"
    assert np.array_equal(g["idx"], want["idx"]), f"{label}: ranking indices"
    assert np.array_equal(g["key"], want["key"]), f"{label}: ranking keys"


def feed(det, exceed, node_mask, node_z, batches):
    """gd_update_ledger on consecutive batches of the uploaded histories."""
    e, n, z = (torch.from_numpy(a).cuda() for a in (exceed, node_mask, node_z))
    t0 = 0
    for c in batches:
        if c:
            det.update_ledger(dict(exceed_mask=e[t0:t0 + c], node_mask=n[t0:t0 + c], node_z=z[t0:t0 + c]), c)
        t0 += c
    assert t0 == exceed.shape[0]
    torch.cuda.synchronize()


CASES = [
    # R, M, W, k, T, batches (None = one call), horizon, limit
    (8, 2, 3, 2, 40, [7, 33], 10, 2),                       # one node
    (64, 1, 4, 3, 50, None, 30, 2),
    (64, 2, 1, 1, 20, [1] * 20, 5, 1),
    (72, 3, 20, 15, 600, None, 200, 3),                     # 256-step chunks: 3 of them
    (72, 3, 20, 15, 600, [1, 5, 300, 294], 200, 3),
    (1024, 4, 50, 40, 2000, None, 700, 3),                  # 10 chunks of 200
    (1024, 4, 50, 40, 2000, [700, 1, 49, 50, 1200], 700, 3),
    (1000, 8, 64, 30, 700, [255, 257, 188], 300, 2),
    (5000, 5, 100, 80, 1500, None, 1000, 4),
    (16384, 4, 100, 80, 900, [450, 450], 400, 3),
    (2048, 2, 1024, 700, 3000, None, 2500, 8),              # the longest window there is
]


@pytest.mark.parametrize("R,M,W,k,T,batches,horizon,limit", CASES)
def test_ledger_on_synthetic_histories(R, M, W, k, T, batches, horizon, limit):
    say(f"case ledger R={R} M={M} W={W} k={k} T={T} batches={batches}")
    N = R // 8
    p = oracle_params(R=R, M=M, W=W, k=k, primary=(W + T) % M, min_signals=min(2, M),
                      directions=(1,) * M)
    seed = R + 13 * W + T
    long_bursts = (max(2, W // 2), 3 * W + 5)
    exceed = exceed_history(seed, T, R, M, 0.03, burst_items=max(4, R // 20), burst_len=long_bursts,
                            gap_len=(1, 2 * W + 3), burst_metrics=M)
    node_mask = exceed_history(seed + 1, T, N, M, 0.03, burst_items=max(3, N // 3), burst_len=long_bursts,
                               gap_len=(1, 2 * W + 3), burst_metrics=M)
    node_z = node_score_history(seed, T, N, scale=3.0)
    node_anom = oracle.combine(node_mask, p.primary, p.min_signals)
    topk_k = min(64, N)
    want = oracle_ledger(p, exceed, node_mask, node_anom, node_z, 64.0, horizon, limit, topk_k)
    det = detector_for(p)
    det.alloc_ledger(max(batches) if batches else T, recur_horizon=horizon, recur_limit=limit)
    feed(det, exceed, node_mask, node_z, batches or [T])
    compare_ledger(want, read_ledger(det, topk_k), f"R{R}-W{W}")
    say("  flagged ranks", int(want["ranks"].flag.sum()), "ever", int((want["ranks"].first >= 0).sum()),
        "nodes ever", int((want["nodes"].first >= 0).sum()), "episodes", np.bincount(want["episodes"]).tolist(),
        "terminal", int((want["terminal"] >= 0).sum()))
    assert (want["ranks"].first >= 0).any() and want["episodes"].any()
    det.close()


def _random_ledger_case(seed):
    rng = np.random.default_rng(5000 + seed)
    R = 8 * int(np.exp(rng.uniform(0, np.log(700))))
    N = R // 8
    M = int(rng.integers(1, 9))
    W = int(np.exp(rng.uniform(0, np.log(300))))
    k = int(rng.integers(1, W + 1))
    T = int(rng.integers(1, 900))
    cuts = sorted(set(rng.integers(1, max(2, T), size=int(rng.integers(0, 5))).tolist()) - {T})
    batches = [b - a for a, b in zip([0] + cuts, cuts + [T])]
    horizon, limit = int(np.exp(rng.uniform(0, np.log(2 * T + 2)))), int(rng.integers(1, 9))
    quant = float(rng.choice([64.0, 1.0, 1000.0, 0.5]))
    p = oracle_params(R=R, M=M, W=W, k=k, primary=int(rng.integers(0, M)), min_signals=int(rng.integers(1, M + 1)),
                      directions=(1,) * M)
    say(f"case random ledger seed={seed} R={R} M={M} W={W} k={k} T={T} batches={batches} horizon={horizon} "
        f"limit={limit} quant={quant} primary={p.primary} min_signals={p.min_signals}")
    rate = float(rng.choice([0.01, 0.1, 0.5]))
    bursts = (max(1, W // 2), 3 * W + 5)
    exceed = exceed_history(seed, T, R, M, rate, burst_items=max(1, R // 10), burst_len=bursts,
                            gap_len=(1, 2 * W + 3), burst_metrics=M)
    node_mask = exceed_history(seed + 7, T, N, M, rate, burst_items=max(1, N // 2), burst_len=bursts,
                               gap_len=(1, 2 * W + 3), burst_metrics=M)
    node_z = node_score_history(seed, T, N, scale=float(rng.choice([0.5, 5.0, 500.0])), outliers=0.05)
    node_anom = oracle.combine(node_mask, p.primary, p.min_signals)
    topk_k = int(rng.integers(1, N + 1))
    want = oracle_ledger(p, exceed, node_mask, node_anom, node_z, quant, horizon, limit, topk_k)
    det = detector_for(p, topk=topk_k)
    det.alloc_ledger(max(batches), score_quant=quant, recur_horizon=horizon, recur_limit=limit)
    feed(det, exceed, node_mask, node_z, batches)
    compare_ledger(want, read_ledger(det, topk_k), f"random ledger {seed}")
    det.close()


@pytest.mark.parametrize("seed", range(24))
def test_ledger_random_configurations(seed):
    """Seeded draws over rank count, metrics, window, k, history length, batch cuts,
    primary metric, number of signals, exceedance rate, horizon, limit and quantisation."""
    _random_ledger_case(seed)


def test_ledger_quantisation_steps():
    """Other quantisation steps, saturation on both sides and a fresh ledger read
    before anything was taken in."""
    R, M, W, T = 256, 2, 16, 100
    N = R // 8
    p = oracle_params(R=R, M=M, W=W, k=8, directions=(1, 1))
    exceed = exceed_history(5, T, R, M, 0.2)
    node_mask = exceed_history(6, T, N, M, 0.3)
    node_anom = oracle.combine(node_mask, p.primary, p.min_signals)
    for quant, scale in ((1.0, 50.0), (4096.0, 1.0), (0.125, 1e4), (64.0, 1e6)):
        node_z = node_score_history(int(quant * 8) + 1, T, N, scale=scale, outliers=0.2)
        want = oracle_ledger(p, exceed, node_mask, node_anom, node_z, quant, 50, 3, N)
        det = detector_for(p)
        det.alloc_ledger(T, score_quant=quant, recur_horizon=50)
        g = read_ledger(det, N)
        assert not g["rank_pflag"].any() and not g["node_score_sum"].any() and not g["node_episodes"].any()
        assert (g["rank_pfirst"] == -1).all() and (g["node_terminal_first"] == -1).all()
        assert g["idx"].tolist() == list(range(N))
        feed(det, exceed, node_mask, node_z, [37, 63])
        compare_ledger(want, read_ledger(det, N), f"quant {quant}")
        det.close()


def test_ledger_behind_the_scoring_kernel():
    """The whole chain on telemetry: gd_score_batch's own outputs feed the ledger; the
    oracle's ledger is computed from the oracle's scores of the same input."""
    w = workload(1)                      # 1024 ranks x 2000 steps x 4 metrics, 8 grey nodes, spikes
    say("case ledger behind scoring", w.name)
    x = generate(w, seed=1)
    p = oracle_params(w)
    o = oracle.score(p, x.numpy(), want_z=False)
    want = oracle_ledger(p, o.exceed_mask, o.node_mask, o.node_anom, o.node_z, 64.0, 600, 2, 64)
    for batches in ([w.T], [1] * 30 + [w.T - 30]):
        det = detector_for(p)
        det.alloc_ledger(max(batches), recur_horizon=600, recur_limit=2)
        t0 = 0
        for c in batches:
            out = gpu_score(det, x[t0:t0 + c], want_z=False)
            det.update_ledger(out, c)
            t0 += c
        torch.cuda.synchronize()
        compare_ledger(want, read_ledger(det, 64), "behind scoring")
        det.close()
    say("  nodes flagged per indicator", int(want["nodes"].flag.sum()), "ranks", int(want["ranks"].flag.sum()),
        "largest score sum", int(want["qsum"].max()))
    assert want["nodes"].flag.sum() >= 4


def test_ledger_at_the_benchmark_size():
    """65 536 ranks x 4 096 steps x 8 metrics in one call, the launch configuration the
    benchmark times.  The oracle re-sums every window, so it follows 2 048 sampled ranks
    and 1 024 sampled nodes for the per-indicator part; the default-rule counts, episodes,
    score sums and the ranking are compared for all 8 192 nodes."""
    R, M, W, k, T = 65536, 8, 256, 200, 4096
    N = R // 8
    say("case ledger at benchmark size")
    p = oracle_params(R=R, M=M, W=W, k=k, directions=(1,) * M)
    exceed = exceed_history(31, T, R, M, 0.014, burst_items=600, burst_len=(150, 900), gap_len=(20, 500))
    node_mask = exceed_history(32, T, N, M, 0.014, burst_items=300, burst_len=(150, 900), gap_len=(20, 500))
    node_z = node_score_history(33, T, N, scale=2.0)
    node_anom = oracle.combine(node_mask, p.primary, p.min_signals)
    rng = np.random.default_rng(9)
    ranks = np.sort(rng.choice(R, 2048, replace=False))
    ranks[:3] = [0, 1, 2]; ranks[-1] = R - 1
    ranks = np.unique(ranks)
    nodes = np.unique(np.concatenate([[0, N - 1], rng.choice(N, 1022, replace=False)]))
    want = oracle_ledger(p, exceed, node_mask, node_anom, node_z, 64.0, 3000, 3, 64, ranks=ranks, nodes=nodes)
    say("  oracle done")
    det = detector_for(p)
    det.alloc_ledger(T, recur_horizon=3000, recur_limit=3)
    feed(det, exceed, node_mask, node_z, [T])
    compare_ledger(want, read_ledger(det, 64),
                   f"benchmark size (per-indicator outputs on {len(ranks)} sampled ranks and {len(nodes)} sampled "
                   "nodes -- items are independent of each other; everything else on all nodes)",
                   ranks=ranks, nodes=nodes)
    say("  sampled ranks ever flagged", int((want["ranks"].first >= 0).sum()), "episodes",
        np.bincount(want["episodes"]).tolist(), "terminal nodes", int((want["terminal"] >= 0).sum()))
    assert (want["terminal"] >= 0).any() and (want["ranks"].first >= 0).any()
    det.close()
