"""GPU parity: the HIP path through the C ABI against the CPU oracle on the same
seeded inputs.  Each test prints the case it is about to run before any launch."""
import numpy as np
import pytest
import torch

import oracle
from gpu_harness import (compare_decision, compare_scores, compare_severity, detector_for, gpu_flags, gpu_score, gpu_topk,
                         oracle_params, run_and_compare)
from workloads import adversarial, generate, workload
from workloads.telemetry import ADVERSARIAL_KINDS

pytestmark = pytest.mark.gpu


@pytest.fixture(params=["auto", "per-run", "per-column"])
def route(request):
    """Short batches can be scored one workgroup per run of steps or one per column:
    the cases that use this fixture run through the library's own choice and through
    each route forced."""
    import gpu_harness
    gpu_harness.STREAMING_STEPS = {"auto": None, "per-run": 0, "per-column": 64}[request.param]
    yield request.param
    gpu_harness.STREAMING_STEPS = None


def say(*a):
    print(*a, flush=True)


# Rank counts spanning every register tiling of the scoring kernel, full and ragged.
SHAPES = [(8, 1), (24, 3), (64, 1), (72, 2), (256, 4), (1000, 2), (1024, 4), (2056, 8), (4096, 3),
          (5000, 2), (16384, 4), (20000, 2), (32768, 8), (40000, 1), (65536, 8)]


@pytest.mark.parametrize("R,M", SHAPES)
def test_shapes_full_and_ragged(R, M, route):
    T = 5 if R <= 16384 else 3
    say(f"case shapes R={R} M={M} T={T}")
    g = torch.Generator().manual_seed(R * 31 + M)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64))
    x[:, :, (R // 8 // 2) * 8: (R // 8 // 2) * 8 + 8] *= 1.07       # one slow node
    x[:, :, 3] *= 1.2                                               # one slow GPU
    x[:, 1::2] = 400.0 / x[:, 1::2]                                  # lower-is-worse metrics
    x = x.to(torch.float32)
    dirs = tuple(1 if m % 2 == 0 else -1 for m in range(M))
    p = oracle_params(R=R, M=M, W=4, k=2, directions=dirs)
    rep = run_and_compare(p, x, topk_k=min(8, R // 8), chunks=[2, T - 2], label=f"R{R}M{M}")
    say("  report", rep)
    assert rep["z_bit_exact"]


def _random_case(seed, n_lo, n_hi, t_hi):
    """One seeded draw over the whole configuration space at once -- rank count (n_lo to
    n_hi nodes, log-uniform), metrics, window, threshold, directions, primary metric,
    number of signals, node rule and its scale, floors, missing samples, signs, ties,
    batch cuts and route -- through the whole path against the oracle."""
    import gpu_harness
    rng = np.random.default_rng(1000 + seed)
    R = 8 * int(np.exp(rng.uniform(np.log(n_lo), np.log(n_hi + 1))))
    M = int(rng.integers(1, 9))
    T = int(rng.integers(3, t_hi + 1))
    W = int(rng.integers(1, 13))
    k = int(rng.integers(1, W + 1))
    dirs = tuple(int(d) for d in rng.choice([1, -1, 0], M))
    kw = dict(R=R, M=M, W=W, k=k, thr=float(rng.choice([3.5, 2.0, 0.5, 0.0, -0.5, 6.0])), directions=dirs,
              primary=int(rng.integers(0, M)), min_signals=int(rng.integers(1, M + 1)),
              node_agg=int(rng.choice([oracle.NODE_SUM_SCALED, oracle.NODE_MAX])),
              node_scale=float(rng.choice([8 ** -0.5, 0.125, 1.0])),
              rel_floor=float(rng.choice([1e-6, 1e-2, 0.0])), abs_floor=float(rng.choice([1e-30, 1e-3])))
    p = oracle_params(**kw)
    g = torch.Generator().manual_seed(seed)
    sigma = float(rng.choice([0.02, 0.2, 1e-4]))
    x = torch.exp(sigma * torch.randn((T, M, R), generator=g, dtype=torch.float64))
    for n in rng.choice(R // 8, size=min(3, R // 8), replace=False):        # slow nodes from some step on
        x[int(rng.integers(0, T)):, :, 8 * n: 8 * n + 8] *= float(rng.uniform(1.05, 1.5))
    x = x.to(torch.float32)
    flavour = seed % 4
    if flavour == 1:                                  # missing samples, scattered and by node
        x[torch.rand((T, M, R), generator=g) < 0.03] = float("nan")
        x[T // 2, 0, : 8 * max(1, R // 64)] = float("nan")
    elif flavour == 2:                                # signs and both zeros
        x = x - 1.0
        x[0, 0, 0] = 0.0
        x[0, 0, 1] = -0.0
    elif flavour == 3:                                # heavy ties
        x = torch.round(x * 8) / 8
    cuts = sorted(set(rng.integers(1, T, size=int(rng.integers(0, 4))).tolist()))
    chunks = [b - a for a, b in zip([0] + cuts, cuts + [T])]
    gpu_harness.STREAMING_STEPS = [None, 0, 64][seed % 3]
    say(f"case random seed={seed} R={R} M={M} T={T} W={W} k={k} chunks={chunks} flavour={flavour} "
        f"route={gpu_harness.STREAMING_STEPS} {kw}")
    try:
        rep = run_and_compare(p, x, topk_k=min(int(rng.integers(1, 70)), R // 8), chunks=chunks,
                              label=f"random{seed}")
    finally:
        gpu_harness.STREAMING_STEPS = None
    say("  report", rep)
    assert rep["z_bit_exact"]


@pytest.mark.parametrize("seed", range(32))
def test_random_configurations(seed):
    _random_case(seed, 1, 1200, 39)


@pytest.mark.parametrize("seed", range(100, 112))
def test_random_configurations_of_many_ranks(seed):
    """The same draws with 8 192 to 65 536 ranks: the large register tilings."""
    _random_case(seed, 1024, 8192, 6)


@pytest.mark.parametrize("kind", ADVERSARIAL_KINDS)
@pytest.mark.parametrize("R", [64, 4096, 65536])
def test_adversarial_columns(kind, R, route):
    T, M = (4, 2) if R < 65536 else (2, 2)
    say(f"case adversarial kind={kind} R={R}")
    x = adversarial(kind, R, T, M, seed=R % 97)
    p = oracle_params(R=R, M=M, W=3, k=2, directions=(1, 0), min_signals=1)
    rep = run_and_compare(p, x, topk_k=min(8, R // 8), label=f"{kind}-R{R}")
    say("  report", rep)
    assert rep["z_bit_exact"]


@pytest.mark.parametrize("agg", [oracle.NODE_SUM_SCALED, oracle.NODE_MAX])
@pytest.mark.parametrize("R", [1024, 16384])
def test_node_aggregation_rules_and_options(agg, R, route):
    say(f"case node_agg={agg} R={R}")
    g = torch.Generator().manual_seed(5)
    x = torch.exp(0.02 * torch.randn((6, 3, R), generator=g, dtype=torch.float64)).to(torch.float32)
    x[2:, :, 64:72] *= 1.06
    p = oracle_params(R=R, M=3, W=5, k=3, node_agg=agg, primary=1, min_signals=3, thr=2.5,
                      node_scale=0.125, rel_floor=1e-3, abs_floor=1e-20, directions=(1, 0, 1))
    rep = run_and_compare(p, x, topk_k=16, chunks=[1, 1, 4], label=f"agg{agg}")
    say("  report", rep)


@pytest.mark.parametrize("thr", [0.0, -0.75, 1e-3, 2.0, 30.0])
def test_thresholds_that_crowd_the_decision_boundary(thr, route):
    """With the threshold inside the bulk of the node scores many estimated node
    scores fall within the rounding margin and must be settled exactly."""
    R, M, T = 65536, 4, 3
    say(f"case crowded threshold thr={thr}")
    g = torch.Generator().manual_seed(17)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64))
    x[:, 1] = 400.0 / x[:, 1]
    x[:, :, 4096:4104] *= 1.05
    x = x.to(torch.float32)
    p = oracle_params(R=R, M=M, W=3, k=2, thr=thr, directions=(1, -1, 1, 0), min_signals=2)
    rep = run_and_compare(p, x, topk_k=16, label=f"thr{thr}")
    say("  report", rep)
    assert rep["z_bit_exact"]


def test_tiny_configuration(route):
    w = workload(0)
    say("case", w.name)
    x = generate(w, seed=0)
    rep = run_and_compare(oracle_params(w), x, topk_k=w.topk, chunks=[1] * 10 + [40, 150], label=w.name)
    say("  report", rep)
    assert rep["rank_flags"] == 2


def test_configuration_1_full():
    w = workload(1)
    say("case", w.name)
    x = generate(w, seed=1)
    rep = run_and_compare(oracle_params(w), x, topk_k=w.topk, chunks=[700, 1, 1299], label=w.name,
                          want_z=True)
    say("  report", rep)
    assert rep["node_flags"] >= 6      # 8 grey nodes slowed 5-30%; the mildest may stay under


def test_configuration_2_prefix():
    w = workload(2, T=320)
    say("case", w.name, "first 320 steps")
    x = generate(w, seed=2)
    rep = run_and_compare(oracle_params(w), x, topk_k=w.topk, chunks=[120, 200], label=w.name,
                          want_z=False)
    say("  report", rep)


def test_configuration_3_prefix_with_window_wrap():
    w = workload(3, T=40, W=16, k=12, fault_ramp=8)
    say("case", w.name, "40 steps, window shortened to 16")
    x = generate(w, seed=3)
    rep = run_and_compare(oracle_params(w), x, topk_k=w.topk, chunks=[24, 16], label=w.name,
                          want_z=False)
    say("  report", rep)


def test_streaming_configuration_prefix(route):
    """Config 4's launch shape: one step per call, ring kept on the device."""
    w = workload(4, T=300, W=64, k=48)
    say("case", w.name, "300 single-step calls, W=64")
    x = generate(w, seed=4)
    # make a few nodes fail-slow early so that flags appear inside the prefix
    x[40:, :, 800:808] *= torch.tensor([1.2, 1.2, 1.2, 1 / 1.2, 1.2, 1 / 1.2, 1 / 1.2, 1 / 1.2])[:, None]
    rep = run_and_compare(oracle_params(w), x, topk_k=w.topk, chunks=[1] * 300, label=w.name,
                          want_z=False)
    say("  report", rep)
    assert rep["node_flags"] >= 1


@pytest.mark.parametrize("R", [64, 1000, 4096, 16384, 32768, 40000, 65536])
@pytest.mark.parametrize("source", ["previous outputs", "garbage"])
def test_one_step_calls_with_hints(R, source):
    """gd_set_streaming_hints: one-step calls that start from the previous call's medians
    and MADs (the output buffers themselves), on data whose level and spread jump, collapse
    to ties, change sign and lose samples between steps -- and calls whose hint arrays
    hold arbitrary bit patterns.  Every output of every step against the oracle."""
    say(f"case one-step hints R={R} {source}")
    M, T = 3, 36
    g = torch.Generator().manual_seed(R + len(source))
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64))
    x[:, 1] = 300.0 / x[:, 1]
    x[8:] *= 1.5                      # level jump
    x[12:14, 0] = 1.0                 # constant columns
    x[16:18] = torch.round(x[16:18] * 16) / 16          # heavy ties
    x[20:, 2] *= torch.exp(0.5 * torch.randn((T - 20, R), generator=g, dtype=torch.float64))   # spread explodes
    x[24, 0, ::5] *= -1.0             # signs
    x[26:28, 1, 3::7] = NAN           # missing samples
    x[30:, :, 8:16] *= 1.2
    x = x.to(torch.float32)
    p = oracle_params(R=R, M=M, W=6, k=3, directions=(1, -1, 0), min_signals=1)
    o = oracle.score(p, x.numpy(), want_z=True)
    det = detector_for(p)
    xd = x.cuda()
    out = det.alloc_outputs(1, want_z=True)
    if source == "previous outputs":
        out["med"].fill_(float("nan")); out["mad"].fill_(float("nan"))
        det.set_streaming_hints(out["med"].view(-1), out["mad"].view(-1))
    else:
        hm = torch.empty(M, dtype=torch.float32, device="cuda")
        hd = torch.empty(M, dtype=torch.float32, device="cuda")
        det.set_streaming_hints(hm, hd)
    rng = np.random.default_rng(R)
    for t in range(T):
        if source == "garbage":       # any bit pattern, or plausible but wrong values
            if t % 3 == 0:
                bits = rng.integers(0, 2**32, size=2 * M, dtype=np.uint64).astype(np.uint32)
                vals = bits.view(np.float32)
            else:
                vals = np.exp(rng.uniform(-3, 3, 2 * M)).astype(np.float32)
            hm.copy_(torch.from_numpy(vals[:M].copy())); hd.copy_(torch.from_numpy(vals[M:].copy()))
        det.score_batch(xd[t:t + 1], out)
        torch.cuda.synchronize()
        part = oracle.Scores(o.med[t:t + 1], o.mad[t:t + 1], o.z[t:t + 1], o.exceed_mask[t:t + 1],
                             o.rank_anom[t:t + 1], o.node_z[t:t + 1], o.node_mask[t:t + 1],
                             o.node_anom[t:t + 1], None, 0, 0)
        rep = compare_scores(part, out, f"step {t}")
        assert rep["z_bit_exact"]
    det.set_streaming_hints(None, None)
    det.close()


@pytest.mark.timeout(900)
def test_streaming_configuration_at_full_length():
    """Config 4 as specified: 100 000 steps of 32 768 ranks x 8 metrics, one step per call
    (W = 256, k = 200), each call hinted by the previous call's outputs, the input made
    1 000 steps at a time.  The oracle scores every one of the 100 000 steps (on the host,
    one chunk behind the GPU) and every scoring output of every step is compared; its
    anomaly words of the whole history then go through its window, which gives the
    counts, flags, first-flag steps and the top-64 that the streamed state must show.
    On top of that the state after 100 000 single-step calls must equal, byte for byte,
    the state after the same data in 1 000-step batches."""
    from concurrent.futures import ThreadPoolExecutor
    w = workload(4)
    say("case", w.name, "at full length")
    assert w.T == 100000 and w.W == 256
    p = oracle_params(w)
    det, det_b = detector_for(p), detector_for(p)
    CH = 1000
    bufs = [det.alloc_outputs(CH, want_z=False) for _ in range(2)]
    out_b = det_b.alloc_outputs(CH, want_z=False)
    host_x = [torch.empty((CH, w.M, w.R), dtype=torch.float32, pin_memory=True) for _ in range(2)]
    RW, NW = (p.R + 63) // 64, (p.N + 63) // 64
    rank_words = np.empty((w.T, RW), np.uint64)          # the oracle's anomaly words of the whole history
    node_words = np.empty((w.T, NW), np.uint64)
    last_node_z = [None]

    def check(c0, xh, got):
        """(worker thread) the oracle on one chunk, every output of every step compared"""
        o = oracle.score(p, xh.numpy(), want_z=False)
        compare_scores(o, got, f"steps {c0}..{c0 + CH - 1}")
        rank_words[c0:c0 + CH] = o.rank_anom
        node_words[c0:c0 + CH] = o.node_anom
        last_node_z[0] = o.node_z[-1].copy()

    pool = ThreadPoolExecutor(1)
    pending = None
    prev = None
    try:
        for ci, c0 in enumerate(range(0, w.T, CH)):
            x = generate(w, seed=4, t0=c0, t1=c0 + CH, device="cuda")
            out = bufs[ci & 1]
            for v in out.values():
                if v is not None:
                    v.view(torch.uint8).fill_(0xA5)
            det_b.score_batch(x, out_b)
            det_b.update_window(out_b, CH)
            for t in range(CH):
                one = {k: (v[t:t + 1] if v is not None else None) for k, v in out.items()}
                if prev is not None:
                    det.set_streaming_hints(prev["med"].view(-1), prev["mad"].view(-1))
                det.score_batch(x[t:t + 1], one)
                det.update_window(one, 1)
                prev = one
            xh = host_x[ci & 1]
            xh.copy_(x, non_blocking=True)
            torch.cuda.synchronize()
            got = {k: v.cpu() for k, v in out.items() if v is not None}
            if pending is not None:
                pending.result()                       # (raises what the comparison raised)
            pending = pool.submit(check, c0, xh, got)
            if ci % 10 == 9:
                say(f"  {c0 + CH} steps streamed, {c0} compared with the oracle")
        pending.result()
    finally:
        pool.shutdown(wait=True)
    det.set_streaming_hints(None, None)
    assert det.steps_seen == w.T == det_b.steps_seen
    say("  every scoring output of every step matches; windows over the whole history ...")
    pr = oracle.window(p.R, rank_words, p.W, p.k)
    say("  rank windows done")
    pn = oracle.window(p.N, node_words, p.W, p.k)
    f = gpu_flags(det)
    assert np.array_equal(f["rank_count"].view(np.uint16), pr.count), "rank counts"
    assert np.array_equal(f["rank_flag"], pr.flag), "rank flags"
    assert np.array_equal(f["rank_first"], pr.first), "rank first-flag steps"
    assert np.array_equal(f["node_count"].view(np.uint16), pn.count), "node counts"
    assert np.array_equal(f["node_flag"], oracle.node_flag_byte(p.G, pn.flag, pr.flag)), "node flag bytes"
    assert np.array_equal(f["node_first"], pn.first), "node first-flag steps"
    idx, key = gpu_topk(det, w.topk)
    want_idx, want_key = oracle.topk(pn.count, last_node_z[0], w.topk)
    assert np.array_equal(idx, want_idx) and np.array_equal(key, want_key), "top-k"
    # extra: the two routes through the library leave the same bytes
    assert torch.equal(det.state, det_b.state), "state after single-step calls != state after batches"
    say("  flagged ranks", int(pr.flag.sum()), "flagged nodes", int(pn.flag.sum()),
        "ranks ever flagged", int((pr.first >= 0).sum()), "nodes ever flagged", int((pn.first >= 0).sum()))
    assert int(pn.flag.sum()) >= 20          # 48 nodes step to +5..20 % during the run
    det.close(); det_b.close()


def test_checkpoint_restore_and_chunking_give_identical_state():
    w = workload(1, T=260)
    say("case checkpoint/chunking", w.name)
    x = generate(w, seed=7)
    p = oracle_params(w)
    states = []
    for chunks in ([260], [1] * 60 + [200], [130, 130]):
        det = detector_for(p)
        t0 = 0
        for c in chunks:
            g = gpu_score(det, x[t0:t0 + c], want_z=False)
            det.update_window(g, c)
            t0 += c
        torch.cuda.synchronize()
        states.append(det.state.cpu().numpy().copy())
        det.close()
    assert np.array_equal(states[0], states[1]) and np.array_equal(states[0], states[2])
    # checkpoint = byte copy of the state + steps consumed
    det = detector_for(p)
    g = gpu_score(det, x[:100], want_z=False)
    det.update_window(g, 100)
    torch.cuda.synchronize()
    snap = det.state.clone()
    det.close()
    det2 = detector_for(p)
    det2.state.copy_(snap)
    g = gpu_score(det2, x[100:], want_z=False)
    det2.update_window(g, 160, first_step_index=100)
    torch.cuda.synchronize()
    assert np.array_equal(det2.state.cpu().numpy(), states[0])
    d = oracle.detect(p, x.numpy(), topk_k=w.topk)
    compare_decision(p, d, det2, w.topk, label="restored")
    det2.close()


def test_runs_are_deterministic():
    w = workload(3, T=6)
    say("case determinism", w.name)
    x = generate(w, seed=9).cuda()
    p = oracle_params(w)
    det = detector_for(p)
    a = gpu_score(det, x, want_z=True)
    b = gpu_score(det, x, want_z=True)
    for k in a:
        assert torch.equal(a[k], b[k]), k
    det.close()


def test_device_division_is_correctly_rounded():
    """The z scores rely on IEEE fp32 division on the device: one column whose
    numerators and scale span many magnitudes, against the oracle's host division."""
    say("case division rounding")
    R = 65536
    g = torch.Generator().manual_seed(11)
    e = torch.rand((4, 1, R), generator=g, dtype=torch.float64) * 40 - 20
    x = (torch.randn((4, 1, R), generator=g, dtype=torch.float64) * torch.pow(2.0, e)).to(torch.float32)
    p = oracle_params(R=R, M=1, W=2, k=1, min_signals=1)
    det = detector_for(p)
    gpu = gpu_score(det, x, want_z=True)
    o = oracle.score(p, x.numpy(), want_z=True)
    rep = compare_scores(o, gpu, "division")
    assert rep["z_bit_exact"]
    det.close()


def _random_severity_case(seed):
    rng = np.random.default_rng(9000 + seed)
    R = 8 * int(np.exp(rng.uniform(0, np.log(600))))
    N, M = R // 8, int(rng.integers(1, 5))
    W = int(np.exp(rng.uniform(0, np.log(400))))
    T = int(rng.integers(1, 3 * W + 3))
    k = int(rng.integers(1, W + 1))
    dirs = tuple(int(d) for d in rng.choice([1, -1, 0], M))
    p = oracle_params(R=R, M=M, W=W, k=k, thr=float(rng.choice([3.5, 1.0])), directions=dirs,
                      primary=int(rng.integers(0, M)), min_signals=1)
    say(f"case random severity seed={seed} R={R} M={M} W={W} T={T} k={k} dirs={dirs} primary={p.primary}")
    g = torch.Generator().manual_seed(seed)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64))
    for n in rng.choice(N, size=min(N, int(rng.integers(1, 6))), replace=False):
        f = float(rng.uniform(1.03, 1.4)) ** float(rng.choice([1, -1]))
        x[int(rng.integers(0, T)):, :, 8 * n: 8 * n + int(rng.integers(1, 9))] *= f
    x = x.to(torch.float32)
    if seed % 3 == 1:
        x[torch.rand((T, M, R), generator=g) < 0.05] = float("nan")
    d = oracle.detect(p, x.numpy(), topk_k=1)
    det = detector_for(p)
    out = gpu_score(det, x, want_z=False)
    compare_scores(d["scores"], out, f"severity {seed}")
    det.update_window(out, T)
    moderate = float(rng.choice([0.10, 0.02, 0.0]))
    rep = compare_severity(p, d, det, x, out, moderate, moderate + float(rng.choice([0.0, 0.05, 0.1])),
                           label=f"severity {seed}")
    det.close()
    return rep


@pytest.mark.parametrize("seed", range(24))
def test_severity_random_configurations(seed):
    """Seeded draws over rank count, window (1 to 400), history length around it, k,
    directions, slowed and sped-up nodes and GPUs, missing samples and tier boundaries."""
    _random_severity_case(seed)


@pytest.mark.parametrize("R", [64, 4096, 65536])
def test_topk_request_sizes(R):
    """k from 1 to N: the short-list route (k <= 64) and the full sort, with many
    equal window counts and equal scores among the keys."""
    say(f"case top-k sizes R={R}")
    T, M = 12, 2
    g = torch.Generator().manual_seed(R + 1)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64)).to(torch.float32)
    x[:, :, : R // 2] = x[:, :, R // 2:]                # every node score appears twice
    x[4:, :, 8:24] *= 1.3                               # two nodes with window counts > 0
    p = oracle_params(R=R, M=M, W=6, k=3, directions=(1, 1), min_signals=1)
    d = oracle.detect(p, x.numpy(), topk_k=1)
    det = detector_for(p)
    gscore = gpu_score(det, x, want_z=False)
    det.update_window(gscore, T)
    N = R // 8
    from gpu_harness import gpu_topk
    for k in sorted({1, 2, min(7, N), min(63, N), min(64, N), min(65, N), min(200, N), N}):
        want_idx, want_key = oracle.topk(d["nodes"].count, d["scores"].node_z[-1], k)
        idx, key = gpu_topk(det, k)
        assert np.array_equal(idx, want_idx), f"k={k}: indices"
        assert np.array_equal(key, want_key), f"k={k}: keys"
    det.close()


@pytest.mark.parametrize("R,M,W,T,direction", [(64, 1, 4, 9, 1), (1024, 3, 16, 40, -1),
                                                  (4096, 2, 1024, 1100, 0), (65536, 2, 6, 5, 1)])
def test_severity_tiers(R, M, W, T, direction):
    """Slowdown and tier of every flagged node, bit for bit, for windows from 4 to the
    longest (1024 steps), histories shorter and longer than the window, each direction."""
    say(f"case severity R={R} M={M} W={W} T={T} dir={direction}")
    g = torch.Generator().manual_seed(R + W)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64))
    prim = M - 1
    f = 1.0 if direction >= 0 else -1.0
    N = R // 8
    # nodes slowed by 4% .. 32% in the primary metric from the first step on, one of them
    # only in a single GPU, one only during the first third of the history
    if N > 8:
        for i, s in enumerate((1.04, 1.09, 1.12, 1.19, 1.21, 1.32)):
            x[:, :, ((i * 5 + 1) % N) * 8:((i * 5 + 1) % N) * 8 + 8] *= s ** f
        x[:, :, ((31 % N) * 8 + 3)] *= 1.25 ** f
        x[: T // 3, :, (37 % N) * 8:(37 % N) * 8 + 8] *= 1.5 ** f
    else:                                   # 8 nodes: slow two of them only
        x[:, :, 8:16] *= 1.12 ** f
        x[:, :, 48:56] *= 1.32 ** f
    x = x.to(torch.float32)
    dirs = tuple(direction for _ in range(M))
    p = oracle_params(R=R, M=M, W=W, k=max(1, min(W, T) // 2), primary=prim, directions=dirs,
                      min_signals=1)
    d = oracle.detect(p, x.numpy(), topk_k=1)
    det = detector_for(p)
    out = gpu_score(det, x, want_z=False)
    det.update_window(out, T)
    rep = compare_severity(p, d, det, x, out, label="default tiers")
    say("  nodes per tier", rep)
    assert sum(rep["tiers"][1:]) >= (3 if N > 8 else 2)
    compare_severity(p, d, det, x, out, moderate=0.05, severe=0.05, label="one threshold")
    # the last steps alone (a batch shorter than the window)
    tail = min(T, 3)
    sev = det.alloc_severity()
    out_tail = {k: (v[T - tail:].contiguous() if v is not None else None) for k, v in out.items()}
    det.severity(x[T - tail:].cuda(), out_tail, sev)
    torch.cuda.synchronize()
    want = oracle.severity(p, x[T - tail:].numpy(), d["scores"].med[T - tail:], d["node_flag_byte"])
    assert np.array_equal(sev["tier"].cpu().numpy(), want[1])
    assert np.array_equal(sev["slowdown"].cpu().numpy().view(np.uint32), want[0].view(np.uint32))
    det.close()


def _full_size_case(w, seed, chunk, min_flagged_nodes):
    """Score the whole workload in ONE gd_score_batch call on GPU-generated data,
    then window / flags / top-k.  The oracle scores every step of the same bytes
    (chunk by chunk through host memory) and every output is compared bit for
    bit; its own anomaly words feed its persistence run over the full history."""
    x = generate(w, seed=seed, device="cuda")
    p = oracle_params(w)
    det = detector_for(p)
    out = det.alloc_outputs(w.T, want_z=False)
    det.score_batch(x, out)
    det.update_window(out, w.T)
    torch.cuda.synchronize()
    ra, na, meds, near = [], [], [], [0, 0]
    last_node_z = None
    for t0 in range(0, w.T, chunk):
        t1 = min(w.T, t0 + chunk)
        o = oracle.score(p, x[t0:t1].cpu().numpy(), want_z=False)
        g = {k: (v[t0:t1] if v is not None else None) for k, v in out.items()}
        compare_scores(o, g, f"steps [{t0},{t1})")
        ra.append(o.rank_anom); na.append(o.node_anom); meds.append(o.med)
        near[0] += o.near_rank; near[1] += o.near_node
        last_node_z = o.node_z[-1]
        say(f"  steps [{t0},{t1}) match")
    pr = oracle.window(p.R, np.concatenate(ra), p.W, p.k)
    pn = oracle.window(p.N, np.concatenate(na), p.W, p.k)
    d = dict(ranks=pr, nodes=pn, node_flag_byte=oracle.node_flag_byte(p.G, pn.flag, pr.flag))
    d["topk_idx"], d["topk_key"] = oracle.topk(pn.count, last_node_z, w.topk)
    compare_decision(p, d, det, w.topk, label="full-size decision")
    # severity of the flagged nodes over the last W steps of the resident batch
    sev = det.alloc_severity()
    det.severity(x, out, sev)
    torch.cuda.synchronize()
    want = oracle.severity(p, x[w.T - p.W:].cpu().numpy(), np.concatenate(meds)[w.T - p.W:],
                           d["node_flag_byte"])
    assert np.array_equal(sev["tier"].cpu().numpy(), want[1]), "full-size tiers"
    assert np.array_equal(sev["slowdown"].cpu().numpy().view(np.uint32), want[0].view(np.uint32))
    say("  nodes per tier", np.bincount(want[1], minlength=4).tolist())
    say("  near-threshold comparisons (rank, node):", near, "flagged ranks", int(pr.flag.sum()),
        "flagged nodes", int(pn.flag.sum()))
    assert int(pn.flag.sum()) >= min_flagged_nodes
    det.close()


def test_bench_workload_at_full_size():
    """The benchmark's own launch configuration: 65 536 ranks x 4 096 steps x 8 metrics
    (8 GiB) in one call."""
    w = workload(3)
    say("case full-size bench workload", w.name)
    _full_size_case(w, seed=3, chunk=256, min_flagged_nodes=20)   # 32 nodes drift to +20%


def test_configuration_2_at_full_size():
    """16 384 ranks x 10 000 steps x 4 metrics (2.6 GB) in one call."""
    w = workload(2)
    say("case full-size", w.name)
    _full_size_case(w, seed=2, chunk=1000, min_flagged_nodes=30)  # 64 grey nodes, 3-20% slow


NAN = float("nan")


@pytest.mark.parametrize("R,M", [(64, 1), (72, 2), (1024, 4), (5000, 2), (16384, 3), (65536, 2)])
def test_missing_samples(R, M, route):
    """NaN = a sample that did not arrive: left out of median and MAD, z = 0, never
    exceeds, adds nothing to its node.  Scattered ranks, whole nodes, a whole
    column, odd and even numbers present, NaNs of either sign, next to columns with
    nothing missing."""
    T = 6
    say(f"case missing samples R={R} M={M}")
    g = torch.Generator().manual_seed(R + 7 * M)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64)).to(torch.float32)
    x[:, :, 16:24] *= 1.2                                  # a slow node
    N = R // 8
    x[0, 0, torch.randperm(R, generator=g)[: max(1, R // 50)]] = NAN     # scattered, even or odd count
    x[1, 0, 5] = NAN                                       # a single one: an odd number present
    x[1, 0, 16:19] = NAN                                   # part of the slow node
    x[2, M - 1, 8 * (N // 2): 8 * (N // 2) + 8] = NAN      # a silent node
    x[3, 0, :] = NAN                                       # nothing arrived for this metric
    x[4, 0, : R - 3] = NAN                                 # three samples left
    x[5, 0, 1::2] = -x[5, 0, 1::2]                         # signs, and NaNs with the sign bit set
    neg_nan = torch.tensor([0xFFC00001], dtype=torch.int64).to(torch.int32).view(torch.float32)
    x[5, 0, 7] = neg_nan[0]
    x[5, 0, 32 % R] = NAN
    dirs = tuple((1, -1, 0, 1)[m % 4] for m in range(M))
    for thr, agg in ((3.5, oracle.NODE_SUM_SCALED), (-0.5, oracle.NODE_MAX)):
        p = oracle_params(R=R, M=M, W=4, k=2, thr=thr, node_agg=agg, directions=dirs, min_signals=1)
        rep = run_and_compare(p, x, topk_k=min(8, N), chunks=[2, 4], label=f"missing-R{R}-thr{thr}")
        say("  report", rep)
        assert rep["z_bit_exact"]


@pytest.mark.parametrize("R,M,T", [(8, 1, 3), (72, 2, 5), (1000, 3, 7), (4096, 8, 4), (65536, 2, 3)])
def test_membership_mask(R, M, T):
    """gd_apply_membership: the tensor after the call is, bit for bit, the oracle's (NaN
    exactly where a rank takes no part, everything else untouched), and the batch scored
    after it is the oracle's scoring of the oracle's masked tensor."""
    say(f"case membership R={R} M={M} T={T}")
    rng = np.random.default_rng(R + T)
    g = torch.Generator().manual_seed(R)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64)).to(torch.float32)
    x[:, :, :8] *= 1.3
    bits = rng.random((T, R)) < 0.9
    bits[0] = True                                  # everybody
    if T > 2:
        bits[2, : R // 2] = False                   # half of the cluster absent
    bits[-1, 8 * (R // 16): 8 * (R // 16) + 8] = False   # a whole node
    RW = (R + 63) // 64
    padded = np.zeros((T, RW * 64), np.uint8)
    padded[:, :R] = bits
    words = np.packbits(padded.reshape(T, RW, 64), axis=2, bitorder="little").view(np.uint64).reshape(T, RW)
    want = oracle.apply_membership(x.numpy(), words)
    p = oracle_params(R=R, M=M, W=3, k=2, directions=(1,) * M, min_signals=1)
    det = detector_for(p)
    xd = x.cuda()
    det.apply_membership(xd, torch.from_numpy(words.view(np.int64)).cuda())
    torch.cuda.synchronize()
    assert np.array_equal(xd.cpu().numpy().view(np.uint32), want.view(np.uint32))
    o = oracle.score(p, want, want_z=True)
    rep = compare_scores(o, gpu_score(det, xd, want_z=True), "after the mask")
    assert rep["z_bit_exact"]
    det.close()


def test_severity_with_missing_samples():
    R, M, W, T = 1024, 2, 8, 20
    say("case severity with missing samples")
    g = torch.Generator().manual_seed(77)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64)).to(torch.float32)
    for i, s in enumerate((1.08, 1.15, 1.3, 1.12)):
        x[:, :, (3 + 7 * i) * 8:(3 + 7 * i) * 8 + 8] *= s
    x[T - 5:, 0, 3 * 8: 3 * 8 + 5] = NAN            # part of a slow node, part of the window
    x[T - 8:, 0, 10 * 8 + 1] = NAN                   # one GPU of a slow node, the whole window: 56 left
    x[T - 3, 0, 17 * 8: 17 * 8 + 8] = NAN            # one step of a slow node
    x[T - 6:, 0, 24 * 8: 24 * 8 + 8] = NAN           # a slow node that fell silent: 2 steps x 8 left
    x[T - 2, 0, ::3] = NAN                           # a step with many samples missing
    p = oracle_params(R=R, M=M, W=W, k=3, directions=(1, 1), min_signals=1)
    d = oracle.detect(p, x.numpy(), topk_k=1)
    det = detector_for(p)
    out = gpu_score(det, x, want_z=False)
    compare_scores(d["scores"], out, "scores")
    det.update_window(out, T)
    rep = compare_severity(p, d, det, x, out, label="missing")
    say("  nodes per tier", rep)
    assert sum(rep["tiers"][1:]) >= 3
    det.close()


def test_missing_samples_and_signs_arriving_in_the_middle_of_a_run():
    """Two steps per workgroup and more (65 536 ranks, 600 steps): the second step of a
    run starts from the first one's median as a hint and finds the column's largest
    bit pattern during its counting pass -- which then has to notice NaNs and signs."""
    R, M, T = 65536, 2, 600
    say("case missing samples inside hinted runs")
    g = torch.Generator().manual_seed(5)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64)).to(torch.float32)
    x[:, :, 4096:4104] *= 1.1
    for t in range(1, T, 7):                       # odd steps are the second of their run
        x[t, 0, (t * 37) % R] = NAN                # a single missing sample
    for t in range(3, T, 31):
        x[t, 1, torch.randperm(R, generator=g)[:5000]] = NAN
    x[301, 0, ::2] = NAN                           # half of the column
    x[303, 1, :] = NAN                             # all of it
    x[305, 0, 100] = -x[305, 0, 100]               # a sign
    x[401, 1, 7] = -0.0
    p = oracle_params(R=R, M=M, W=16, k=8, directions=(1, -1), min_signals=1)
    det = detector_for(p)
    det.set_streaming_steps(0)
    out = gpu_score(det, x, want_z=False)
    o = oracle.score(p, x.numpy(), want_z=False)
    rep = compare_scores(o, out, "hinted runs with missing samples")
    say("  report", rep)
    det.close()


@pytest.mark.parametrize("B", [1, 5, 4096, 8192 + 3])
def test_single_node_sweep_scoring(B):
    say(f"case sweep scoring B={B}")
    rng = np.random.default_rng(B)
    flops = (400.0 * np.exp(0.03 * rng.standard_normal((B, 8)))).astype(np.float32)
    bw = (300.0 * np.exp(0.04 * rng.standard_normal((B, 8, 8)))).astype(np.float32)
    for b in range(0, B, 3):                       # throttled GPUs, one-way and two-way slow links
        flops[b, rng.integers(8)] *= np.float32(rng.uniform(0.6, 0.97))
    for b in range(1, B, 4):
        i, j = rng.choice(8, 2, replace=False)
        bw[b, i, j] *= np.float32(rng.uniform(0.4, 0.95))
        if b % 8 == 1:
            bw[b, j, i] = bw[b, i, j]
    bw[0, :, :] = bw[0, 0, 1]                      # ties everywhere
    p = oracle_params(R=64, M=1, W=2, k=1)
    det = detector_for(p)
    for tc, ts, tb in ((0.05, 0.10, 0.15), (0.0, 0.0, 0.0), (0.5, 0.02, 0.9)):
        want = oracle.sweep(flops, bw, tc, ts, tb)
        got = det.sweep_score(torch.from_numpy(flops).cuda(), torch.from_numpy(bw).cuda(), tc, ts, tb)
        torch.cuda.synchronize()
        assert np.array_equal(got["shortfall"].cpu().numpy().view(np.uint32), want[0].view(np.uint32))
        assert np.array_equal(got["gpu_mask"].cpu().numpy(), want[1])
        assert np.array_equal(got["link_mask"].cpu().numpy().view(np.uint32), want[2])
        assert np.array_equal(got["verdict"].cpu().numpy(), want[3])
    say("  verdicts", np.bincount(want[3], minlength=4).tolist())
    det.close()


@pytest.mark.parametrize("W,T,chunks", [(64, 65, [65]), (64, 300, [200, 100]), (128, 293, [293]),
                                        (256, 700, [1, 699]), (512, 1100, [600, 500]),
                                        (1024, 1030, [1030]), (192, 500, [500])])
def test_windows_of_whole_64_step_blocks(W, T, chunks):
    """Windows that are a whole number of 64-step blocks long take a route of their own in
    the window kernel when the batch is longer than the window; batches that are not a
    whole number of blocks, that start inside a window, and a length (192) without that
    route are all checked against the oracle's re-summed windows."""
    say(f"case window W={W} T={T} chunks={chunks}")
    R, M = 2048, 1
    g = torch.Generator().manual_seed(W + T)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64))
    # ranks and nodes that are anomalous on and off, so that counts rise and fall
    for i in range(40):
        r = int(torch.randint(0, R, (1,), generator=g))
        on = torch.rand(T, generator=g) < (0.2 + 0.02 * i)
        x[on, 0, r] *= 1.5
    for n in (3, 77, 200):
        on = torch.rand(T, generator=g) < 0.6
        x[on, 0, n * 8:(n + 1) * 8] *= 1.2
    x = x.to(torch.float32)
    p = oracle_params(R=R, M=M, W=W, k=max(1, W // 3), min_signals=1)
    rep = run_and_compare(p, x, topk_k=16, chunks=chunks, label=f"W{W}", want_z=False)
    say("  report", rep)
    assert rep["rank_flags"] >= 1


def _random_window_case(seed, long_batches=False):
    """gd_update_window / gd_flags / gd_topk_nodes on seeded random anomaly words and node
    scores (not on scoring outputs), against the oracle's re-summed windows.
    long_batches: short windows and histories of many windows in few calls."""
    rng = np.random.default_rng(3000 + seed + (500000 if long_batches else 0))
    R = 8 * int(np.exp(rng.uniform(0, np.log(300 if long_batches else 2000))))
    N = R // 8
    if long_batches:
        W = int(rng.choice([1, 3, 17, 64, 100, 128, 130, 192]))
        T = int(rng.integers(4 * W + 600, 24 * W + 3000))
    else:
        W = int(rng.choice([int(np.exp(rng.uniform(0, np.log(1024)))), 64 * int(rng.integers(1, 17))]))
        T = int(rng.integers(1, 3 * W + 70))
    k = int(rng.integers(1, W + 1))
    cuts = sorted(set(rng.integers(1, max(2, T), size=int(rng.integers(0, 4))).tolist()) - {T})
    batches = [b - a for a, b in zip([0] + cuts, cuts + [T])]
    say(f"case random window seed={seed} R={R} W={W} k={k} T={T} batches={batches}")
    if long_batches and max(batches) <= max(4 * W, 512):
        batches = [T]
    density = rng.choice([0.02, 0.3, 0.7, 0.97], size=(1, R))                 # per rank
    rank_bits = rng.random((T, R)) < density
    node_bits = rng.random((T, N)) < rng.choice([0.05, 0.5, 0.9], size=(1, N))

    def pack(bits):
        n = bits.shape[1]
        padded = np.zeros((T, (n + 63) // 64 * 64), np.uint8)
        padded[:, :n] = bits
        return np.packbits(padded.reshape(T, -1, 64), axis=2, bitorder="little").view(np.uint64).reshape(T, -1)

    ra, na = pack(rank_bits), pack(node_bits)
    node_z = rng.standard_normal((T, N)).astype(np.float32)
    node_z[rng.random((T, N)) < 0.3] = 0.25          # equal scores: ties in the ranking
    p = oracle_params(R=R, M=1, W=W, k=k, min_signals=1)
    pr, pn = oracle.window(R, ra, W, k), oracle.window(N, na, W, k)
    topk_k = int(rng.integers(1, N + 1))
    d = dict(ranks=pr, nodes=pn, node_flag_byte=oracle.node_flag_byte(8, pn.flag, pr.flag))
    d["topk_idx"], d["topk_key"] = oracle.topk(pn.count, node_z[-1], topk_k)
    det = detector_for(p, topk=topk_k)
    dra, dna, dnz = (torch.from_numpy(a.view(np.int64) if a.dtype == np.uint64 else a).cuda() for a in (ra, na, node_z))
    t0 = 0
    for c in batches:
        det.update_window(dict(rank_anom=dra[t0:t0 + c], node_anom=dna[t0:t0 + c], node_z=dnz[t0:t0 + c]), c)
        t0 += c
    compare_decision(p, d, det, topk_k, label=f"random window {seed}")
    det.close()


@pytest.mark.parametrize("seed", range(24))
def test_window_random_configurations(seed):
    _random_window_case(seed)


@pytest.mark.parametrize("seed", range(16))
def test_window_random_long_batches(seed):
    _random_window_case(seed, long_batches=True)


@pytest.mark.parametrize("R,T", [(256, 9000), (1024, 9000), (4096, 2400), (16384, 2400), (65536, 800)])
def test_hinted_runs_under_regime_changes(R, T):
    _regime_case(R, T, R // 7 + T)


def _regime_case(R, T, seed):
    """Long enough batches that every workgroup scores several consecutive steps and
    carries the previous step's median, reach and MAD over as hints -- on data whose
    level, spread and character keep changing from one step to the next: level jumps,
    spread collapsing to ties or exploding, two-valued and constant columns, signs,
    missing samples, then calm again."""
    say(f"case regime changes R={R} T={T} seed={seed}")
    M = 2
    g = torch.Generator().manual_seed(seed)
    level = torch.ones(T, dtype=torch.float64)
    spread = torch.full((T,), 0.02, dtype=torch.float64)
    kind = torch.zeros(T, dtype=torch.int64)
    t = 0
    while t < T:
        run = int(torch.randint(1, 12, (1,), generator=g))
        k = int(torch.randint(0, 10, (1,), generator=g))
        lv = float(torch.exp(torch.randn(1, generator=g) * (3.0 if k == 1 else 0.05)))
        sp = [0.02, 0.02, 2.0, 1e-6, 0.0, 0.02, 0.02, 0.02, 0.3, 0.02][k]
        level[t:t + run] = lv
        spread[t:t + run] = sp
        kind[t:t + run] = k
        t += run
    x = level[:, None, None] * torch.exp(spread[:, None, None] *
                                         torch.randn((T, M, R), generator=g, dtype=torch.float64))
    x[:, 1] = 300.0 / x[:, 1]
    for t in range(T):
        k = int(kind[t])
        if k == 5:                                   # two values
            x[t, 0] = torch.where(torch.rand(R, generator=g, dtype=torch.float64) < 0.5, level[t], level[t] * 1.01)
        elif k == 6:                                 # signs
            x[t, 0, ::3] = -x[t, 0, ::3]
        elif k == 7:                                 # missing samples
            x[t, 0, torch.randperm(R, generator=g)[: max(1, R // 9)]] = NAN
            x[t, 1, int(torch.randint(0, R, (1,), generator=g))] = NAN
    x[:, :, 8:16] *= 1.15
    x = x.to(torch.float32)
    p = oracle_params(R=R, M=M, W=8, k=4, directions=(1, -1), min_signals=1)
    det = detector_for(p)
    det.set_streaming_steps(0)
    out = gpu_score(det, x, want_z=False)
    o = oracle.score(p, x.numpy(), want_z=False)
    rep = compare_scores(o, out, "regime changes")
    say("  report", rep)
    det.close()


HINTED_KINDS = ["binade", "huge", "integers", "tied_centre", "denormal", "ramp", "one_sided", "bimodal",
                "narrowing"]


@pytest.mark.parametrize("R", [1024, 4096, 65536])
@pytest.mark.parametrize("kind", HINTED_KINDS)
def test_hinted_selection_on_stationary_runs_of_awkward_columns(kind, R):
    """Several consecutive steps of the same kind of column in exact-fit tilings, so that from
    the second step on the hinted selection runs (bracket, median and MAD carried over): columns
    centred on a power of two, magnitudes beyond its key limit, integer sensors, a third of the
    ranks tied at the centre, denormals, sorted ranks (every candidate in one wave), one-sided
    and bimodal distributions (the two distance ranges far from symmetric, or falling into a
    gap), and a spread that shrinks a hundredfold from one step to the next."""
    # (a batch is dealt out in runs of ceil(T / workgroups) consecutive steps: three steps per run here)
    T, M = {1024: 12300, 4096: 3080, 65536: 772}[R], 3
    say(f"case hinted selection kind={kind} R={R} T={T}")
    g = torch.Generator().manual_seed(len(kind) * 1000 + R)
    n = torch.randn((T, M, R), generator=g, dtype=torch.float32).to(torch.float64)
    u = torch.rand((T, M, R), generator=g, dtype=torch.float32).to(torch.float64).clamp_(1e-7, 1.0)
    if kind == "binade":
        centre = torch.tensor([1.0, 2.0, 0.5], dtype=torch.float64)[None, :, None]
        x = centre * (1.0 + 3e-4 * n)
    elif kind == "huge":
        x = 1.5e38 * torch.exp(0.02 * n)
        x[:, 1] = 2e37 * torch.exp(0.3 * n[:, 1])
    elif kind == "integers":
        x = torch.round(65.0 + 2.0 * n)
        x[:, 2] = torch.round(1000.0 + 40.0 * n[:, 2])
    elif kind == "tied_centre":
        x = torch.exp(0.02 * n)
        x = torch.where(u < 0.33, torch.ones_like(x), x)
    elif kind == "denormal":
        x = 3e-41 * torch.exp(0.1 * n)
        x[:, 1] = 1.2e-38 * (1.0 + 0.01 * n[:, 1])         # straddles the smallest normal number
    elif kind == "ramp":
        x = (1.0 + torch.arange(R, dtype=torch.float64) / R)[None, None, :] * (1.0 + 1e-3 * n[:, :, :1])
        x[:, 1] = torch.flip(x[:, 1], dims=[-1])
    elif kind == "one_sided":
        x = 1.0 - torch.log(u) * 0.05                        # exponential tail to the right only
        x[:, 2] = 400.0 + torch.log(u[:, 2]) * 7.0           # ... and to the left only
    elif kind == "bimodal":
        x = torch.where(u < 0.5, 1.0 + 0.001 * n, 1.3 + 0.001 * n)
        x[:, 1] = torch.where(u[:, 1] < 0.26, 0.8 + 0.01 * n[:, 1], 1.0 + 0.0005 * n[:, 1])
    elif kind == "narrowing":
        spread = torch.tensor([0.05 * 0.01 ** (t % 3) for t in range(T)], dtype=torch.float64)[:, None, None]
        x = 1.0 + spread * n
    x = x.to(torch.float32)
    x[:, :, 8:16] *= 1.2 if kind != "huge" else 1.0           # one slow node
    dirs = (1, -1, 1)
    p = oracle_params(R=R, M=M, W=4, k=2, directions=dirs)
    import gpu_harness
    gpu_harness.STREAMING_STEPS = 0                             # whole-run route: hints carried from step to step
    try:
        rep = run_and_compare(p, x, topk_k=min(8, R // 8), chunks=[T], label=f"{kind}-R{R}")
    finally:
        gpu_harness.STREAMING_STEPS = None
    say("  report", rep)
    assert rep["z_bit_exact"]


# (threads, float4 rows) of the exact-fit tiling of a rank count: the sample behind a run's
# first hints is register row 0, i.e. ranks (w % rows) * threads * 4 + thread * 4 + 0..3 of
# thread (w * 64 + lane)
_SAMPLE_TILING = {1024: (64, 4), 4096: (256, 4), 16384: (256, 16), 65536: (1024, 16)}
SAMPLE_KINDS = ["far_above", "other_scale", "too_tight", "missing", "negative", "constant", "lowest_values"]


@pytest.mark.parametrize("R", sorted(_SAMPLE_TILING))
@pytest.mark.parametrize("kind", SAMPLE_KINDS)
def test_first_step_hints_from_unrepresentative_samples(kind, R):
    """The first step of a run takes its hints from a sample of the column (one register row
    per thread).  Here exactly the sampled ranks are made misleading -- far above the rest, on
    another scale, squeezed around the centre, missing, negative, constant, or the lowest
    values of the column -- so that the sampled median, quartiles or both point the wrong way;
    the selection must notice and still return the exact statistics.  Every step of these short
    batches is a first step."""
    nt, rows = _SAMPLE_TILING[R]
    T, M = 5, 3
    say(f"case sampled hints kind={kind} R={R}")
    g = torch.Generator().manual_seed(len(kind) * 77 + R)
    n = torch.randn((T, M, R), generator=g, dtype=torch.float64)
    x = torch.exp(0.02 * n)
    x[:, 1] = 400.0 / x[:, 1]
    thread = torch.arange(nt)
    first = ((thread // 64) % rows) * nt * 4 + thread * 4
    sampled = (first[:, None] + torch.arange(4)[None, :]).reshape(-1)
    assert int(sampled.max()) < R and len(set(sampled.tolist())) == 4 * nt
    s = x[:, :, sampled]
    if kind == "far_above":
        s = s * 50.0
    elif kind == "other_scale":
        s = 1.0 + (s - 1.0) * 300.0
        s[:, 1] = 400.0 + (x[:, 1][:, sampled] - 400.0) * 300.0
        s = s.abs() + 1e-3
    elif kind == "too_tight":
        c = x.median(dim=-1, keepdim=True).values
        s = c + (s - c) * 1e-3
    elif kind == "missing":
        s = torch.full_like(s, float("nan"))
        s[:, 2] = x[:, 2][:, sampled]                       # (one metric keeps its samples)
    elif kind == "negative":
        s = -s
    elif kind == "constant":
        s = torch.full_like(s, 1.0)
    elif kind == "lowest_values":
        srt = torch.sort(x, dim=-1).values                  # the sample holds the lowest values,
        rest = torch.ones(R, dtype=torch.bool)              # the other ranks the rest in order
        rest[sampled] = False
        x[:, :, rest] = srt[:, :, 4 * nt:]
        s = srt[:, :, : 4 * nt]
    x[:, :, sampled] = s
    x = x.to(torch.float32)
    p = oracle_params(R=R, M=M, W=4, k=2, directions=(1, -1, 0))
    import gpu_harness
    gpu_harness.STREAMING_STEPS = 0                             # whole-run route
    try:
        rep = run_and_compare(p, x, topk_k=min(8, R // 8), chunks=[T], label=f"sample-{kind}-R{R}")
    finally:
        gpu_harness.STREAMING_STEPS = None
    say("  report", rep)


@pytest.mark.parametrize("R", [16384, 65536])
def test_node_mask_at_any_byte_offset(R):
    """The node mask is a byte array and may start at any address: the batch route writes it
    eight bytes at a time where the address allows and byte by byte otherwise.  Both ways
    must give the oracle's bytes (and leave the bytes around the array alone)."""
    T, M = 3, 2
    say(f"case node mask offsets R={R}")
    g = torch.Generator().manual_seed(R + 5)
    x = torch.exp(0.02 * torch.randn((T, M, R), generator=g, dtype=torch.float64))
    x[:, :, 64:72] *= 1.3                                    # a slow node: some node bits are set
    x[:, :, 4096:4104] *= 1.2
    x = x.to(torch.float32)
    p = oracle_params(R=R, M=M, W=4, k=2, directions=(1, 1))
    want = oracle.score(p, x.numpy(), want_z=False)
    assert want.node_mask.any()
    det = detector_for(p)
    det.set_streaming_steps(0)                              # the batch route
    xd = x.cuda()
    N = R // 8
    for off in (0, 1, 4, 7):
        out = det.alloc_outputs(T)
        big = torch.full((T * N + 32,), 0xAB, dtype=torch.uint8, device="cuda")
        out["node_mask"] = big[8 + off: 8 + off + T * N].view(T, N)
        assert out["node_mask"].data_ptr() % 8 == off
        det.score_batch(xd, out)
        torch.cuda.synchronize()
        assert np.array_equal(out["node_mask"].cpu().numpy(), want.node_mask), f"offset {off}"
        assert np.array_equal(out["node_anom"].cpu().numpy().view(np.uint64), want.node_anom), f"offset {off}"
        assert bool((big[: 8 + off] == 0xAB).all()) and bool((big[8 + off + T * N:] == 0xAB).all())
    det.close()
