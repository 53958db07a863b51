"""Pins for the oracle's persistence, node flag byte, ranking and whole path."""
import numpy as np
import pytest

import oracle
from workloads import generate, workload


def pack_bits(a):
    """a[T][n] of 0/1 -> u64 words [T][ceil(n/64)], bit i%64 of word i/64."""
    T, n = a.shape
    words = (n + 63) // 64
    out = np.zeros((T, words), np.uint64)
    for i in range(n):
        out[:, i // 64] |= a[:, i].astype(np.uint64) << np.uint64(i % 64)
    return out


# ---------------------------------------------------------------- persistence
@pytest.mark.parametrize("W,k", [(1, 1), (5, 3), (20, 15), (64, 64), (7, 1)])
def test_window_counts_against_prefix_sums(W, k):
    rng = np.random.default_rng(W * 100 + k)
    T, n = 150, 70
    a = (rng.random((T, n)) < 0.6).astype(np.uint8)
    a[:, 3] = 1
    a[:, 4] = 0
    o = oracle.window(n, pack_bits(a), W, k, want_hist=True)
    cs = np.vstack([np.zeros((1, n), np.int64), np.cumsum(a, axis=0)])
    for t in range(T):
        lo = max(0, t + 1 - W)
        assert np.array_equal(o.count_hist[t], cs[t + 1] - cs[lo])
    flags = o.count_hist >= k
    assert np.array_equal(o.count, o.count_hist[-1])
    assert np.array_equal(o.flag.astype(bool), flags[-1])
    first = np.where(flags.any(0), flags.argmax(0), -1)
    assert np.array_equal(o.first, first)
    assert o.first[3] == k - 1 and o.first[4] == -1       # warm-up: no flag before step k-1


def test_window_empty_history():
    o = oracle.window(16, np.zeros((0, 1), np.uint64), 5, 3)
    assert not o.count.any() and not o.flag.any() and (o.first == -1).all()


def test_run_of_anomalies_flags_and_unflags_at_exact_steps():
    W, k, T = 20, 15, 200
    t0, t1 = 50, 120                      # anomalous on [t0, t1)
    a = np.zeros((T, 1), np.uint8)
    a[t0:t1] = 1
    o = oracle.window(1, pack_bits(a), W, k, want_hist=True)
    flagged = np.flatnonzero(o.count_hist[:, 0] >= k)
    assert o.first[0] == t0 + k - 1 == flagged[0]
    assert flagged[-1] + 1 == t1 + W - k    # first unflagged step after the run
    assert o.count_hist[:, 0].max() == W


def test_spikes_never_flag_when_rarer_than_k_per_window():
    rng = np.random.default_rng(0)
    W, k, T, n = 50, 4, 3000, 256
    a = np.zeros((T, n), np.uint8)
    # one spike per block of 25 steps: 50 consecutive steps touch at most 3 blocks
    for i in range(n):
        for b in range(0, T, 25):
            if rng.random() < 0.7:
                a[b + rng.integers(0, 25), i] = 1
    o = oracle.window(n, pack_bits(a), W, k, want_hist=True)
    assert o.count_hist.max() <= 3 and not o.flag.any() and (o.first == -1).all()


# ---------------------------------------------------------------- constructed margin
def test_injected_straggler_is_recovered_at_the_constructed_step():
    """Raise one rank to med + (thr + delta) * s on [t0, t1), using the column's
    own post-injection med and s, and check the first/last flagged steps."""
    rng = np.random.default_rng(12)
    R, T, W, k = 256, 160, 20, 15
    t0, t1, r0 = 30, 110, 77
    thr, delta = 3.5, 0.75
    x = np.exp(0.02 * rng.standard_normal((T, 1, R))).astype(np.float32)
    p = oracle.Params(R=R, M=1, W=W, k=k, min_signals=1, thr=thr)
    for t in range(t0, t1):
        x[t, 0, r0] = 10.0                      # any value far above; med/s are then fixed
        s = oracle.score(p, x[t:t + 1])
        scale = max(np.float32(1.4826) * s.mad[0, 0], np.float32(1e-6) * abs(s.med[0, 0]))
        x[t, 0, r0] = np.float32(s.med[0, 0] + (thr + delta) * scale)
    # clean steps: keep rank r0 well below the threshold
    for t in list(range(0, t0)) + list(range(t1, T)):
        x[t, 0, r0] = np.float32(np.median(x[t, 0]))
    d = oracle.detect(p, x, topk_k=4, want_z=True)
    z = d["scores"].z[:, 0, r0]
    assert np.all(np.abs(z[t0:t1] - (thr + delta)) < 0.05)
    hist = oracle.window(R, d["scores"].rank_anom, W, k, want_hist=True).count_hist[:, r0]
    flagged = np.flatnonzero(hist >= k)
    assert flagged[0] == t0 + k - 1 == d["ranks"].first[r0]
    assert flagged[-1] + 1 == t1 + W - k
    others = np.delete(np.arange(R), r0)
    assert (d["ranks"].first[others] == -1).all()


def test_whole_node_injection_flags_the_node_not_its_gpus():
    rng = np.random.default_rng(13)
    R, T, W, k, node = 512, 80, 10, 8, 9
    x = np.exp(0.02 * rng.standard_normal((T, 2, R))).astype(np.float32)
    x[20:, :, node * 8: node * 8 + 8] *= np.float32(1.045)   # ~2.2 sigma per GPU, ~6.2 per node
    p = oracle.Params(R=R, M=2, W=W, k=k)
    d = oracle.detect(p, x, topk_k=3)
    assert d["nodes"].first[node] == 20 + k - 1
    assert (np.delete(d["nodes"].first, node) == -1).all()
    assert (d["ranks"].first == -1).all()
    assert d["node_flag_byte"][node] == 1 and d["topk_idx"][0] == node


# ---------------------------------------------------------------- node flag byte, top-k
def test_node_flag_byte():
    nf = np.array([0, 1, 0, 1], np.uint8)
    rf = np.zeros(32, np.uint8)
    rf[8 * 2 + 7] = 1
    rf[8 * 3] = 1
    assert oracle.node_flag_byte(8, nf, rf).tolist() == [0, 1, 2, 3]


def order_key(f):
    b = np.asarray(f, np.float32).view(np.uint32).astype(np.uint64)
    return np.where(b & np.uint64(0x80000000), ~b & np.uint64(0xFFFFFFFF), b | np.uint64(0x80000000))


def test_topk_against_brute_force_sort():
    rng = np.random.default_rng(2)
    N = 300
    cnt = rng.integers(0, 4, N).astype(np.uint16)
    z = rng.standard_normal(N).astype(np.float32)
    z[10:40] = z[9]             # ties in score -> index decides
    z[50] = 0.0
    z[51] = -0.0                # numerically equal zeros -> index decides
    cnt[50] = cnt[51] = 3
    z[52] = 0.0; cnt[52] = 3
    tup = sorted(range(N), key=lambda n: (-int(cnt[n]), -float(z[n]), n))
    for k in (0, 1, 64, N):
        idx, key = oracle.topk(cnt, z, k)
        assert idx.tolist() == tup[:k]
        if k:
            zc = np.where(z[idx] == 0, np.float32(0), z[idx])
            want = (cnt[idx].astype(np.uint64) << np.uint64(48)) | (order_key(zc) << np.uint64(16)) \
                | (np.uint64(0xFFFF) - idx.astype(np.uint64))
            assert np.array_equal(key, want)
            assert np.all(key[:-1] > key[1:])     # keys are unique and sorted high to low
    i50, i51, i52 = tup.index(50), tup.index(51), tup.index(52)
    assert i50 < i51 < i52


# ---------------------------------------------------------------- the tiny configuration
def test_tiny_configuration_end_to_end():
    w = workload(0)
    x = generate(w, seed=0).numpy()
    p = oracle.Params(R=w.R, M=w.M, W=w.W, k=w.k, thr=w.thr, directions=w.directions)
    d = oracle.detect(p, x, topk_k=w.topk, want_z=True)
    z = d["scores"].z[:, 0, :]
    # a 15% slowdown at sigma = 2% is ~7 robust sigmas
    assert 5.0 < np.median(z[50:, 5]) < 9.5 and 5.0 < np.median(z[50:, 42]) < 9.5
    flagged = set(np.flatnonzero(d["ranks"].first >= 0).tolist())
    assert flagged == {5, 42}
    assert d["ranks"].first[5] == 50 + w.k - 1 and d["ranks"].first[42] == 50 + w.k - 1
    nb = d["node_flag_byte"]
    assert nb[0] & 2 and nb[5] & 2 and not (np.delete(nb, [0, 5]) & 2).any()
