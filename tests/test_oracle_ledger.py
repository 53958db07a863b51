"""Pins of the oracle's bookkeeping beyond the default rule -- persistence kept per
indicator, the ranking by the node score averaged over the window, and the
recurrence count of the triage workflow (three times within a week, Section 7) --
against things other than the oracle: sliding sums by cumulative sums, the already
pinned single-ring persistence in the cases where the two rules coincide, hand-built
timelines with known answers, exactly representable scores and Python's sort."""
import numpy as np
import pytest

import oracle


def sliding_counts(bits, W):
    """bits [T][n] of 0/1 -> number of ones among the last W steps, by cumulative sums."""
    c = np.cumsum(bits.astype(np.int64), axis=0)
    out = c.copy()
    out[W:] -= c[:-W]
    return out


def pack_bits(bits):
    T, n = bits.shape
    words = np.zeros((T, (n + 63) // 64), np.uint64)
    for i in range(n):
        words[:, i // 64] |= bits[:, i].astype(np.uint64) << np.uint64(i % 64)
    return words


# ---- the per-step rule on exceed bytes ------------------------------------------------

def test_combine_reproduces_the_anomaly_words_of_the_scoring_oracle():
    """go_score applies the rule while it scores (pinned there on constructed cases); the
    stand-alone version must give the same words from the same bytes."""
    rng = np.random.default_rng(8)
    for M, primary, min_signals in ((4, 0, 2), (3, 2, 1), (8, 5, 4), (1, 0, 1)):
        p = oracle.Params(R=136, M=M, W=4, k=2, thr=0.3, primary=primary, min_signals=min_signals,
                          directions=(1, -1, 0, 1, 1, -1, 0, 1)[:M])
        x = np.exp(0.1 * rng.standard_normal((7, M, 136))).astype(np.float32)
        s = oracle.score(p, x, want_z=False)
        assert s.exceed_mask.any() and s.rank_anom.any()
        assert np.array_equal(oracle.combine(s.exceed_mask, primary, min_signals), s.rank_anom)
        assert np.array_equal(oracle.combine(s.node_mask, primary, min_signals), s.node_anom)


def test_combine_by_hand():
    byte = np.array([[0b0000, 0b0001, 0b0010, 0b0011, 0b0110, 0b0111, 0b1111] + [0] * 60 + [0b0101]], np.uint8)
    w = oracle.combine(byte, 0, 2)            # needs bit 0 and one more
    assert w.shape == (1, 2)
    assert int(w[0, 0]) == (1 << 3) | (1 << 5) | (1 << 6) and int(w[0, 1]) == 1 << 3
    w = oracle.combine(byte, 1, 3)            # needs bit 1 and two more
    assert int(w[0, 0]) == (1 << 5) | (1 << 6) and int(w[0, 1]) == 0
    w = oracle.combine(byte, 2, 1)            # bit 2 alone is enough
    assert int(w[0, 0]) == (1 << 4) | (1 << 5) | (1 << 6) and int(w[0, 1]) == 1 << 3


# ---- persistence per indicator ------------------------------------------------------

@pytest.mark.parametrize("W,k", [(1, 1), (5, 3), (16, 16), (40, 7)])
def test_metric_window_against_cumulative_sums(W, k):
    rng = np.random.default_rng(W * 100 + k)
    T, n = 90, 37
    mask = (rng.random((T, n, 8)) < [0.6, 0.4, 0.5, 0.3, 0.7, 0.2, 0.5, 0.9]).astype(np.uint8)
    byte = (mask << np.arange(8, dtype=np.uint8)).sum(axis=2).astype(np.uint8)
    primary, min_signals = 2, 3
    o = oracle.metric_window(byte, primary, min_signals, W, k)
    counts = np.stack([sliding_counts(mask[:, :, m], W) for m in range(8)])      # [8][T][n]
    persistent = counts >= k
    flag = persistent[primary] & (persistent.sum(axis=0) >= min_signals)         # [T][n]
    assert np.array_equal(o.count, counts[:, -1].astype(np.uint16))
    want_pmask = (persistent[:, -1].astype(np.uint8) << np.arange(8, dtype=np.uint8)[:, None]).sum(axis=0)
    assert np.array_equal(o.pmask, want_pmask.astype(np.uint8))
    assert np.array_equal(o.flag, flag[-1].astype(np.uint8))
    first = np.where(flag.any(axis=0), flag.argmax(axis=0), -1)
    assert np.array_equal(o.first, first.astype(np.int32))


def test_one_metric_is_the_single_ring_persistence():
    """With one indicator both rules are the same rule: the result must equal the
    single-ring persistence (pinned on its own) of the same bits."""
    rng = np.random.default_rng(1)
    T, n, W, k = 120, 70, 12, 9
    bits = (rng.random((T, n)) < 0.7).astype(np.uint8)
    o = oracle.metric_window(bits, 0, 1, W, k)
    ref = oracle.window(n, pack_bits(bits), W, k)
    assert np.array_equal(o.count[0], ref.count) and not o.count[1:].any()
    assert np.array_equal(o.flag, ref.flag) and np.array_equal(o.first, ref.first)
    assert np.array_equal(o.pmask, ref.flag)


def test_where_the_two_readings_differ():
    """Two indicators that deviate on alternate steps never coincide, so combining per
    step finds nothing, while each is sustained on its own (k of W = 4 of 10)."""
    T, W, k = 30, 10, 4
    byte = np.zeros((T, 2), np.uint8)
    byte[0::2, 0] = 1          # item 0: metric 0 on even steps,
    byte[1::2, 0] = 2          #         metric 1 on odd steps
    byte[:, 1] = 1             # item 1: only the primary, all the time
    o = oracle.metric_window(byte, 0, 2, W, k)
    assert o.flag.tolist() == [1, 0] and o.pmask.tolist() == [3, 1]
    # metric 0 reaches 4 at step 6 (0,2,4,6), metric 1 at step 7 (1,3,5,7)
    assert o.first.tolist() == [7, -1]
    per_step = ((byte & 1) > 0) & ((byte & 2) > 0)
    assert not per_step.any()
    # the primary is required: sustained supporting indicators alone do not flag
    o = oracle.metric_window(np.where(byte == 1, 0, byte).astype(np.uint8) | np.uint8(4), 0, 2, W, k)
    assert not o.flag.any() and (o.pmask & 4).all()


def test_metric_window_ends_when_the_deviation_does():
    T, W, k = 60, 8, 6
    byte = np.zeros((T, 1), np.uint8)
    byte[10:30, 0] = 3
    o = oracle.metric_window(byte[:30], 0, 2, W, k)
    assert o.flag[0] == 1 and o.first[0] == 15 and o.count[:2, 0].tolist() == [8, 8]
    o = oracle.metric_window(byte[:33], 0, 2, W, k)          # 3 clean steps: 5 of 8 left
    assert o.flag[0] == 0 and o.first[0] == 15 and o.count[0, 0] == 5
    o = oracle.metric_window(byte[:0], 0, 2, W, k)
    assert not o.flag.any() and not o.count.any() and o.first[0] == -1


# ---- windowed score sum and its ranking ---------------------------------------------

def test_score_ring_on_exactly_representable_scores():
    rng = np.random.default_rng(2)
    T, N, W = 50, 24, 16
    units = rng.integers(-500, 500, (T, N))                  # scores that are whole multiples of 1/64
    z = (units / 64.0).astype(np.float32)
    assert np.array_equal(oracle.score_ring(z, W), units[-W:].sum(axis=0).astype(np.int32))
    assert np.array_equal(oracle.score_ring(z[:5], W), units[:5].sum(axis=0).astype(np.int32))
    assert not oracle.score_ring(z[:0], W).any()
    # another grid: quant = 4 keeps quarters
    z4 = (units / 4.0).astype(np.float32)
    assert np.array_equal(oracle.score_ring(z4, W, 4.0), units[-W:].sum(axis=0).astype(np.int32))


def test_score_ring_rounding_clamping_and_missing():
    f = np.float32
    z = np.array([[0.5 / 64, 1.5 / 64, 2.5 / 64, -0.5 / 64, -1.5 / 64, 0.49 / 64, 0.51 / 64,
                   511.99, 512.0, 1e30, -512.0, -513.0, -1e30, np.inf, -np.inf, np.nan]], f)
    want = [0, 2, 2, 0, -2, 0, 1, 32767, 32767, 32767, -32768, -32768, -32768, 32767, -32768, 0]
    assert oracle.score_ring(z, 4).tolist() == want
    # the window sum of saturated scores stays far inside 32 bits
    big = np.full((1024, 1), 1e9, f)
    assert oracle.score_ring(big, 1024)[0] == 1024 * 32767


def test_score_ring_only_the_last_w_steps():
    z = np.zeros((40, 2), np.float32)
    z[:30, 0] = 5.0                  # over before the window starts
    z[30:, 1] = 0.25
    assert oracle.score_ring(z, 10).tolist() == [0, 10 * 16]
    assert oracle.score_ring(z, 11).tolist() == [320, 10 * 16]


def test_topk_mean_against_python_sort():
    rng = np.random.default_rng(3)
    N = 300
    count = rng.integers(0, 4, N).astype(np.uint16)
    s = rng.integers(-40, 40, N).astype(np.int32)            # many ties in both fields
    s[:3] = [-2**31 + 5, 2**25, -2**25]
    idx, key = oracle.topk_mean(count, s, 50)
    order = sorted(range(N), key=lambda n: (-int(count[n]), -int(s[n]), n))[:50]
    assert idx.tolist() == order
    for j, n in enumerate(order):
        want = (int(count[n]) << 48) | ((int(s[n]) + 2**31) << 16) | (0xFFFF - n)
        assert int(key[j]) == want
    assert all(int(key[j]) > int(key[j + 1]) for j in range(49))


# ---- recurrence ------------------------------------------------------------------------

def timeline(T, spans):
    f = np.zeros((T, 1), np.uint8)
    for a, b in spans:
        f[a:b, 0] = 1
    return f


def test_three_episodes_within_the_horizon():
    f = timeline(100, [(10, 20), (30, 40), (50, 60)])
    ep, tf = oracle.recurrence(f, 45, 3)         # starts 10, 30, 50; at t = 50 all lie in (5, 50]
    assert tf[0] == 50
    ep, tf = oracle.recurrence(f, 41, 3)         # (9, 50] still holds the start at 10
    assert tf[0] == 50
    ep, tf = oracle.recurrence(f, 40, 3)         # (10, 50] does not
    assert tf[0] == -1
    # episodes still inside the horizon at the last step (t = 99)
    assert oracle.recurrence(f, 100, 3)[0][0] == 3
    assert oracle.recurrence(f, 60, 3)[0][0] == 1          # (39, 99]: the start at 50
    assert oracle.recurrence(f, 70, 3)[0][0] == 2          # (29, 99]: 30 and 50
    assert oracle.recurrence(f, 49, 3)[0][0] == 0
    assert oracle.recurrence(f, 1000, 2)[0][0] == 2        # saturates at the limit
    assert oracle.recurrence(f, 1000, 2)[1][0] == 30


def test_one_long_episode_counts_once_and_step_zero_can_start_one():
    f = timeline(50, [(0, 50)])
    ep, tf = oracle.recurrence(f, 1000, 2)
    assert ep[0] == 1 and tf[0] == -1
    f = timeline(50, [(0, 1), (2, 3), (4, 5)])
    ep, tf = oracle.recurrence(f, 1000, 3)
    assert ep[0] == 3 and tf[0] == 4
    ep, tf = oracle.recurrence(f[:0], 10, 3)
    assert ep[0] == 0 and tf[0] == -1


def test_recurrence_against_numpy_edges():
    rng = np.random.default_rng(4)
    T, N, H, J = 400, 20, 90, 3
    f = np.zeros((T, N), np.uint8)
    for n in range(N):
        t = 0
        while t < T:
            t += int(rng.integers(5, 60))
            d = int(rng.integers(1, 30))
            f[t:t + d, n] = 1
            t += d
    ep, tf = oracle.recurrence(f, H, J)
    prev = np.vstack([np.zeros((1, N), np.uint8), f[:-1]])
    rises = (f == 1) & (prev == 0)
    in_window = sliding_counts(rises, H)                     # starts within (t - H, t]
    want_tf = np.where((in_window >= J).any(axis=0), (in_window >= J).argmax(axis=0), -1)
    assert np.array_equal(tf, want_tf.astype(np.int32))
    assert np.array_equal(ep, np.minimum(in_window[-1], J).astype(np.uint8))
    assert (tf >= 0).any() and (tf < 0).any()
