"""Pins of the oracle's severity tiers (Section 4.2, tiered response by the size
of the slowdown) against things other than the oracle itself: exact rational
arithmetic with explicit fp32 rounding, numpy's median of float32, slowdowns
constructed to be exactly representable, the extent of the window, both
directions and the tier boundaries."""
from fractions import Fraction

import numpy as np
import pytest

import oracle
from exactfp import F, add32, div32, mul32, sub32


def params(R=64, M=2, W=4, **kw):
    return oracle.Params(R=R, M=M, W=W, k=min(2, W), **kw)


def flat_history(T, M, R, value=1.0):
    return np.full((T, M, R), value, np.float32)


def test_exactly_representable_slowdowns_and_tiers():
    p = params()
    T = 6
    x = flat_history(T, p.M, p.R, 2.0)
    med = np.full((T, p.M), 2.0, np.float32)
    x[:, 0, 8:16] = 2.5       # node 1: quotient 1.25 exactly   -> 0.25, severe
    x[:, 0, 16:24] = 2.25     # node 2: 1.125                    -> 0.125, moderate
    x[:, 0, 24:32] = 2.125    # node 3: 1.0625                   -> 0.0625, no observable impact
    x[:, 0, 32:40] = 1.5      # node 4: faster than its peers    -> -0.25
    flag = np.zeros(p.N, np.uint8)
    flag[1:5] = 1
    flag[6] = 2               # flagged through one of its ranks, no slowdown
    slow, tier = oracle.severity(p, x, med, flag)
    assert slow[1] == np.float32(0.25) and tier[1] == 3
    assert slow[2] == np.float32(0.125) and tier[2] == 2
    assert slow[3] == np.float32(0.0625) and tier[3] == 1
    assert slow[4] == np.float32(-0.25) and tier[4] == 1
    assert slow[6] == 0.0 and tier[6] == 1
    # nodes that are not flagged report nothing, whatever their data
    x[:, 0, 40:48] = 9.0
    slow, tier = oracle.severity(p, x, med, flag)
    assert slow[5] == 0.0 and tier[5] == 0 and slow[0] == 0.0 and tier[0] == 0


def test_tier_boundaries_are_inclusive_below():
    p = params()
    x = flat_history(3, p.M, p.R, 1.0)
    med = np.ones((3, p.M), np.float32)
    x[:, 0, 0:8] = 1.25
    flag = np.zeros(p.N, np.uint8)
    flag[0] = 1
    for moderate, severe, want in [(0.25, 0.5, 2), (0.1, 0.25, 3), (0.26, 0.5, 1), (0.1, 0.26, 2)]:
        slow, tier = oracle.severity(p, x, med, flag, moderate, severe)
        assert slow[0] == np.float32(0.25) and tier[0] == want, (moderate, severe)


def test_only_the_last_w_steps_count():
    p = params(W=4)
    T = 10
    x = flat_history(T, p.M, p.R, 1.0)
    med = np.ones((T, p.M), np.float32)
    x[:6, 0, 8:16] = 3.0              # a slowdown that ended before the window
    x[6:, 0, 16:24] = 1.5             # one that fills the window exactly
    x[7:, 0, 24:32] = 1.5             # 3 of the 4 window steps: the median is the slow value
    x[8:, 0, 32:40] = 1.5             # half of the window: mean of the two middle quotients
    x[9:, 0, 40:48] = 1.5             # a quarter: the median ignores it
    flag = np.ones(p.N, np.uint8)
    slow, _ = oracle.severity(p, x, med, flag)
    assert slow[1] == 0.0
    assert slow[2] == np.float32(0.5) and slow[3] == np.float32(0.5)
    assert slow[4] == np.float32(0.25)
    assert slow[5] == 0.0
    # a history shorter than the window uses what there is
    slow, _ = oracle.severity(p, x[8:], med[8:], flag)
    assert slow[4] == np.float32(0.5) and slow[5] == np.float32(0.25)


def test_the_other_metrics_and_other_nodes_do_not_matter():
    p = params(M=3, primary=1)
    rng = np.random.default_rng(3)
    T = 5
    x = rng.uniform(0.5, 2.0, (T, p.M, p.R)).astype(np.float32)
    med = rng.uniform(0.9, 1.1, (T, p.M)).astype(np.float32)
    flag = np.ones(p.N, np.uint8)
    slow, tier = oracle.severity(p, x, med, flag)
    y = x.copy()
    y[:, 0] = 77.0
    y[:, 2] = 0.01
    y[:, 1, 8:] = rng.uniform(0.5, 2.0, (T, p.R - 8)).astype(np.float32)
    slow2, tier2 = oracle.severity(p, y, med, flag)
    assert slow2[0] == slow[0] and tier2[0] == tier[0]


@pytest.mark.parametrize("direction", [1, -1, 0])
def test_against_exact_rational_arithmetic(direction):
    """Quotient, median (mean of the two middle values, then halved) and the final
    subtraction, each rounded once to fp32, recomputed with fractions."""
    rng = np.random.default_rng(11 + direction)
    p = params(R=16, M=1, W=3, directions=(direction,))
    T = 5
    x = rng.uniform(0.7, 1.6, (T, 1, p.R)).astype(np.float32)
    med = rng.uniform(0.9, 1.2, (T, 1)).astype(np.float32)
    flag = np.ones(p.N, np.uint8)
    slow, tier = oracle.severity(p, x, med, flag, 0.1, 0.2)
    for n in range(p.N):
        q = []
        for t in range(T - 3, T):
            for g in range(8):
                xv, m = x[t, 0, n * 8 + g], med[t, 0]
                if direction > 0:
                    r = div32(xv, m)
                elif direction < 0:
                    r = div32(m, xv)
                else:
                    r = div32(xv, m) if F(xv) >= F(m) else div32(m, xv)
                q.append(r)
        q.sort(key=F)
        mid = mul32(np.float32(0.5), add32(q[11], q[12]))
        want = sub32(mid, np.float32(1.0))
        assert slow[n] == want, (n, slow[n], want)
        assert tier[n] == (3 if F(want) >= F(np.float32(0.2)) else 2 if F(want) >= F(np.float32(0.1)) else 1)


def test_against_numpy_median_of_the_quotients():
    rng = np.random.default_rng(5)
    p = params(R=256, M=2, W=16, primary=1)
    T = 40
    x = np.exp(0.05 * rng.standard_normal((T, p.M, p.R))).astype(np.float32)
    x[:, 1, 64:72] *= np.float32(1.17)
    med = np.median(x, axis=2).astype(np.float32)
    flag = np.ones(p.N, np.uint8)
    slow, tier = oracle.severity(p, x, med, flag)
    for n in range(p.N):
        q = (x[T - 16:, 1, n * 8:(n + 1) * 8] / med[T - 16:, 1][:, None]).astype(np.float32).ravel()
        want = np.float32(np.median(q)) - np.float32(1.0)
        assert slow[n] == np.float32(want), n
    assert tier[8] == 2 and abs(float(slow[8]) - 0.17) < 0.02


def test_power_of_two_rescaling_changes_nothing():
    rng = np.random.default_rng(9)
    p = params(R=64, M=1, W=8, directions=(-1,))
    T = 8
    x = rng.uniform(0.5, 2.0, (T, 1, p.R)).astype(np.float32)
    med = np.median(x, axis=2).astype(np.float32)
    flag = np.ones(p.N, np.uint8)
    a = oracle.severity(p, x, med, flag)
    b = oracle.severity(p, x * np.float32(2.0 ** 20), med * np.float32(2.0 ** 20), flag)
    c = oracle.severity(p, x * np.float32(2.0 ** -30), med * np.float32(2.0 ** -30), flag)
    for u in (b, c):
        assert np.array_equal(a[0], u[0]) and np.array_equal(a[1], u[1])


def test_lower_is_worse_and_two_sided_quotients():
    T = 4
    med = np.full((T, 1), 4.0, np.float32)
    flag = np.ones(8, np.uint8)
    x = flat_history(T, 1, 64, 4.0)
    x[:, 0, 0:8] = 3.2          # 4 / 3.2 = 1.25: a throughput-like metric 20% below its peers
    x[:, 0, 8:16] = 5.0         # 4 / 5 = 0.8: better than its peers
    lo, _ = oracle.severity(params(M=1, directions=(-1,)), x, med, flag)
    assert lo[0] == sub32(div32(np.float32(4.0), np.float32(3.2)), np.float32(1.0))
    assert lo[1] == sub32(div32(np.float32(4.0), np.float32(5.0)), np.float32(1.0)) and lo[1] < 0
    both, _ = oracle.severity(params(M=1, directions=(0,)), x, med, flag)
    assert both[0] == lo[0]
    assert both[1] == np.float32(0.25)


def test_negative_zero_reads_as_zero_and_empty_history():
    p = params(M=1, directions=(0,))
    x = flat_history(2, 1, 64, 1.0)
    x[:, 0, 0:8] = -0.0
    med = np.ones((2, 1), np.float32)
    flag = np.ones(p.N, np.uint8)
    slow, _ = oracle.severity(p, x, med, flag)
    assert np.isinf(slow[0]) and slow[0] > 0          # 1 / +0, not 1 / -0
    slow, tier = oracle.severity(p, x[:0], med[:0], flag)
    assert not slow.any() and not tier.any()


def test_missing_samples_are_left_out_of_the_quotients():
    p = params(W=4)
    T = 4
    x = flat_history(T, p.M, p.R, 1.0)
    med = np.ones((T, p.M), np.float32)
    nan = np.float32("nan")
    x[:, 0, 8:16] = 1.5
    x[1:, 0, 8:13] = nan            # node 1: 8 + 3*3 = 17 quotients left (odd), all 1.5
    x[:, 0, 16:24] = [1.0, 1.1, 1.2, 1.3, 1.4, nan, nan, nan]     # node 2: 5 per step, 20 in all
    x[:, 0, 24:32] = nan            # node 3: nothing arrived
    med[0, 0] = nan                 # and a step without a median counts for nobody
    flag = np.ones(p.N, np.uint8)
    slow, tier = oracle.severity(p, x, med, flag)
    assert slow[1] == np.float32(0.5) and tier[1] == 3
    q = np.sort(np.tile(np.array([1.0, 1.1, 1.2, 1.3, 1.4], np.float32), 3))     # 3 steps count
    assert slow[2] == np.float32(np.median(q)) - np.float32(1.0)
    assert slow[3] == 0.0 and tier[3] == 1
    assert slow[0] == 0.0 and tier[0] == 1
