"""Pins for the oracle's scoring (median, MAD, robust z, masks, node scores).

None of these re-type the oracle: they use the counting definition of a
median, exact rational arithmetic with explicit fp32 rounding, numpy's own
median, closed forms, and invariances.
"""
import itertools
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from exactfp import F, add32, div32, mul32, rn32, sub32

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def P(R, M=1, **kw):
    kw.setdefault("W", 4)
    kw.setdefault("k", 2)
    return oracle.Params(R=R, M=M, **kw)


def counting_median(vals):
    """Median from the counting definition, exact: an order statistic v is the
    j-th smallest (0-based) iff #less <= j < #less + #equal."""
    vals = [Fraction(float(v)) for v in vals]
    n = len(vals)

    def stat(j):
        for v in vals:
            less = sum(1 for u in vals if u < v)
            eq = sum(1 for u in vals if u == v)
            if less <= j < less + eq:
                return v
        raise AssertionError

    if n % 2:
        return rn32(stat(n // 2))
    return mul32(np.float32(0.5), rn32(stat(n // 2 - 1) + stat(n // 2)))


def exact_chain(col, thr=3.5, rel_floor=1e-6, abs_floor=1e-30, dirn=1):
    """med, mad, z', exceed via the counting definition + exact fp32 roundings."""
    col = [np.float32(0.0) if v == 0 else np.float32(v) for v in col]
    md = counting_median(col)
    dev = [np.float32(abs(sub32(v, md))) for v in col]
    ma = counting_median(dev)
    s = mul32(np.float32(1.4826), ma)
    s = max(s, mul32(np.float32(rel_floor), np.float32(abs(md))), np.float32(abs_floor))
    z = [div32(sub32(v, md), s) for v in col]
    zs = [zz if dirn > 0 else (np.float32(-zz) if dirn < 0 else np.float32(abs(zz))) for zz in z]
    e = [bool(F(v) > Fraction(float(np.float32(thr)))) for v in zs]
    return md, ma, z, zs, e


def golden_rows():
    rows = {}
    with open(os.path.join(GOLD, "closed_forms.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                name, *vals = line.split()
                rows[name] = vals
    return rows


def bits(a):
    return np.asarray(a, np.float32).view(np.uint32)


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("R", [8, 16])
def test_tiny_columns_against_counting_definition(R):
    rng = np.random.default_rng(R)
    pools = [
        rng.normal(1.0, 0.02, 64).astype(np.float32),
        np.array([0.0, -0.0, 1.0, -1.0, 2.5, -2.5, 1.0, 1.0, 3.0], np.float32),
        rng.integers(-3, 4, 64).astype(np.float32),
    ]
    T = 40
    x = np.empty((T, 1, R), np.float32)
    for t in range(T):
        x[t, 0] = rng.choice(pools[t % 3], R)
    s = oracle.score(P(R), x)
    for t in range(T):
        md, ma, z, zs, e = exact_chain(x[t, 0])
        assert bits(s.med[t, 0]) == bits(md)
        assert bits(s.mad[t, 0]) == bits(ma)
        assert np.array_equal(bits(s.z[t, 0]), bits(z))
        assert np.array_equal((s.exceed_mask[t] & 1).astype(bool), np.array(e))


def test_median_is_permutation_invariant_exhaustively():
    base = np.array([1.0, 1.02, 0.98, 1.02, -0.5, 0.0, -0.0, 7.0], np.float32)
    perms = list(itertools.permutations(range(8)))[::97]
    x = np.stack([base[list(p)] for p in perms])[:, None, :]
    s = oracle.score(P(8), x)
    md, ma, *_ = exact_chain(base)
    assert np.all(bits(s.med) == bits(md)) and np.all(bits(s.mad) == bits(ma))


def test_odd_count_uses_middle_value():
    # the product needs R % 8 == 0; the oracle's median rule is pinned for odd counts too
    col = np.array([4, 100, 1, 3, 2], np.float32)
    assert oracle.median(col) == 3
    assert oracle.median(np.abs(col - 3)) == 1
    rng = np.random.default_rng(0)
    for n in (1, 3, 7, 9, 101):
        v = rng.standard_normal(n).astype(np.float32)
        assert bits(oracle.median(v)) == bits(counting_median(v)) == bits(np.median(v))
    md, ma, z, _, _ = exact_chain(col)
    want = np.array([int(h, 16) for h in golden_rows()["odd5_z"]], np.uint32)
    assert np.array_equal(np.sort(bits(z)), np.sort(want))


# ---------------------------------------------------------------- numpy.median
@pytest.mark.parametrize("R", [8, 64, 1024, 4096])
def test_median_and_mad_equal_numpy(R):
    rng = np.random.default_rng(R + 1)
    x = np.exp(0.02 * rng.standard_t(3, (6, 3, R))).astype(np.float32)
    x[1] *= -1.0
    x[2, :, : R // 2] = 1.0   # massive ties
    s = oracle.score(P(R, 3), x)
    med = np.median(x, axis=2)
    assert med.dtype == np.float32
    assert np.array_equal(bits(s.med), bits(med))
    mad = np.median(np.abs(x - med[:, :, None]), axis=2)
    assert np.array_equal(bits(s.mad), bits(mad))


# ---------------------------------------------------------------- closed forms


def test_ramp_closed_form():
    g = golden_rows()
    for R, name in ((64, "ramp64"), (8, "ramp8")):
        x = np.arange(R, dtype=np.float32)[None, None, :]
        s = oracle.score(P(R), x)
        # median of 0..R-1 is (R-1)/2, MAD is R/4 (deviations 0.5,0.5,1.5,1.5,...)
        assert s.med[0, 0] == (R - 1) / 2 and s.mad[0, 0] == R / 4
        zlast = div32(np.float32((R - 1) / 2), mul32(np.float32(1.4826), np.float32(R / 4)))
        assert bits(s.z[0, 0, R - 1]) == bits(zlast) == int(g[name + "_zlast"][0], 16)
        assert bits(s.z[0, 0, 0]) == bits(np.float32(-zlast))  # antisymmetric ramp


def test_worked_eight_rank_column():
    g = golden_rows()
    col = np.array([1.00, 1.02, 0.98, 1.01, 0.99, 1.03, 0.97, 1.15], np.float32)
    s = oracle.score(P(8), col[None, None, :])
    assert bits(s.med[0, 0]) == int(g["worked8_med"][0], 16)
    assert bits(s.mad[0, 0]) == int(g["worked8_mad"][0], 16)
    assert bits(s.z[0, 0, 7]) == int(g["worked8_z7"][0], 16)
    assert s.exceed_mask[0].tolist() == [0, 0, 0, 0, 0, 0, 0, 1]
    assert abs(float(s.z[0, 0, 7]) - 4.8900619) < 1e-6
    assert np.sort(s.z[0, 0])[-2] < 0.85


# ---------------------------------------------------------------- invariances
def test_power_of_two_rescale_is_exact():
    rng = np.random.default_rng(5)
    x = np.exp(0.02 * rng.standard_normal((10, 2, 256))).astype(np.float32)
    x[:, :, 17] *= 1.2
    p = P(256, 2, rel_floor=1e-6, abs_floor=1e-37)
    a = oracle.score(p, x)
    for j in (-20, -3, 5, 40):
        b = oracle.score(p, x * np.float32(2.0 ** j))
        assert np.array_equal(bits(b.med), bits(a.med * np.float32(2.0 ** j)))
        assert np.array_equal(bits(b.mad), bits(a.mad * np.float32(2.0 ** j)))
        assert np.array_equal(bits(b.z), bits(a.z))
        assert np.array_equal(b.exceed_mask, a.exceed_mask)
        assert np.array_equal(b.node_mask, a.node_mask)
        assert np.array_equal(bits(b.node_z), bits(a.node_z))


def test_affine_rescale_keeps_scores_and_negation_flips_them():
    rng = np.random.default_rng(6)
    x = np.exp(0.02 * rng.standard_normal((8, 1, 512))).astype(np.float32)
    p = P(512)
    a = oracle.score(p, x)
    y = (np.float64(x) * 3.0 + 10.0).astype(np.float32)
    b = oracle.score(p, y)
    assert np.allclose(b.z, a.z, rtol=0, atol=2e-4)   # rounding of 3x+10 costs ~1e-6/0.03
    c = oracle.score(p, -x)
    assert np.array_equal(bits(c.med), bits(-a.med))
    assert np.array_equal(bits(c.mad), bits(a.mad))
    assert np.array_equal(bits(c.z), bits(-a.z))


def test_rank_permutation():
    rng = np.random.default_rng(7)
    R = 128
    x = np.exp(0.02 * rng.standard_normal((12, 3, R))).astype(np.float32)
    x[:, :, 40:48] *= 1.08
    p = P(R, 3, directions=(1, -1, 0))
    a = oracle.score(p, x, want_node_all=True)
    perm = rng.permutation(R)
    b = oracle.score(p, x[:, :, perm])
    assert np.array_equal(bits(b.med), bits(a.med)) and np.array_equal(bits(b.mad), bits(a.mad))
    assert np.array_equal(bits(b.z), bits(a.z[:, :, perm]))
    assert np.array_equal(b.exceed_mask, a.exceed_mask[:, perm])
    # moving whole nodes permutes the node outputs bit for bit
    nperm = rng.permutation(R // 8)
    rp = (nperm[:, None] * 8 + np.arange(8)[None, :]).ravel()
    c = oracle.score(p, x[:, :, rp], want_node_all=True)
    assert np.array_equal(bits(c.node_z_all), bits(a.node_z_all[:, :, nperm]))
    assert np.array_equal(c.node_mask, a.node_mask[:, nperm])


def test_noise_free_column_scores_zero():
    x = np.full((5, 2, 64), 1.25, np.float32)
    s = oracle.score(P(64, 2), x)
    assert np.all(s.mad == 0) and np.all(s.med == 1.25)
    assert np.all(bits(s.z) == 0) and not s.exceed_mask.any() and not s.rank_anom.any()
    assert not s.node_mask.any() and not s.node_anom.any()


def test_lone_outlier_on_identical_data_is_finite_and_flagged():
    x = np.ones((1, 1, 64), np.float32)
    x[0, 0, 9] = 1.5
    s = oracle.score(P(64, 1, min_signals=1), x)
    assert s.mad[0, 0] == 0
    # scale falls to rel_floor*|med| = 1e-6
    want = div32(np.float32(0.5), np.float32(1e-6))
    assert bits(s.z[0, 0, 9]) == bits(want) and np.isfinite(s.z).all()
    assert s.exceed_mask[0, 9] == 1 and s.exceed_mask[0].sum() == 1
    assert s.rank_anom[0, 0] == np.uint64(1 << 9)


def test_negative_zero_reads_as_positive_zero():
    x = np.array([-0.0, 0.0, -0.0, 0.0, -1.0, 1.0, -0.0, -0.0], np.float32)[None, None, :]
    s = oracle.score(P(8), x)
    assert bits(s.med[0, 0]) == 0 and bits(s.mad[0, 0]) == 0


# ---------------------------------------------------------------- direction, combine
def test_direction_and_strict_threshold():
    R = 64
    base = np.arange(R, dtype=np.float32)          # med 31.5, mad 16, s = fl(1.4826*16)
    s_ = mul32(np.float32(1.4826), np.float32(16))
    x = np.stack([base, base, base])[None]          # three identical metrics
    p = P(R, 3, directions=(1, -1, 0), min_signals=1, thr=float(div32(np.float32(20.5), s_)))
    s = oracle.score(p, x)
    z = s.z[0, 0]
    thr = np.float32(p.thr)
    # strict '>' : rank 52 has z == thr exactly and must not exceed
    assert z[52] == thr
    e0 = z > thr
    e1 = -z > thr
    e2 = np.abs(z) > thr
    want = e0.astype(np.uint8) | (e1.astype(np.uint8) << 1) | (e2.astype(np.uint8) << 2)
    assert np.array_equal(s.exceed_mask[0], want)
    assert want[53] == 0b101 and want[52] == 0 and want[10] == 0b110 and want[11] == 0
    assert s.near_rank >= 3


def test_multi_signal_rule_needs_primary_and_count():
    R, M = 64, 4
    rng = np.random.default_rng(11)
    x = (1.0 + 0.01 * rng.standard_normal((1, M, R))).astype(np.float32)
    x[0, 0, 3] = 2.0                       # primary only
    x[0, 1, 4] = 2.0; x[0, 2, 4] = 2.0      # two supporting metrics, no primary
    x[0, 0, 5] = 2.0; x[0, 3, 5] = 2.0      # primary + one supporting
    for prim, ms, want in ((0, 2, {5}), (0, 1, {3, 5}), (1, 2, {4}), (0, 3, set())):
        s = oracle.score(P(R, M, primary=prim, min_signals=ms), x)
        got = {r for r in range(R) if (int(s.rank_anom[0, 0]) >> r) & 1}
        assert got == want
        m = s.exceed_mask[0]
        assert m[3] == 1 and m[4] == 0b0110 and m[5] == 0b1001


# ---------------------------------------------------------------- node scores
def test_node_sum_tree_order_and_scale():
    # Choose scores whose fp32 sum depends on the association order, and check
    # the oracle against the one fixed tree ((0+1)+(2+3))+((4+5)+(6+7)) evaluated
    # exactly with explicit roundings.
    R = 64
    rng = np.random.default_rng(3)
    x = np.zeros((1, 1, R), np.float32)
    x[0, 0] = rng.standard_normal(R).astype(np.float32) * np.float32(1e-3)
    x[0, 0, 8:16] = np.array([1e4, 1.0, -1e4, 1.0, 3e-4, 5.0, 7e3, -7e3], np.float32)
    p = P(R, 1, min_signals=1)
    s = oracle.score(p, x, want_node_all=True)
    z = s.z[0, 0]
    sc = np.float32(p.node_scale)
    assert bits(sc) == bits(rn32(Fraction(1) / Fraction(8) ** Fraction(1, 2))) or abs(float(sc) - 8 ** -0.5) < 3e-8
    tree_differs = False
    for n in range(R // 8):
        q = z[8 * n: 8 * n + 8]
        tree = mul32(sc, add32(add32(add32(q[0], q[1]), add32(q[2], q[3])),
                               add32(add32(q[4], q[5]), add32(q[6], q[7]))))
        assert bits(s.node_z[0, n]) == bits(tree)
        seq = q[0]
        for v in q[1:]:
            seq = add32(seq, v)
        tree_differs |= bits(mul32(sc, seq)) != bits(tree)
        assert bool(s.node_mask[0, n] & 1) == bool(F(tree) > F(np.float32(p.thr)))
    assert tree_differs, "test data must distinguish the tree from a sequential sum"


def test_node_scale_value_is_inverse_sqrt8():
    assert bits(np.float32(oracle.Params(R=8, M=1, W=1, k=1).node_scale)) == 0x3EB504F3


def test_node_max_rule_and_whole_node_sensitivity():
    R = 1024
    rng = np.random.default_rng(21)
    x = np.exp(0.02 * rng.standard_normal((4, 2, R))).astype(np.float32)
    x[:, :, 80:88] *= np.float32(1.05)       # whole node 10 slowed by 5% (2.5 sigma per GPU)
    p = P(R, 2)
    s = oracle.score(p, x, want_node_all=True)
    # no single GPU of that node needs to exceed, but the scaled sum does (2.5*sqrt(8) ~ 7)
    assert all(s.node_anom[t, 0] & np.uint64(1 << 10) for t in range(4))
    assert (s.node_z[:, 10] > 5).all()
    pm = P(R, 2, node_agg=oracle.NODE_MAX)
    sm = oracle.score(pm, x, want_node_all=True)
    zs = s.z   # directions +1: z' = z
    want = zs.reshape(4, 2, R // 8, 8).max(axis=3)
    assert np.array_equal(bits(sm.node_z_all), bits(want))


def test_node_max_of_zeros_of_both_signs_is_plus_zero():
    """Ranks that sit exactly on the median score +0, or -0 when the metric is
    lower-is-worse; the largest of such zeros is reported as +0 whatever their order,
    while the scaled sum keeps the sign that IEEE addition gives it."""
    R = 32
    x = np.full((1, 3, R), 2.0, np.float32)
    x[0, :, 8:16] = [2.0, 2.0, 3.0, 2.0, 1.0, 2.0, 2.0, 2.0]       # node 1: some ranks off the median
    x[0, :, 16:24] = [1.0, 1.5, 1.0, 1.0, 1.0, 1.0, 1.0, 1.0]      # node 2: all below the median
    for dirs in ((1, -1, 0), (-1, 1, 0)):
        pm = P(R, 3, node_agg=oracle.NODE_MAX, directions=dirs, min_signals=1)
        sm = oracle.score(pm, x, want_node_all=True, want_z=True)
        assert (sm.med == 2.0).all() and (sm.mad == 0.0).all()
        for m, d in enumerate(dirs):
            nz = sm.node_z_all[0, m]
            assert bits(nz[0]) == 0 and bits(nz[3]) == 0          # all eight on the median: +0, never -0
            zp = sm.z[0, m] if d > 0 else (-sm.z[0, m] if d < 0 else np.abs(sm.z[0, m]))
            assert nz[1] == zp[8:16].max() and nz[2] == zp[16:24].max()
        ps = P(R, 3, directions=dirs, min_signals=1)
        ss = oracle.score(ps, x, want_node_all=True)
        for m, d in enumerate(dirs):
            assert bits(ss.node_z_all[0, m, 0]) == (0x80000000 if d < 0 else 0)


def test_signed_scores_feed_the_node_sum():
    # a lower-is-worse metric: the node score uses -z, so a node whose GPUs all
    # run low gets a positive node score
    R = 64
    rng = np.random.default_rng(4)
    x = (400.0 * np.exp(0.02 * rng.standard_normal((1, 1, R)))).astype(np.float32)
    x[0, 0, 16:24] *= np.float32(0.9)
    s = oracle.score(P(R, 1, directions=(-1,), min_signals=1), x)
    assert s.node_z[0, 2] > 3.5 and (s.node_mask[0] == np.eye(8, dtype=np.uint8)[2]).all()


# ---------------------------------------------------------------- statistics (soft)
def test_scale_estimates_sigma_on_clean_lognormal_and_student():
    rng = np.random.default_rng(8)
    R = 65536
    x = np.exp(0.02 * rng.standard_normal((1, 1, R))).astype(np.float32)
    s = oracle.score(P(R, 1, min_signals=1), x)
    assert abs(1.4826 * s.mad[0, 0] / (0.02 * s.med[0, 0]) - 1) < 0.03
    rate = np.count_nonzero(s.exceed_mask) / R
    assert 0.5e-4 < rate < 6e-4            # normal upper tail at 3.5 is 2.3e-4
    x = np.exp(0.02 * rng.standard_t(3, (1, 1, R))).astype(np.float32)
    s = oracle.score(P(R, 1, min_signals=1), x)
    assert abs(1.4826 * s.mad[0, 0] / 0.02 - 1.134) < 0.04
    rate = np.count_nonzero(s.exceed_mask) / R
    assert 0.008 < rate < 0.022            # t(3) tail beyond 3.5*1.134 is ~1.4e-2
