"""Pins of the oracle's rule for missing samples (NaN = the sample did not arrive;
telemetry polled every 30-60 s does not always answer, Section 7.1): numpy's
nanmedian on float32, exact rational arithmetic, the same cluster without the
silent nodes, and the cases in which a missing sample must not count."""
import numpy as np
import pytest

import oracle
from exactfp import F, add32, div32, mul32, sub32

NAN = np.float32("nan")


def params(R=64, M=1, **kw):
    return oracle.Params(R=R, M=M, W=4, k=2, **kw)


@pytest.mark.parametrize("n_missing", [1, 2, 7, 31, 63])
def test_median_and_mad_are_those_of_the_samples_present(n_missing):
    rng = np.random.default_rng(n_missing)
    p = params(R=64, M=2)
    x = np.exp(0.1 * rng.standard_normal((3, 2, 64))).astype(np.float32)
    for t in range(3):
        x[t, 0, rng.choice(64, n_missing, replace=False)] = NAN
    s = oracle.score(p, x, want_z=True)
    for t in range(3):
        col = x[t, 0]
        med = np.nanmedian(col)                       # float32 in, float32 out
        assert med.dtype == np.float32 and s.med[t, 0] == med
        mad = np.nanmedian(np.abs(col - med))
        assert s.mad[t, 0] == mad
        # the other metric of the step, with nothing missing, is what it was
        assert s.med[t, 1] == np.median(x[t, 1])


def test_scores_of_present_ranks_and_zero_for_missing_ones():
    p = params(R=8, M=1, thr=3.5)
    col = np.array([1.00, 1.02, NAN, 1.01, 0.99, NAN, 0.97, 1.15], np.float32)
    s = oracle.score(p, col[None, None, :], want_z=True)
    present = sorted([v for v in col if not np.isnan(v)], key=F)       # 6 values: even count
    med = mul32(np.float32(0.5), add32(present[2], present[3]))
    dev = sorted([abs(sub32(v, med)) for v in present], key=F)
    mad = mul32(np.float32(0.5), add32(dev[2], dev[3]))
    assert s.med[0, 0] == med and s.mad[0, 0] == mad
    scale = mul32(np.float32(1.4826), mad)
    for r, v in enumerate(col):
        want = np.float32(0.0) if np.isnan(v) else div32(sub32(v, med), scale)
        assert s.z[0, 0, r] == want, r
    assert s.exceed_mask[0].tolist() == [0, 0, 0, 0, 0, 0, 0, 1]
    # node score: the missing members add nothing to the pairwise sum
    z = s.z[0, 0]
    total = add32(add32(add32(z[0], z[1]), add32(z[2], z[3])), add32(add32(z[4], z[5]), add32(z[6], z[7])))
    assert s.node_z[0, 0] == mul32(np.float32(p.node_scale), total)


def test_odd_number_present_takes_the_middle_value():
    p = params(R=8, M=1)
    col = np.array([5.0, NAN, 1.0, 3.0, 2.0, 4.0, NAN, NAN], np.float32)       # 5 present
    s = oracle.score(p, col[None, None, :], want_z=False)
    assert s.med[0, 0] == np.float32(3.0) and s.mad[0, 0] == np.float32(1.0)


def test_a_missing_sample_never_exceeds_whatever_the_threshold():
    rng = np.random.default_rng(2)
    x = np.exp(0.05 * rng.standard_normal((2, 2, 64))).astype(np.float32)
    x[:, :, 5] = NAN
    x[0, 1, 17] = NAN
    for thr in (-2.0, 0.0, 3.5):
        for d in (1, -1, 0):
            p = params(R=64, M=2, thr=thr, directions=(d, d), min_signals=1)
            s = oracle.score(p, x, want_z=True)
            assert not s.exceed_mask[:, 5].any() and not (s.exceed_mask[0, 17] & 2)
            assert not (s.rank_anom[:, 0] >> np.uint64(5) & np.uint64(1)).any()
            assert (s.z[:, :, 5] == 0).all() and s.z[0, 1, 17] == 0


def test_a_column_with_nothing_present():
    p = params(R=16, M=2, min_signals=1)
    x = np.ones((1, 2, 16), np.float32)
    x[0, 0] = NAN
    s = oracle.score(p, x, want_z=True)
    assert np.isnan(s.med[0, 0]) and np.isnan(s.mad[0, 0])
    assert not s.exceed_mask.any() and not s.node_mask.any()
    assert (s.z[0, 0] == 0).all() and (s.node_z[0] == 0).all()
    assert s.med[0, 1] == 1.0


@pytest.mark.parametrize("agg", [oracle.NODE_SUM_SCALED, oracle.NODE_MAX])
def test_silent_nodes_leave_the_rest_of_the_cluster_as_if_they_were_not_there(agg):
    """All 8 GPUs of some nodes missing: medians, MADs, scores and node scores of
    the others equal those of the cluster without these nodes."""
    rng = np.random.default_rng(7)
    R, M, T = 128, 3, 4
    x = np.exp(0.05 * rng.standard_normal((T, M, R))).astype(np.float32)
    x[:, :, 40:48] *= np.float32(1.3)
    silent = [2, 9, 10]
    keep = np.array([r for r in range(R) if r // 8 not in silent])
    y = x.copy()
    for n in silent:
        y[:, :, n * 8:(n + 1) * 8] = NAN
    kw = dict(M=M, node_agg=agg, directions=(1, -1, 0), min_signals=1)
    a = oracle.score(params(R=R, **kw), y, want_z=True)
    b = oracle.score(params(R=R - 8 * len(silent), **kw), np.ascontiguousarray(x[:, :, keep]), want_z=True)
    assert np.array_equal(a.med.view(np.uint32), b.med.view(np.uint32))
    assert np.array_equal(a.mad.view(np.uint32), b.mad.view(np.uint32))
    assert np.array_equal(a.z[:, :, keep].view(np.uint32), b.z.view(np.uint32))
    assert np.array_equal(a.exceed_mask[:, keep], b.exceed_mask)
    kept_nodes = [n for n in range(R // 8) if n not in silent]
    assert np.array_equal(a.node_z[:, kept_nodes].view(np.uint32), b.node_z.view(np.uint32))
    assert np.array_equal(a.node_mask[:, kept_nodes], b.node_mask)
    assert not a.node_mask[:, silent].any() and (a.node_z[:, silent] == 0).all()


def test_nothing_missing_is_the_old_behaviour():
    rng = np.random.default_rng(4)
    x = np.exp(0.05 * rng.standard_normal((3, 2, 64))).astype(np.float32)
    s = oracle.score(params(R=64, M=2), x, want_z=True)
    for t in range(3):
        for m in range(2):
            assert s.med[t, m] == np.median(x[t, m])
            assert s.mad[t, m] == np.median(np.abs(x[t, m] - s.med[t, m]))


def test_membership_mask_turns_absent_ranks_into_missing_samples():
    """Against numpy: unpack the bit words, put NaN where the bit is clear; and scoring the
    masked tensor is scoring the cluster without the absent nodes."""
    rng = np.random.default_rng(12)
    T, M, R = 5, 3, 136
    x = np.exp(0.05 * rng.standard_normal((T, M, R))).astype(np.float32)
    bits = rng.random((T, R)) < 0.8
    bits[1] = True                      # a step with everybody
    bits[3] = False                     # a step with nobody
    padded = np.zeros((T, 192), np.uint8)
    padded[:, :R] = bits
    words = np.packbits(padded.reshape(T, 3, 64), axis=2, bitorder="little").view(np.uint64).reshape(T, 3)
    y = oracle.apply_membership(x, words)
    want = np.where(bits[:, None, :], x, np.float32("nan"))
    assert np.array_equal(y.view(np.uint32) == 0x7FC00000, ~np.broadcast_to(bits[:, None, :], x.shape))
    assert np.array_equal(np.isnan(y), np.isnan(want)) and np.array_equal(y[~np.isnan(y)], want[~np.isnan(want)])
    assert not np.isnan(x).any()        # the input is left alone
    # whole nodes absent from every step: the others score as a smaller cluster
    absent = [3, 11]
    act = np.ones((T, R), bool)
    for n in absent:
        act[:, 8 * n:8 * n + 8] = False
    padded[:, :R] = act
    words = np.packbits(padded.reshape(T, 3, 64), axis=2, bitorder="little").view(np.uint64).reshape(T, 3)
    keep = np.array([r for r in range(R) if r // 8 not in absent])
    a = oracle.score(params(R=R, M=M, directions=(1, 1, 1)), oracle.apply_membership(x, words), want_z=False)
    b = oracle.score(params(R=R - 16, M=M, directions=(1, 1, 1)), np.ascontiguousarray(x[:, :, keep]), want_z=False)
    assert np.array_equal(a.med.view(np.uint32), b.med.view(np.uint32))
    assert np.array_equal(a.exceed_mask[:, keep], b.exceed_mask)
