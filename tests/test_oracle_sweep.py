"""Pins of the oracle's single-node sweep scoring (Section 5: consistent sustained
throughput across a node's GPUs; connectivity and symmetry of the pairwise
bandwidth): exact rational arithmetic, numpy's medians, and nodes built with a
known throttled GPU or a known degraded link."""
import numpy as np

import oracle
from exactfp import F, add32, div32, mul32, sub32

PAIRS = [(i, j) for i in range(8) for j in range(i + 1, 8)]


def healthy(B, rng=None, flops=400.0, bw=300.0, noise=0.0):
    f = np.full((B, 8), flops, np.float32)
    w = np.full((B, 8, 8), bw, np.float32)
    if rng is not None and noise:
        f *= np.exp(noise * rng.standard_normal(f.shape)).astype(np.float32)
        w *= np.exp(noise * rng.standard_normal(w.shape)).astype(np.float32)
    return f, w


def test_healthy_nodes_pass_and_the_diagonal_is_ignored():
    f, w = healthy(5)
    for b in range(5):
        np.fill_diagonal(w[b], 0.0 if b % 2 else 1e9)
    sf, gm, lm, vd = oracle.sweep(f, w)
    assert not sf.any() and not gm.any() and not lm.any() and not vd.any()


def test_a_throttled_gpu_and_a_degraded_link_are_named():
    f, w = healthy(4)
    f[1, 5] = 300.0                       # 25 % below its peers
    f[2, 0] = 384.0                       # 4 %: inside the tolerance
    w[3, 2, 6] = 150.0                    # one direction of the link 2-6 at half rate
    w[0, 4, 7] = w[0, 7, 4] = 240.0       # a link degraded in both directions: 20 % below the rest
    sf, gm, lm, vd = oracle.sweep(f, w, tol_compute=0.05, tol_sym=0.10, tol_bw=0.15)
    assert gm.tolist() == [0, 1 << 5, 0, 0]
    assert sf[1, 5] == np.float32(0.25) and sf[2, 0] == div32(np.float32(16.0), np.float32(400.0))
    assert lm[3] == 1 << PAIRS.index((2, 6)) and lm[0] == 1 << PAIRS.index((4, 7))
    assert lm[1] == 0 and lm[2] == 0
    assert vd.tolist() == [2, 1, 0, 2]
    # the symmetric slow link is caught by the bandwidth rule alone, the one-way one by both
    _, _, lm2, _ = oracle.sweep(f, w, tol_compute=0.05, tol_sym=0.10, tol_bw=0.9)
    assert lm2[0] == 0 and lm2[3] == 1 << PAIRS.index((2, 6))
    _, _, lm3, _ = oracle.sweep(f, w, tol_compute=0.05, tol_sym=0.9, tol_bw=0.15)
    assert lm3[0] == 1 << PAIRS.index((4, 7)) and lm3[3] == 1 << PAIRS.index((2, 6))


def test_against_exact_rational_arithmetic_and_numpy_medians():
    rng = np.random.default_rng(1)
    f, w = healthy(6, rng, noise=0.08)
    tc, ts, tb = 0.05, 0.10, 0.07
    sf, gm, lm, vd = oracle.sweep(f, w, tc, ts, tb)
    for b in range(6):
        m8 = np.median(f[b])
        assert m8.dtype == np.float32
        off = np.array([w[b, i, j] for i in range(8) for j in range(8) if i != j], np.float32)
        m56 = np.median(off)
        want_g = 0
        for g in range(8):
            s = div32(sub32(m8, f[b, g]), m8)
            assert sf[b, g] == s
            if F(s) > F(np.float32(tc)):
                want_g |= 1 << g
        want_l = 0
        for p, (i, j) in enumerate(PAIRS):
            hi, lo = max(w[b, i, j], w[b, j, i]), min(w[b, i, j], w[b, j, i])
            asym = div32(sub32(hi, lo), hi)
            short = div32(sub32(m56, lo), m56)
            if F(asym) > F(np.float32(ts)) or F(short) > F(np.float32(tb)):
                want_l |= 1 << p
        assert gm[b] == want_g and lm[b] == want_l
        assert vd[b] == (1 if want_g else 0) | (2 if want_l else 0)


def test_rescaling_and_relabelling():
    rng = np.random.default_rng(2)
    f, w = healthy(3, rng, noise=0.1)
    a = oracle.sweep(f, w)
    b = oracle.sweep(f * np.float32(2.0 ** 12), w * np.float32(2.0 ** -9))
    for u, v in zip(a, b):
        assert np.array_equal(u, v)
    # relabel the GPUs: shortfalls and mask bits move with them
    perm = np.array([3, 0, 7, 1, 6, 2, 5, 4])
    c = oracle.sweep(f[:, perm], w[:, perm][:, :, perm])
    assert np.array_equal(c[0], a[0][:, perm])
    for bnode in range(3):
        assert c[1][bnode] == sum(((int(a[1][bnode]) >> int(perm[g])) & 1) << g for g in range(8))
        want = 0
        for p, (i, j) in enumerate(PAIRS):
            oi, oj = sorted((int(perm[i]), int(perm[j])))
            want |= ((int(a[2][bnode]) >> PAIRS.index((oi, oj))) & 1) << p
        assert c[2][bnode] == want
    assert np.array_equal(c[3], a[3])
