"""CPU oracle for the straggler detector -- TEST INFRASTRUCTURE, not product.

Thin numpy/ctypes front end of ``guard_oracle.cpp`` (sort-based median and
MAD, explicit loops, fp32 with one rounding per operation).  Only ``tests/``,
the smoke check and the benchmark's CPU-baseline leg may import this package;
the GPU library and its Python binding never do, and nothing here imports
them.

Parity pins (all in ``tests/test_oracle_*.py``): brute-force counting median
on tiny columns, ``numpy.median`` on float32, closed forms on ramps, a worked
8-rank column, power-of-two rescaling, rank permutation, noise-free data,
stragglers injected with a constructed margin, spike immunity, brute-force
top-k; for the severity tiers: exact rational arithmetic on small cases,
``numpy.median`` of the quotients, constructed slowdowns, the window's extent,
both directions, tier boundaries; for missing samples (NaN): ``numpy.nanmedian``,
exact rational arithmetic, and the same cluster without its silent nodes; for
the single-node sweep: exact rational arithmetic, numpy medians, constructed
throttling and asymmetry; for the ledger (persistence per indicator, windowed
score sums and their ranking, recurrence): the scoring oracle's own anomaly
words for the stand-alone multi-signal rule, sliding sums by cumulative sums,
the single-ring persistence where both rules coincide, a history on which they
differ, scores that are whole multiples of the quantisation step, rounding and
saturation cases, Python's sort, hand-built flag timelines.  No function here
is "parity unpinned".
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "guard_oracle.cpp")
_LIB = os.path.join(_HERE, "libguard_oracle.so")
# GUARD_ORACLE_SANITIZE=1 (set by the sanitizer test for its child process, which also
# preloads the sanitizer runtime) selects a build with -fsanitize=address,undefined.
_SANITIZE = os.environ.get("GUARD_ORACLE_SANITIZE", "") == "1"
if _SANITIZE:
    _LIB = os.path.join(_HERE, "libguard_oracle_san.so")


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        opt = ["-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined",
               "-fno-omit-frame-pointer"] if _SANITIZE else ["-O2"]
        cmd = ["g++", "-std=c++17", *opt, "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-fPIC", "-shared", "-Wall", "-Wextra", "-o", _LIB, _SRC]
        subprocess.run(cmd, check=True)
    return _LIB


class _Cfg(ctypes.Structure):
    _fields_ = [("n_ranks", ctypes.c_uint32), ("gpus_per_node", ctypes.c_uint32),
                ("n_metrics", ctypes.c_uint32), ("primary_metric", ctypes.c_uint32),
                ("min_signals", ctypes.c_uint32), ("window", ctypes.c_uint32),
                ("persist_k", ctypes.c_uint32), ("node_agg", ctypes.c_uint32),
                ("z_threshold", ctypes.c_float), ("node_scale", ctypes.c_float),
                ("rel_floor", ctypes.c_float), ("abs_floor", ctypes.c_float),
                ("direction", ctypes.c_int8 * 8)]


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = ctypes.CDLL(_LIB)
        vp = ctypes.c_void_p
        _lib.go_score.argtypes = [ctypes.POINTER(_Cfg), vp, ctypes.c_uint64] + [vp] * 10
        _lib.go_score.restype = None
        _lib.go_num_threads.argtypes = []
        _lib.go_num_threads.restype = ctypes.c_int
        _lib.go_set_threads.argtypes = [ctypes.c_int]
        _lib.go_set_threads.restype = None
        _lib.go_median.argtypes = [vp, ctypes.c_uint64]
        _lib.go_median.restype = ctypes.c_float
        _lib.go_window.argtypes = [ctypes.c_uint32, vp, ctypes.c_uint64, ctypes.c_uint32,
                                   ctypes.c_uint32, vp, vp, vp, vp]
        _lib.go_window.restype = None
        _lib.go_node_flag_byte.argtypes = [ctypes.c_uint32, ctypes.c_uint32, vp, vp, vp]
        _lib.go_node_flag_byte.restype = None
        _lib.go_topk.argtypes = [ctypes.c_uint32, vp, vp, ctypes.c_uint32, vp, vp]
        _lib.go_topk.restype = None
        _lib.go_sweep.argtypes = [ctypes.c_uint32, vp, vp, ctypes.c_float, ctypes.c_float,
                                  ctypes.c_float, vp, vp, vp, vp]
        _lib.go_sweep.restype = None
        _lib.go_severity.argtypes = [ctypes.POINTER(_Cfg), vp, ctypes.c_uint64, vp, vp,
                                     ctypes.c_float, ctypes.c_float, vp, vp]
        _lib.go_severity.restype = None
        u32, u64 = ctypes.c_uint32, ctypes.c_uint64
        _lib.go_apply_membership.argtypes = [vp, u64, u32, u32, vp]
        _lib.go_apply_membership.restype = None
        _lib.go_combine.argtypes = [u32, u32, u32, vp, u64, vp]
        _lib.go_combine.restype = None
        _lib.go_metric_window.argtypes = [u32, u32, u32, vp, u64, u32, u32, vp, vp, vp, vp]
        _lib.go_metric_window.restype = None
        _lib.go_score_ring.argtypes = [u32, vp, u64, u32, ctypes.c_float, vp]
        _lib.go_score_ring.restype = None
        _lib.go_topk_mean.argtypes = [u32, vp, vp, u32, vp, vp]
        _lib.go_topk_mean.restype = None
        _lib.go_recurrence.argtypes = [u32, vp, u64, u64, u32, vp, vp]
        _lib.go_recurrence.restype = None
    return _lib


NODE_SUM_SCALED = 0
NODE_MAX = 1


@dataclass
class Params:
    """Detector parameters; defaults are the stated readings of Section 4.2."""

    R: int
    M: int
    W: int
    k: int
    G: int = 8
    primary: int = 0
    min_signals: Optional[int] = None          # default min(2, M)
    node_agg: int = NODE_SUM_SCALED
    thr: float = 3.5
    node_scale: Optional[float] = None         # default 1/sqrt(G), rounded to fp32
    rel_floor: float = 1e-6
    abs_floor: float = 1e-30
    directions: Sequence[int] = field(default_factory=lambda: (1,) * 8)

    def __post_init__(self):
        if self.min_signals is None:
            self.min_signals = min(2, self.M)
        if self.node_scale is None:
            self.node_scale = float(np.float32(1.0) / np.sqrt(np.float32(self.G)))

    @property
    def N(self) -> int:
        return self.R // self.G

    def _c(self) -> _Cfg:
        c = _Cfg()
        c.n_ranks, c.gpus_per_node, c.n_metrics = self.R, self.G, self.M
        c.primary_metric, c.min_signals = self.primary, self.min_signals
        c.window, c.persist_k, c.node_agg = self.W, self.k, self.node_agg
        c.z_threshold, c.node_scale = self.thr, self.node_scale
        c.rel_floor, c.abs_floor = self.rel_floor, self.abs_floor
        d = list(self.directions)[: self.M] + [1] * (8 - min(8, self.M))
        for i in range(8):
            c.direction[i] = int(d[i])
        return c


@dataclass
class Scores:
    med: np.ndarray          # [T][M] f32
    mad: np.ndarray          # [T][M] f32
    z: Optional[np.ndarray]  # [T][M][R] f32
    exceed_mask: np.ndarray  # [T][R] u8
    rank_anom: np.ndarray    # [T][RW] u64
    node_z: np.ndarray       # [T][N] f32 (primary metric)
    node_mask: np.ndarray    # [T][N] u8
    node_anom: np.ndarray    # [T][NW] u64
    node_z_all: Optional[np.ndarray]  # [T][M][N] f32
    near_rank: int
    near_node: int


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def num_threads() -> int:
    """Threads the oracle's column-parallel loops use."""
    return int(_load().go_num_threads())


def set_threads(n: int) -> None:
    """Threads for the column-parallel loops from now on (timing one core: n = 1)."""
    _load().go_set_threads(int(n))


def median(v: np.ndarray) -> np.float32:
    """The oracle's median rule on one vector of any length >= 1."""
    v = np.ascontiguousarray(v, dtype=np.float32).ravel()
    assert v.size >= 1
    return np.float32(_load().go_median(_ptr(v), v.size))


def score(p: Params, x: np.ndarray, want_z: bool = True, want_node_all: bool = False) -> Scores:
    """Median, MAD, robust z, exceedance masks and node scores of x[t][m][r]."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    T = x.shape[0]
    assert x.shape == (T, p.M, p.R) and p.G == 8 and p.R % p.G == 0
    RW, NW = (p.R + 63) // 64, (p.N + 63) // 64
    o = Scores(
        med=np.empty((T, p.M), np.float32), mad=np.empty((T, p.M), np.float32),
        z=np.empty((T, p.M, p.R), np.float32) if want_z else None,
        exceed_mask=np.empty((T, p.R), np.uint8), rank_anom=np.empty((T, RW), np.uint64),
        node_z=np.empty((T, p.N), np.float32), node_mask=np.empty((T, p.N), np.uint8),
        node_anom=np.empty((T, NW), np.uint64),
        node_z_all=np.empty((T, p.M, p.N), np.float32) if want_node_all else None,
        near_rank=0, near_node=0)
    near = np.zeros(2, np.uint64)
    c = p._c()
    _load().go_score(ctypes.byref(c), _ptr(x), T, _ptr(o.med), _ptr(o.mad), _ptr(o.z),
                     _ptr(o.exceed_mask), _ptr(o.rank_anom), _ptr(o.node_z), _ptr(o.node_mask),
                     _ptr(o.node_anom), _ptr(o.node_z_all), _ptr(near))
    o.near_rank, o.near_node = int(near[0]), int(near[1])
    return o


@dataclass
class Persistence:
    count: np.ndarray   # [n] u16, at the last step
    flag: np.ndarray    # [n] u8, at the last step
    first: np.ndarray   # [n] i32, first flagged step or -1
    count_hist: Optional[np.ndarray]  # [T][n] u16


def window(n: int, anom: np.ndarray, W: int, k: int, want_hist: bool = False) -> Persistence:
    """k-of-W persistence over the whole history anom[T][ceil(n/64)] (from step 0)."""
    anom = np.ascontiguousarray(anom, dtype=np.uint64)
    T = anom.shape[0]
    assert anom.shape == (T, (n + 63) // 64)
    o = Persistence(np.zeros(n, np.uint16), np.zeros(n, np.uint8), np.full(n, -1, np.int32),
                    np.zeros((T, n), np.uint16) if want_hist else None)
    _load().go_window(n, _ptr(anom), T, W, k, _ptr(o.count), _ptr(o.flag), _ptr(o.first),
                      _ptr(o.count_hist))
    return o


def node_flag_byte(G: int, node_flag: np.ndarray, rank_flag: np.ndarray) -> np.ndarray:
    node_flag = np.ascontiguousarray(node_flag, np.uint8)
    rank_flag = np.ascontiguousarray(rank_flag, np.uint8)
    N = node_flag.shape[0]
    assert rank_flag.shape[0] == N * G
    out = np.empty(N, np.uint8)
    _load().go_node_flag_byte(N, G, _ptr(node_flag), _ptr(rank_flag), _ptr(out))
    return out


def topk(node_count: np.ndarray, node_z_last: np.ndarray, k: int):
    """(idx[k] i32, key[k] u64) of the k slowest nodes."""
    node_count = np.ascontiguousarray(node_count, np.uint16)
    node_z_last = np.ascontiguousarray(node_z_last, np.float32)
    N = node_count.shape[0]
    assert node_z_last.shape[0] == N and 0 <= k <= N and N <= 65536
    idx = np.empty(k, np.int32)
    key = np.empty(k, np.uint64)
    _load().go_topk(N, _ptr(node_count), _ptr(node_z_last), k, _ptr(idx), _ptr(key))
    return idx, key


def severity(p: Params, x: np.ndarray, med: np.ndarray, node_flag_byte: np.ndarray,
             moderate: float = 0.10, severe: float = 0.20):
    """(slowdown[N] f32, tier[N] u8) of the flagged nodes over the last min(T, W) steps of x."""
    x = np.ascontiguousarray(x, np.float32)
    T, M, R = x.shape
    assert (M, R) == (p.M, p.R)
    med = np.ascontiguousarray(med, np.float32)
    assert med.shape == (T, M)
    nfb = np.ascontiguousarray(node_flag_byte, np.uint8)
    assert nfb.shape == (p.N,)
    slow = np.empty(p.N, np.float32)
    tier = np.empty(p.N, np.uint8)
    c = p._c()
    _load().go_severity(ctypes.byref(c), _ptr(x), T, _ptr(med), _ptr(nfb), moderate, severe,
                        _ptr(slow), _ptr(tier))
    return slow, tier


def sweep(flops: np.ndarray, bw: np.ndarray, tol_compute: float = 0.05, tol_sym: float = 0.10,
          tol_bw: float = 0.15):
    """Single-node sweep scoring of B nodes: flops[B][8], bw[B][8][8] ->
    (shortfall[B][8] f32, gpu_mask[B] u8, link_mask[B] u32, verdict[B] u8)."""
    flops = np.ascontiguousarray(flops, np.float32)
    bw = np.ascontiguousarray(bw, np.float32)
    B = flops.shape[0]
    assert flops.shape == (B, 8) and bw.shape == (B, 8, 8)
    sf = np.empty((B, 8), np.float32)
    gm = np.empty(B, np.uint8)
    lm = np.empty(B, np.uint32)
    vd = np.empty(B, np.uint8)
    _load().go_sweep(B, _ptr(flops), _ptr(bw), tol_compute, tol_sym, tol_bw, _ptr(sf), _ptr(gm),
                     _ptr(lm), _ptr(vd))
    return sf, gm, lm, vd


@dataclass
class MetricPersistence:
    count: np.ndarray   # [8][n] u16 per-metric window counts at the last step
    pmask: np.ndarray   # [n] u8, bit m = metric m persistent at the last step
    flag: np.ndarray    # [n] u8 at the last step
    first: np.ndarray   # [n] i32 first flagged step or -1


def apply_membership(x: np.ndarray, active: np.ndarray) -> np.ndarray:
    """A copy of x[T][M][R] with NaN wherever active[T][ceil(R/64)] (u64 bit words) says the
    rank does not take part in the step."""
    x = np.array(x, dtype=np.float32, order="C", copy=True)
    T, M, R = x.shape
    active = np.ascontiguousarray(active, np.uint64)
    assert active.shape == (T, (R + 63) // 64)
    _load().go_apply_membership(_ptr(x), T, M, R, _ptr(active))
    return x


def combine(mask: np.ndarray, primary: int, min_signals: int) -> np.ndarray:
    """Anomaly words [T][ceil(n/64)] u64 of the per-step multi-signal rule on exceed bytes mask[T][n]."""
    mask = np.ascontiguousarray(mask, np.uint8)
    T, n = mask.shape
    out = np.zeros((T, (n + 63) // 64), np.uint64)
    _load().go_combine(n, primary, min_signals, _ptr(mask), T, _ptr(out))
    return out


def metric_window(mask: np.ndarray, primary: int, min_signals: int, W: int, k: int) -> MetricPersistence:
    """Per-metric k-of-W persistence over the whole history of exceed bytes mask[T][n]."""
    mask = np.ascontiguousarray(mask, np.uint8)
    T, n = mask.shape
    o = MetricPersistence(np.zeros((8, n), np.uint16), np.zeros(n, np.uint8), np.zeros(n, np.uint8),
                          np.full(n, -1, np.int32))
    _load().go_metric_window(n, primary, min_signals, _ptr(mask), T, W, k, _ptr(o.count),
                             _ptr(o.pmask), _ptr(o.flag), _ptr(o.first))
    return o


def score_ring(node_z: np.ndarray, W: int, quant: float = 64.0) -> np.ndarray:
    """sum[N] i32 of the quantised primary node scores over the last min(T, W) steps."""
    node_z = np.ascontiguousarray(node_z, np.float32)
    T, N = node_z.shape
    out = np.zeros(N, np.int32)
    _load().go_score_ring(N, _ptr(node_z), T, W, quant, _ptr(out))
    return out


def topk_mean(node_count: np.ndarray, score_sum: np.ndarray, k: int):
    """(idx[k] i32, key[k] u64) of the k slowest nodes by (count, windowed score sum, index)."""
    node_count = np.ascontiguousarray(node_count, np.uint16)
    score_sum = np.ascontiguousarray(score_sum, np.int32)
    N = node_count.shape[0]
    assert score_sum.shape[0] == N and 0 <= k <= N and N <= 65536
    idx = np.empty(k, np.int32)
    key = np.empty(k, np.uint64)
    _load().go_topk_mean(N, _ptr(node_count), _ptr(score_sum), k, _ptr(idx), _ptr(key))
    return idx, key


def recurrence(flag_hist: np.ndarray, horizon: int, limit: int = 3):
    """(episodes[N] u8, terminal_first[N] i32) from the per-step node flags flag_hist[T][N]."""
    flag_hist = np.ascontiguousarray(flag_hist, np.uint8)
    T, N = flag_hist.shape
    ep = np.zeros(N, np.uint8)
    tf = np.full(N, -1, np.int32)
    _load().go_recurrence(N, _ptr(flag_hist), T, horizon, limit, _ptr(ep), _ptr(tf))
    return ep, tf


def detect(p: Params, x: np.ndarray, topk_k: int, want_z: bool = False):
    """The whole path on one history x[t][m][r] starting at step 0."""
    s = score(p, x, want_z=want_z)
    pr = window(p.R, s.rank_anom, p.W, p.k)
    pn = window(p.N, s.node_anom, p.W, p.k)
    nf = node_flag_byte(p.G, pn.flag, pr.flag)
    last = s.node_z[-1] if x.shape[0] else np.zeros(p.N, np.float32)
    idx, key = topk(pn.count, last, topk_k)
    return dict(scores=s, ranks=pr, nodes=pn, node_flag_byte=nf, topk_idx=idx, topk_key=key)
