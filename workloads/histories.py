"""Synthetic histories of what the scoring step hands to the bookkeeping that
follows it: one exceed byte per (step, item) -- bit m set when metric m of that
rank or node deviates -- and one node score per (step, node).

They stand in for the scoring outputs of long production runs (Section 4.2:
deviations that are sustained, next to isolated one-step spikes, Section 3) at
sizes and event rates chosen by the caller: a background of independent rare
bits, plus `bursts` -- stretches of consecutive steps in which an item deviates
in its first `burst_metrics` metrics, separated by quiet gaps, so that flags
rise, fall and rise again.

Random bits and numbers only: nothing here counts, windows, thresholds or ranks.
"""
from __future__ import annotations

import numpy as np


def exceed_history(seed: int, T: int, n: int, M: int, p_bit: float = 0.02, burst_items: int = 0,
                   burst_len=(10, 60), gap_len=(5, 80), burst_metrics: int = 2,
                   burst_density: float = 0.9) -> np.ndarray:
    """u8 [T][n]: bit m (m < M) set independently with probability p_bit; `burst_items`
    randomly chosen items additionally carry bursts."""
    rng = np.random.default_rng(seed)
    out = np.zeros((T, n), np.uint8)
    cut = np.uint16(min(65535, round(p_bit * 65536)))     # 16 random bits per draw
    for m in range(M):
        out |= (rng.integers(0, 65536, (T, n), dtype=np.uint16) < cut).astype(np.uint8) << np.uint8(m)
    if burst_items and T:
        items = rng.choice(n, size=min(burst_items, n), replace=False)
        bits = np.uint8((1 << min(burst_metrics, M)) - 1)
        for i in items:
            t = int(rng.integers(0, gap_len[1] + 1))
            while t < T:
                d = int(rng.integers(burst_len[0], burst_len[1] + 1))
                on = rng.random(min(d, T - t)) < burst_density
                out[t:t + d, i] |= np.where(on, bits, np.uint8(0)).astype(np.uint8)
                t += d + int(rng.integers(gap_len[0], gap_len[1] + 1))
    return out


def node_score_history(seed: int, T: int, N: int, scale: float = 1.0, outliers: float = 0.01) -> np.ndarray:
    """f32 [T][N] node scores: normal with the given scale, a fraction `outliers` of them
    100x larger (some beyond any 16-bit quantisation), and a sprinkle of exact halves
    of the 1/64 grid, zeros of both signs and infinities."""
    rng = np.random.default_rng(seed + 1)
    z = rng.standard_normal((T, N)) * scale
    big = rng.random((T, N)) < outliers
    z = np.where(big, z * 100.0, z)
    half = rng.random((T, N)) < 0.02
    z = np.where(half, (rng.integers(-200, 200, (T, N)) + 0.5) / 64.0, z)
    z = z.astype(np.float32)
    if T and N:
        flat = z.reshape(-1)
        k = max(1, flat.size // 500)
        flat[rng.choice(flat.size, k, replace=False)] = np.float32(-0.0)
        flat[rng.choice(flat.size, max(1, k // 4), replace=False)] = np.float32(np.inf)
        flat[rng.choice(flat.size, max(1, k // 4), replace=False)] = np.float32(-np.inf)
    return z
