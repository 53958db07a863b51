"""Synthetic per-rank x per-step x per-metric telemetry tensors.

The paper's detector consumes production telemetry (training-step time as the
primary signal plus hardware indicators, Section 4.1 / 4.2; 8-GPU nodes,
Section 7.1) that is not public.  The tensors made here stand in for it: dense
fp32 ``x[t][m][r]`` (rank innermost), with the two slowdown behaviours the
paper describes in Section 3 -- nodes that are persistently slower than their
peers, and transient one-step spikes -- injected at known places.

Everything is drawn in fp64 from a ``torch.Generator`` seeded per
(seed, workload, chunk of steps), then rounded once to fp32, so any range of
steps can be produced independently, on the CPU or on a GPU.  The values for a
given seed differ between devices (torch's CPU and GPU generators differ);
what matters is that one tensor, once made, is handed to every consumer as the
same bytes.

Nothing in this file scores, ranks, thresholds or windows anything.
"""
from __future__ import annotations

import dataclasses
import math
from dataclasses import dataclass
from typing import Iterator, List, Optional, Sequence, Tuple

import numpy as np
import torch

N_CONFIGS = 5


@dataclass(frozen=True)
class Fault:
    """One injected slowdown: ranks [rank_lo, rank_hi) are multiplied in step
    time by a factor that is 1 before ``onset`` and reaches ``factor`` after
    ``ramp`` further steps (``ramp == 0``: immediately)."""

    kind: str          # "node" (all 8 GPUs of a node) or "gpu" (one rank)
    rank_lo: int
    rank_hi: int
    onset: int
    factor: float
    ramp: int = 0


@dataclass(frozen=True)
class Workload:
    """Shape, detector parameters and generator recipe of one configuration."""

    name: str
    index: int
    R: int                      # ranks
    T: int                      # steps
    M: int                      # metrics
    W: int                      # persistence window
    k: int                      # flags needed inside the window
    topk: int
    directions: Tuple[int, ...]  # +1 higher is worse, -1 lower is worse
    noise: str                  # "lognormal" or "student_t3"
    recipe: str                 # "single", "derived4", "indep8"
    G: int = 8
    thr: float = 3.5
    primary: int = 0
    sigma: float = 0.02
    spike_p: float = 0.0
    n_fault_nodes: int = 0
    n_fault_gpus: int = 0
    fault_lo: float = 1.0
    fault_hi: float = 1.0
    fault_ramp: int = 0
    chunk_steps: int = 64

    @property
    def N(self) -> int:
        return self.R // self.G

    @property
    def min_signals(self) -> int:
        return min(2, self.M)

    @property
    def samples(self) -> int:
        return self.R * self.T * self.M


# Bases of the eight metrics of the heavy-tailed recipe: step time (s), compute
# time (s), collective wait (s), achieved TFLOPS, GPU temperature (C), GPU clock
# (GHz), power (W), NIC transmission rate (Gb/s) -- the indicator families of
# Section 4.1; the exponent says how the metric moves when the rank slows down.
_BASES8 = (1.0, 0.7, 0.3, 400.0, 65.0, 1.93, 700.0, 400.0)
_EXPS8 = (1, 1, 1, -1, 1, -1, -1, -1)


def workload(index: int, **override) -> Workload:
    """The five configurations; ``override`` (e.g. ``T=8``) gives a reduced or
    reshaped variant with the same recipe (fault counts are capped to the
    number of nodes available)."""
    if index == 0:
        w = Workload("tiny-64r-200s-1m", 0, R=64, T=200, M=1, W=20, k=15, topk=8,
                     directions=(1,), noise="lognormal", recipe="single")
    elif index == 1:
        w = Workload("1024r-2000s-4m", 1, R=1024, T=2000, M=4, W=50, k=40, topk=64,
                     directions=(1, 1, 1, -1), noise="lognormal", recipe="derived4",
                     spike_p=0.001, n_fault_nodes=8, fault_lo=1.05, fault_hi=1.30)
    elif index == 2:
        w = Workload("16384r-10000s-4m", 2, R=16384, T=10000, M=4, W=100, k=80, topk=64,
                     directions=(1, 1, 1, -1), noise="lognormal", recipe="derived4",
                     spike_p=0.005, n_fault_nodes=64, fault_lo=1.03, fault_hi=1.20)
    elif index == 3:
        w = Workload("65536r-4096s-8m", 3, R=65536, T=4096, M=8, W=256, k=200, topk=64,
                     directions=_EXPS8, noise="student_t3", recipe="indep8",
                     n_fault_nodes=32, n_fault_gpus=16, fault_lo=1.20, fault_hi=1.20,
                     fault_ramp=2000, chunk_steps=16)
    elif index == 4:
        w = Workload("stream-32768r-8m", 4, R=32768, T=100000, M=8, W=256, k=200, topk=64,
                     directions=_EXPS8, noise="student_t3", recipe="indep8",
                     n_fault_nodes=48, fault_lo=1.05, fault_hi=1.20, chunk_steps=32)
    else:
        raise ValueError(f"no configuration {index}")
    if override:
        w = dataclasses.replace(w, **override)
        if w.R % w.G:
            raise ValueError("R must be a multiple of G")
        cap = max(1, w.N // 16)
        w = dataclasses.replace(w, n_fault_nodes=min(w.n_fault_nodes, cap),
                                n_fault_gpus=min(w.n_fault_gpus, cap),
                                topk=min(w.topk, w.N), k=min(w.k, w.W))
    return w


def faults(w: Workload, seed: int) -> List[Fault]:
    """Where the slowdowns go, as a deterministic function of (workload, seed)."""
    if w.index == 0:
        return [Fault("gpu", r, r + 1, 50, 1.15) for r in (5, 42) if r < w.R]
    rng = np.random.Generator(np.random.PCG64([seed, w.index, 0xFA17]))
    out: List[Fault] = []
    n_nodes = min(w.n_fault_nodes, w.N)
    nodes = rng.choice(w.N, size=n_nodes, replace=False) if n_nodes else np.zeros(0, int)
    for n in nodes:
        factor = float(rng.uniform(w.fault_lo, w.fault_hi))
        if w.index == 3:
            onset = int(rng.integers(0, max(1, w.T - w.fault_ramp + 1)))
        elif w.index == 4:
            onset = int(rng.integers(0, w.T))
        else:
            onset = int(rng.integers(0, max(1, w.T // 2)))
        out.append(Fault("node", int(n) * w.G, int(n) * w.G + w.G, onset, factor, w.fault_ramp))
    if w.n_fault_gpus:
        free = np.setdiff1d(np.arange(w.N), nodes)
        hosts = rng.choice(free, size=min(w.n_fault_gpus, len(free)), replace=False)
        for n in hosts:
            r = int(n) * w.G + int(rng.integers(0, w.G))
            onset = int(rng.integers(0, max(1, w.T // 2)))
            out.append(Fault("gpu", r, r + 1, onset, 1.10))
    return out


def _slow(w: Workload, fl: Sequence[Fault], t0: int, t1: int, device) -> torch.Tensor:
    """slow[t][r] >= 1 for steps t0..t1-1, fp64."""
    s = torch.ones((t1 - t0, w.R), dtype=torch.float64, device=device)
    t = torch.arange(t0, t1, dtype=torch.float64, device=device)
    for f in fl:
        if f.onset >= t1:
            continue
        if f.ramp > 0:
            frac = ((t - f.onset) / float(f.ramp)).clamp_(0.0, 1.0)
        else:
            frac = (t >= f.onset).to(torch.float64)
        s[:, f.rank_lo:f.rank_hi] *= (1.0 + (f.factor - 1.0) * frac)[:, None]
    return s


def _chunk_generator(w: Workload, seed: int, chunk: int, device) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed((seed * 1_000_003 + w.index * 7_919 + 1) * 2_654_435_761 % (2**62) + chunk)
    return g


def _noise(w: Workload, shape, g: torch.Generator, device) -> torch.Tensor:
    """Log-space noise, fp64: sigma*N(0,1) or sigma*Student-t(3)."""
    z = torch.randn(shape, dtype=torch.float64, device=device, generator=g)
    if w.noise == "student_t3":
        c = torch.randn((3,) + tuple(shape), dtype=torch.float64, device=device, generator=g)
        z = z / torch.sqrt((c * c).sum(0) / 3.0)
    elif w.noise != "lognormal":
        raise ValueError(w.noise)
    return z.mul_(w.sigma)


def _make_chunk(w: Workload, fl: Sequence[Fault], seed: int, chunk: int, device) -> torch.Tensor:
    """Steps [chunk*chunk_steps, (chunk+1)*chunk_steps) clipped to T: fp32 [t][M][R]."""
    t0 = chunk * w.chunk_steps
    t1 = min(w.T, t0 + w.chunk_steps)
    n = t1 - t0
    g = _chunk_generator(w, seed, chunk, device)
    slow = _slow(w, fl, t0, t1, device)
    if w.recipe == "single":
        step = torch.exp(_noise(w, (n, w.R), g, device)) * slow
        return step.to(torch.float32)[:, None, :].contiguous()
    if w.recipe == "derived4":
        step = torch.exp(_noise(w, (n, w.R), g, device)) * slow
        if w.spike_p > 0:
            hit = torch.rand((n, w.R), dtype=torch.float64, device=device, generator=g) < w.spike_p
            step = torch.where(hit, step * 2.0, step)
        x = torch.empty((n, 4, w.R), dtype=torch.float32, device=device)
        x[:, 0] = step.to(torch.float32)
        x[:, 1] = (0.7 * step).to(torch.float32)
        x[:, 2] = x[:, 0] - x[:, 1]          # collective wait = step - compute, in fp32
        x[:, 3] = (400.0 / step).to(torch.float32)
        return x[:, : w.M].contiguous()
    if w.recipe == "indep8":
        noise = _noise(w, (n, w.M, w.R), g, device)
        base = torch.tensor(_BASES8[: w.M], dtype=torch.float64, device=device)[None, :, None]
        e = torch.tensor(_EXPS8[: w.M], dtype=torch.float64, device=device)[None, :, None]
        x = base * torch.pow(slow[:, None, :], e) * torch.exp(noise)
        return x.to(torch.float32).contiguous()
    raise ValueError(w.recipe)


def generate_chunks(w: Workload, seed: int, t0: int = 0, t1: Optional[int] = None,
                    device="cpu") -> Iterator[Tuple[int, torch.Tensor]]:
    """Yield (first_step, x[t][M][R] fp32) pieces covering steps [t0, t1)."""
    t1 = w.T if t1 is None else t1
    if not (0 <= t0 <= t1 <= w.T):
        raise ValueError("bad step range")
    fl = faults(w, seed)
    c = t0 // w.chunk_steps
    while c * w.chunk_steps < t1:
        x = _make_chunk(w, fl, seed, c, device)
        lo = c * w.chunk_steps
        a, b = max(t0, lo) - lo, min(t1, lo + x.shape[0]) - lo
        yield lo + a, x[a:b]
        c += 1


def generate(w: Workload, seed: int, t0: int = 0, t1: Optional[int] = None, device="cpu",
             out: Optional[torch.Tensor] = None) -> torch.Tensor:
    """x[t][M][R] fp32 for steps [t0, t1) as one contiguous tensor."""
    t1 = w.T if t1 is None else t1
    if out is None:
        out = torch.empty((t1 - t0, w.M, w.R), dtype=torch.float32, device=device)
    for first, piece in generate_chunks(w, seed, t0, t1, device):
        out[first - t0: first - t0 + piece.shape[0]] = piece
    return out


def adversarial(kind: str, R: int, T: int, M: int, seed: int) -> torch.Tensor:
    """Small CPU tensors that stress the selection rather than look like
    telemetry: ties, signs, zeros, wide dynamic range, sorted input."""
    g = torch.Generator().manual_seed(seed * 7 + 13)
    shape = (T, M, R)
    if kind == "constant":            # every rank identical per column
        col = 0.5 + torch.rand((T, M, 1), generator=g, dtype=torch.float64)
        x = col.expand(shape).clone()
    elif kind == "ramp":              # x_r = r
        x = torch.arange(R, dtype=torch.float64).expand(shape).clone()
    elif kind == "ramp_desc":
        x = torch.arange(R - 1, -1, -1, dtype=torch.float64).expand(shape).clone()
    elif kind == "ties":              # few distinct values, like an integer sensor
        x = torch.randint(60, 70, shape, generator=g).to(torch.float64)
    elif kind == "two_values":        # half the ranks at one value
        x = torch.where(torch.rand(shape, generator=g, dtype=torch.float64) < 0.5, 1.0, 1.25)
        x = x.to(torch.float64)
    elif kind == "mixed_sign":        # negatives, positives, both zeros
        x = torch.randn(shape, generator=g, dtype=torch.float64)
        z = torch.rand(shape, generator=g, dtype=torch.float64)
        x = torch.where(z < 0.1, torch.zeros_like(x), x)
        x = torch.where((z >= 0.1) & (z < 0.2), -torch.zeros_like(x), x)
    elif kind == "wide_range":        # magnitudes over many binades, both signs
        e = torch.rand(shape, generator=g, dtype=torch.float64) * 60.0 - 30.0
        s = torch.where(torch.rand(shape, generator=g, dtype=torch.float64) < 0.5, -1.0, 1.0)
        x = s * torch.pow(torch.tensor(2.0, dtype=torch.float64), e)
    elif kind == "negative":          # an all-negative metric
        x = -(1.0 + 0.02 * torch.randn(shape, generator=g, dtype=torch.float64))
    elif kind == "lone_outlier":      # identical data with a single outlier per column
        x = torch.ones(shape, dtype=torch.float64)
        idx = torch.randint(0, R, (T, M, 1), generator=g)
        x.scatter_(2, idx, 3.0)
    elif kind == "denormal":          # subnormal magnitudes
        x = torch.randint(-2000, 2000, shape, generator=g).to(torch.float64) * 2.0 ** -149
    elif kind == "huge":              # large magnitudes, both signs
        x = (1.0 + torch.rand(shape, generator=g, dtype=torch.float64)) * 2.0 ** 100
        s = torch.where(torch.rand(shape, generator=g, dtype=torch.float64) < 0.3, -1.0, 1.0)
        x = x * s
    elif kind == "gauss":
        x = 1.0 + 0.02 * torch.randn(shape, generator=g, dtype=torch.float64)
    else:
        raise ValueError(kind)
    return x.to(torch.float32).contiguous()


ADVERSARIAL_KINDS = ("constant", "ramp", "ramp_desc", "ties", "two_values", "mixed_sign",
                     "wide_range", "negative", "lone_outlier", "denormal", "huge", "gauss")
