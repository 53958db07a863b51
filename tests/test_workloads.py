"""The synthetic inputs: shapes, determinism, chunk independence, recipes."""
import numpy as np
import pytest
import torch

from workloads import adversarial, generate, workload
from workloads.telemetry import ADVERSARIAL_KINDS, faults


def test_configuration_shapes():
    shapes = [(64, 200, 1, 20, 15), (1024, 2000, 4, 50, 40), (16384, 10000, 4, 100, 80),
              (65536, 4096, 8, 256, 200), (32768, 100000, 8, 256, 200)]
    for i, (R, T, M, W, k) in enumerate(shapes):
        w = workload(i)
        assert (w.R, w.T, w.M, w.W, w.k) == (R, T, M, W, k) and w.G == 8 and w.thr == 3.5
    assert workload(3).samples == 2 ** 31 and workload(3).topk == 64


@pytest.mark.parametrize("i", [0, 1, 3])
def test_any_step_range_can_be_made_independently(i):
    w = workload(i, R=min(workload(i).R, 256), T=150)
    full = generate(w, seed=3)
    assert full.shape == (150, w.M, w.R) and full.dtype == torch.float32
    part = generate(w, seed=3, t0=37, t1=141)
    assert torch.equal(part, full[37:141])
    assert not torch.equal(generate(w, seed=4), full)
    assert torch.isfinite(full).all() and (full > 0).all()


def test_derived_metrics_recipe():
    w = workload(1, T=64)
    x = generate(w, seed=1)
    assert torch.equal(x[:, 2], x[:, 0] - x[:, 1])
    assert torch.allclose(x[:, 1], 0.7 * x[:, 0], rtol=1e-6)
    assert torch.allclose(x[:, 3] * x[:, 0], torch.full_like(x[:, 0], 400.0), rtol=1e-6)
    step = x[:, 0].double()
    assert abs(float(step.log().median())) < 2e-3
    q = torch.quantile(step.log().flatten(), torch.tensor([0.25, 0.75], dtype=torch.float64))
    assert abs(float(q[1] - q[0]) / 1.349 - 0.02) < 2e-3    # interquartile range of N(0, 0.02)


def test_faults_are_injected_where_the_ground_truth_says():
    w = workload(1)
    fl = faults(w, seed=1)
    assert len(fl) == 8 and len({f.rank_lo for f in fl}) == 8
    x = generate(w, seed=1, t0=1500, t1=1600)
    for f in fl:
        assert f.rank_hi - f.rank_lo == 8 and 1.05 <= f.factor <= 1.30 and f.onset < 1000
        got = float(x[:, 0, f.rank_lo:f.rank_hi].double().log().mean().exp())
        assert abs(got / f.factor - 1) < 0.02
    w3 = workload(3, T=64)
    assert len(faults(workload(3), 3)) == 48


def test_adversarial_inputs_are_finite_fp32():
    for kind in ADVERSARIAL_KINDS:
        x = adversarial(kind, 64, 3, 2, seed=1)
        assert x.shape == (3, 2, 64) and x.dtype == torch.float32 and torch.isfinite(x).all()
