"""Seeded synthetic telemetry inputs.

This package only *produces input tensors* (and the ground truth of what was
injected into them).  It contains none of the detector's arithmetic: no median,
no MAD, no score, no window logic.  Both the CPU oracle's tests and the GPU
path's tests draw their inputs from here so that the two sides always see the
same bytes.
"""
from .telemetry import (  # noqa: F401
    Workload,
    Fault,
    workload,
    generate,
    generate_chunks,
    adversarial,
    N_CONFIGS,
)
