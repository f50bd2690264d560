"""Seeded synthetic inputs for pipelined-reduction-schedule sweeps.

This module only draws numbers: it holds none of the method's arithmetic (no
segmentation, no cost model, no scheduling).  Both the CPU oracle's tests and
the GPU path read the arrays produced here, so random-number generation is not
part of any parity claim.

The parameter ranges follow the simulation set-ups of the paper (Section 5.2:
p = 2^k <= 1024, alpha in {0..1000}, beta = 1, gamma in {0,1}; Section 6.1:
alpha = 50000, beta = 6, gamma = 1; Section 8: m = 10 with all segmentations),
widened to log-uniform draws so a sweep covers the whole range in one batch.
"""
from .sweeps import (  # noqa: F401
    SweepConfigs,
    tiny_sweep,
    random_sweep,
    uni_sweep,
    large_p_sweep,
    replay_config,
    replay_buffers,
    SEED_UNI,
    SEED_LARGE_P,
    SEED_REPLAY,
)
