"""Seeded synthetic inputs for the fused generation + scoring stage.

This package only *draws inputs* (model weights, prompts, output lengths).  It holds
none of the method's arithmetic: no transformer maths, no scheduling.  Both the CPU
oracle's tests and the HIP library's callers take their inputs from here, so that the
two sides see the same bytes.
"""
from .configs import CONFIGS, ModelCfg, WorkloadCfg, get_config  # noqa: F401
from .generate import (  # noqa: F401
    ROLE_NAMES,
    draw_lengths,
    make_prompts,
    make_weights,
    make_workload,
    weight_shapes,
)
