"""Seeded synthetic workloads for the multi-step SSM verification path.

This package only draws random inputs (shapes, distributions, acceptance
lengths).  It contains none of the method's arithmetic and is the one module
that both the CPU oracle's tests and the HIP path's tests/bench may share.
"""
from .configs import Workload, CONFIGS, get_workload  # noqa: F401
from .generate import (  # noqa: F401
    WorkloadData, RoundInputs, LayerParams, generate, round_to_io, draw_accepted, BlockExtras, block_extras,
)
