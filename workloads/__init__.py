"""Seeded synthetic ASNN workloads (edge lists, weights, input batches).

This package only *draws* networks and inputs.  It contains none of the
method's arithmetic (no level computation, no activation): both the CPU
oracle and the HIP library consume what it produces, and neither is imported
from here.
"""
from .gen import (  # noqa: F401
    Workload,
    tiny_neat,
    pruned_mlp,
    layered_skip,
    deep_narrow,
    population,
    make_config,
    CONFIG_NAMES,
)
