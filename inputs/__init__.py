"""Seeded synthetic inputs for the RoCo hot path.

This package holds only input generation (random draws, the heavy-hitter
structure of the workload, bf16 rounding of the *inputs*).  It contains none
of the method's arithmetic: no attention, no statistics, no selection.  Both
the CPU oracle's tests and the HIP path's tests draw their inputs from here.
"""
from .heavy_hitter import (  # noqa: F401
    CONFIGS,
    WorkloadConfig,
    UnitInputs,
    make_unit,
    make_units,
    round_to_bf16,
    unit_ids,
)
