"""Seeded synthetic DNN-shaped variable traces (input generator only).

This module produces the inputs shared by the CPU oracle and the HIP path.  It
contains none of the planner's arithmetic: no load profile, no placement, no
score is computed here.
"""
from .dnn import (  # noqa: F401
    CONFIG_NAMES,
    ORDER_SEED,
    TRACE_SEED_BASE,
    Trace,
    make_config,
    make_orderings,
    random_trace,
    tile_in_time,
)
