"""Seeded synthetic inputs: cost tables, cluster descriptions and candidate lists.

This package only *draws inputs*.  It holds none of the simulator's arithmetic
(no schedules, no recurrence, no collective-cost evaluation of the method): the
per-layer event times it emits play the role of the profiled event times that
DistSim's event profiler would deliver (Sec. 4.2), and the candidate lists play
the role of the strategy grid of Sec. 6.
"""
from .configs import (  # noqa: F401
    Workload,
    make_workload,
    enumerate_triples,
    subset,
    total_stages,
    CONFIG_NAMES,
    make_operator_records,
    make_comm_profiles,
)
