"""Seeded synthetic inputs for the Placeto policy forward pass.

This package only *draws inputs*: DAG topologies shaped like the paper's workloads
(Section 3 and Appendix A.2: Inception-V3, NMT, NASNet training graphs), per-node raw
features (Section 2.1), mid-episode states and network weights.  It contains none of the
method's arithmetic (no message passing, no levels, no reachability, no rounding of
weights); both the float64 CPU oracle and the HIP library consume what it produces.
"""
from .synthetic import (  # noqa: F401
    CONFIG_NAMES,
    Workload,
    make_workload,
    make_states,
    make_episode,
    tiny_random_dag,
    weight_layout,
    weight_count,
)
