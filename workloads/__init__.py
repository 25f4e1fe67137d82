"""Seeded synthetic inputs: data-flow DAGs, device models and candidate partitions.

This package only *draws inputs*.  It holds none of the method's arithmetic (no
vertex or edge cost, no longest-path recurrence): both the CPU oracle's tests and
the GPU path's tests are fed from here, and neither of those imports the other.
"""
from .dags import (  # noqa: F401
    CONFIG_NAMES,
    Workload,
    asap_levels,
    build_csr,
    make_workload,
    random_layered_dag,
)
