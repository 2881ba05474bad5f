"""Seeded synthetic inputs for the ES-SpMM hot path.

This package only *builds inputs* (CSR graphs, edge values, dense feature
matrices).  It contains none of the method's arithmetic (no sampling rule, no
SpMM) and is the one module shared by the CPU oracle's tests and the HIP path's
tests / benchmark.
"""
from .graphs import (  # noqa: F401
    CONFIG_IDS,
    Workload,
    make_workload,
    csr_from_degrees,
    gcn_operands,
    powerlaw_degrees,
    random_csr,
)
