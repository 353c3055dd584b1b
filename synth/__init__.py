"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests.

Holds record layouts, payload value generators, the multipath arrival model and
the workload builders.  It contains none of the data path's arithmetic and imports
neither the oracle nor the GPU library.
"""
from . import layout, payload, arrivals, workloads, control_sim  # noqa: F401
