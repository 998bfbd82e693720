"""Seeded synthetic workload generators (inputs only).

This package draws the arrays a scheduling tick consumes: job profiles,
progress points, gaps and per-job preferences.  It holds none of the method's
arithmetic (no prefix sums over profiles, no fit test, no scores), so both the
CPU oracle's tests and the GPU path can be fed from it without sharing any
computation.
"""
from .workloads import CONFIGS, Workload, make_workload, make_gaps, make_channels, config_names  # noqa: F401
