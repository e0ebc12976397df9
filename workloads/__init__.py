"""Seeded synthetic workloads (shapes, value recipes, bit plans) shared by tests and bench.py.

This package holds none of the method's arithmetic: it only names tensor shapes, draws random
inputs and moves them into device memory.
"""
from .configs import Workload, get_workload, WORKLOADS  # noqa: F401
