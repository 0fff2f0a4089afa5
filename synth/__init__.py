"""Seeded synthetic inputs (shared by the CPU checker's tests and the GPU library's tests)."""
from . import rng, workloads
from .workloads import WORKLOADS, Workload

__all__ = ["rng", "workloads", "WORKLOADS", "Workload"]
