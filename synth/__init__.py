"""Seeded synthetic input generators (shared by oracle tests and GPU tests)."""
from .gradients import WORKLOADS, Segment, Workload, generate, to_numpy_bits, workload  # noqa: F401
