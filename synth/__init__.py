"""Seeded synthetic inputs (shapes, weights, hidden-state streams) shared by tests, bench and smoke."""
from .workloads import CONFIGS, MoEWorkload  # noqa: F401
