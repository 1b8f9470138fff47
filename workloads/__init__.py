"""Seeded synthetic workloads (shapes, recipes, margins) shared by tests and bench."""
from .configs import ORDER, WORKLOADS, Workload  # noqa: F401
from .generate import generate, generate_all, generate_sequences  # noqa: F401
