"""Seeded synthetic workload generators shared by the CPU oracle's tests and the GPU harness."""
from .gen import *  # noqa: F401,F403
