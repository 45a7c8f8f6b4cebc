"""Seeded synthetic input generators shared by the oracle's tests and the GPU path's tests."""
from .gen import *  # noqa: F401,F403
from .gen import CONFIGS, Workload  # noqa: F401
