"""Seeded synthetic latency workloads shared by the tests, the benchmark and the smoke check.

`spec` defines the tensors, `host` generates them on the CPU, `device` in GPU memory.
Nothing of the simulated method lives here.
"""
from . import spec  # noqa: F401
from .spec import CONFIG_NAMES, Recipe, config  # noqa: F401
