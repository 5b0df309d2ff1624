"""Seeded synthetic workloads: layer shapes (`configs`) and tensor generators (`gen`)."""
from . import configs, gen  # noqa: F401
