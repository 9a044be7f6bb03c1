"""Seeded synthetic input generators and workload records (data only)."""
from .configs import CONFIGS, Config, get  # noqa: F401
from . import generate  # noqa: F401
