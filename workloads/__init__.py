"""Seeded synthetic workloads: tensor-shape recipes and value generators. No method arithmetic here."""
from . import shapes
from .generate import Workload, FULL, small, config1, config2, config3, config4, config5, table1

__all__ = ["shapes", "Workload", "FULL", "small", "config1", "config2", "config3", "config4", "config5", "table1"]
