"""Seeded synthetic input generators (no aggregation arithmetic lives here)."""
from . import counter
from .synthetic import C1, C2, C3, C4, C5, CONFIGS, E14, EXTRA, Workload, resnet50_layer_sizes, stream, to_oracle_input

__all__ = ["counter", "C1", "C2", "C3", "C4", "C5", "CONFIGS", "E14", "EXTRA", "Workload", "resnet50_layer_sizes", "stream", "to_oracle_input"]
