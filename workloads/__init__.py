"""Seeded synthetic PQ-code workloads shaped like the paper's datasets.

This package holds input generators only -- none of the method's arithmetic --
so that the CPU oracle and the HIP path can both be fed the same bytes without
importing each other.
"""
from .synth import (CONFIGS, Workload, codewords, codes_numpy, codes_torch, codes_at,
                    init_center_indices, templates)

__all__ = ["CONFIGS", "Workload", "codewords", "codes_numpy", "codes_torch", "codes_at",
           "init_center_indices", "templates"]
