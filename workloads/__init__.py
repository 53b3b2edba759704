"""Seeded synthetic workloads shared by the oracle's tests and the GPU path's tests."""
from .generators import (CONFIGS, FP8, FP16, FP32, FP64, MASTER_SEED, Workload, covariance,
                         decay_rect, morton_points, paper_ratio, random_maps, tiny)

__all__ = ["CONFIGS", "FP8", "FP16", "FP32", "FP64", "MASTER_SEED", "Workload", "covariance",
           "decay_rect", "morton_points", "paper_ratio", "random_maps", "tiny"]
