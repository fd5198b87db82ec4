"""Seeded synthetic inputs shared by the CPU oracle, the tests and the benchmark.

This package generates inputs only: Gaussian-mixture sample matrices, grown
forests (flattened trees plus bootstrap in-bag counts and leaf class labels) and random start blocks.
It contains none of the proximity path's arithmetic.

The five workloads follow the shapes of the paper's evaluation: its only
measured data set is 178 rows x 13 features in 3 classes (Results,
"Datasets"), and its scalability tables go from 10k to 200k rows (Results,
"Memory Feasibility Analysis").  Those records are not available, so seeded
Gaussian mixtures of the same shapes stand in for them.
"""
from .mixture import CONFIGS, WorkloadConfig, gaussian_mixture, random_int8_factor, start_block, workload
from .forest import Forest, build_grower, grow_forest, leaf_classes, load_or_grow

__all__ = [
    "CONFIGS",
    "WorkloadConfig",
    "gaussian_mixture",
    "start_block",
    "random_int8_factor",
    "workload",
    "Forest",
    "build_grower",
    "grow_forest",
    "leaf_classes",
    "load_or_grow",
]
