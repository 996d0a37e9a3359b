"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU path's tests.

This package only draws random vectors; it contains none of the method's
arithmetic (no quantiser, no lookup table, no distance).
"""
from .gmm import (CONFIGS, SEED_DATABASE, SEED_MIXTURE, SEED_QUERIES, SEED_TRAIN, GaussianMixture,
                  WorkloadConfig, get_config, near_tie_vectors)

__all__ = ["GaussianMixture", "CONFIGS", "WorkloadConfig", "get_config",
           "SEED_MIXTURE", "SEED_TRAIN", "SEED_DATABASE", "SEED_QUERIES", "near_tie_vectors"]
