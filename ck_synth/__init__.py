"""Seeded synthetic workloads shared by the tests, the benchmark and the CPU checker.

This package holds input generation only: shapes of the five benchmark
configurations, the Gaussian-mixture key/value/query generator and the random
draws K-means consumes (the shuffled candidate order for its initial centroids).
It contains none of the method's arithmetic.
"""
from .configs import CONFIGS, Config, get_config
from .mixture import MixtureWorkload, sample_init_indices

__all__ = ["CONFIGS", "Config", "get_config", "MixtureWorkload", "sample_init_indices"]
