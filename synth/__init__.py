"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP library's tests."""
from .workloads import (FLAT, HYPER, ITER_BATCHES, ITER_DRIFT, ITER_K, ITER_NPROBE, ITER_ROUNDS, KSUB, MID,
                        TINY, FlatConfig, GaussianMixture, IvfPqConfig, build_index, build_upper_level, drift_queries,
                        make_flat, make_queries, random_index)
from .indexfile import write_index
