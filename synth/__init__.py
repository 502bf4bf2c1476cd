"""Seeded synthetic inputs for the KV-reclaim path (workloads and byte content).

Shared by the tests, the benchmark and the smoke check.  Contains input
generation only: nothing of the relocation method itself.
"""
from .workloads import (CONFIGS, KVConfig, Workload, bitmap_from_ids, bitmap_to_bools, config,
                        dense_offsets, make_workload, weight_shapes_8b)

__all__ = ["CONFIGS", "KVConfig", "Workload", "bitmap_from_ids", "bitmap_to_bools", "config",
           "dense_offsets", "make_workload", "weight_shapes_8b"]
