"""Seeded synthetic inputs for the Task-KV hot path.

This module is the ONLY code shared by the HIP path's tests/benchmark and the
CPU oracle's tests.  It holds none of the method's arithmetic: it draws random
tensors with the shapes, value distributions and structure of the five named
workloads and knows nothing about scores, selections or attention.  The
budget constants of the 32-layer workload are literals (a CPU test checks
them against the oracle's budget formula).
"""
from .workloads import (Workload, WORKLOADS, LayerData, make_layer, layer_params,
                        small_workload, to_numpy)

__all__ = ["Workload", "WORKLOADS", "LayerData", "make_layer", "layer_params",
           "small_workload", "to_numpy"]
