"""Seeded synthetic inputs (graphs, partitions, tensors) for the SAT hot path.

This package holds no arithmetic of the method itself: it only draws random
graphs, partition vectors, feature / weight / noise tensors and labels. Both
the CPU oracle's tests and the HIP library's tests and benchmark take their
inputs from here, so the two sides see identical bytes without sharing code.
"""
from .configs import CONFIGS, get_config
from .graphs import (Graph, sbm_graph, chung_lu_planted_graph, chung_lu_partition_rows,
                     ring_graph, make_graph, cached_graph)
from .tensors import (substreams, normal_f32, glorot_uniform_f32, labels_i32,
                      predictor_params_f32, history_standin_f32, bf16_bits_from_f32,
                      f32_from_bf16_bits, device_normal, device_history_standin, gat_heads,
                      attention_vectors_f32, drifting_history_f32)

__all__ = [
    "CONFIGS", "get_config", "Graph", "sbm_graph", "chung_lu_planted_graph",
    "ring_graph", "make_graph", "cached_graph", "substreams", "normal_f32",
    "glorot_uniform_f32", "labels_i32", "predictor_params_f32",
    "history_standin_f32", "bf16_bits_from_f32", "f32_from_bf16_bits",
    "chung_lu_partition_rows", "device_normal", "device_history_standin", "gat_heads",
    "attention_vectors_f32", "drifting_history_f32",
]
