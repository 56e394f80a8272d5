"""Seeded synthetic inputs shared by the GPU tests, the bench and the CPU checker.

This package only *generates data* (random fields, matrices, graphs, task
lists with arrival times).  It contains none of the arithmetic of the
scheduling method or of the task kernels, and imports neither the HIP library
binding nor the CPU checker.
"""
from .rng import (raw64, uniform01, normal, task_seed, f32_to_bf16_bits,
                  bf16_bits_to_f32, exponential)
from .data import (jacobi_field, gemm_operands_f32, gemm_operands_bf16, er_digraph_csr,
                   er_graph_csr, cnn_layers, cnn_weights, cnn_input, task_data)
from .mixes import TaskSpec, mix4, mix16, cnn8, pressure32, mixed128, kinds5, MIXES

__all__ = [
    "raw64", "uniform01", "normal", "task_seed", "f32_to_bf16_bits",
    "bf16_bits_to_f32", "exponential", "jacobi_field", "gemm_operands_f32",
    "gemm_operands_bf16", "er_graph_csr", "er_digraph_csr", "cnn_layers", "cnn_weights",
    "cnn_input", "task_data", "TaskSpec", "mix4", "mix16", "cnn8", "pressure32", "kinds5",
    "mixed128", "MIXES",
]
