"""Seeded synthetic workloads shared by the CPU oracle and the GPU library (no method arithmetic)."""
from .graph import Graph, Node, min_hbm_bytes, ELEM_BYTES, FREE_OPS  # noqa: F401
from .configs import (  # noqa: F401
    workload, softmax_graph, softmax_inputs, layernorm_gelu_graph, layernorm_gelu_inputs,
    elementwise20_graph, elementwise20_inputs, multi_reduce_graph, multi_reduce_inputs,
    random_dag_graph, random_dag_inputs, layernorm_grad_graph, layernorm_grad_inputs,
    softmax_grad_graph, softmax_grad_inputs, f32_to_bf16_bits, bf16_bits_to_f32, sha256_of, BASE_SEED,
)
