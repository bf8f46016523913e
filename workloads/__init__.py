"""Synthetic workloads: subgraph descriptors and seeded inputs (no op arithmetic)."""
from .graphs import (DTYPE_BYTES, DTYPES, EXPLORE_CONFIGS, FULL_CONFIGS, GENERIC_CONFIGS, NEXT_CONFIGS, OPCODES, PACK_CONFIGS, GraphSpec, OpSpec, TensorSpec,
                     add_bias_layernorm_graph, attention_scores_graph, bias_gelu_dbias_graph,
                     bias_gelu_graph, layernorm_backward_graph, rmsnorm_graph, softmax_backward_graph, softmax_graph,
                     transpose_chain_graph, transpose_graph, layernorm_stats_graph, silu_gate_graph, bias_gradient_chain_graph, log_softmax_graph, sigmoid_gate_graph, l1_l2_scale_graph,
                     scaled_softmax_colbias_graph, normalize_from_stats_graph, outer_scale_graph, random_row_pattern, transformer_block_graph, transformer_stack_graph, random_multi_pattern, independent_tiny_patterns_graph, masked_scores_gate_graph,
                     bias_head_split_graph, head_merge_residual_graph, transpose_chain_stats_graph, transposed_softmax_graph,
                     gelu_backward_graph, rmsnorm_backward_graph, transformer_block_backward_graph,
                     layernorm_backward_bias_graph)
from .inputs import f64_to_bf16_bits, make_inputs, quantise, valid_lengths

__all__ = [
    "DTYPE_BYTES", "DTYPES", "EXPLORE_CONFIGS", "FULL_CONFIGS", "GENERIC_CONFIGS", "NEXT_CONFIGS", "OPCODES", "PACK_CONFIGS", "GraphSpec", "OpSpec", "TensorSpec",
    "add_bias_layernorm_graph", "attention_scores_graph", "bias_gelu_dbias_graph", "bias_gelu_graph",
    "softmax_graph", "softmax_backward_graph", "layernorm_backward_graph", "rmsnorm_graph", "transpose_chain_graph", "transpose_graph",
    "layernorm_stats_graph", "silu_gate_graph", "bias_gradient_chain_graph", "log_softmax_graph", "sigmoid_gate_graph", "l1_l2_scale_graph", "scaled_softmax_colbias_graph", "normalize_from_stats_graph",
    "outer_scale_graph", "random_row_pattern", "transformer_block_graph", "transformer_stack_graph", "random_multi_pattern", "independent_tiny_patterns_graph", "masked_scores_gate_graph", "bias_head_split_graph", "head_merge_residual_graph",
    "transpose_chain_stats_graph", "transposed_softmax_graph", "gelu_backward_graph", "rmsnorm_backward_graph", "transformer_block_backward_graph", "layernorm_backward_bias_graph", "f64_to_bf16_bits", "make_inputs", "quantise", "valid_lengths",
]
