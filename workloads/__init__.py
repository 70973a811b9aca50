"""Seeded synthetic inputs shared by the CPU oracle and the HIP path.

This package only *draws data*: model shapes, random weights, random K/V
context and draft-tree shapes.  It contains none of the method's arithmetic
(no transformer layer, no attention, no acceptance rule), so that the oracle
and the device library can be fed byte-identical inputs without sharing code.
"""
from .configs import ModelConfig, CONFIGS, get_config            # noqa: F401
from .rng import normal_f32, f32_to_bf16_bits, bf16_bits_to_f32  # noqa: F401
from .weights import gen_weights, tensor_shapes, TENSOR_KINDS    # noqa: F401
from .kv import gen_context_kv                                   # noqa: F401
from .trees import (chain_tree, schema_retrieval_tree, bfs_tree,  # noqa: F401
                    retrieval_tree, mutate_chain, tree_depths, root_token, load_greedy,
                    random_tree, decision_sweep_case)
