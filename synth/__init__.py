"""Seeded synthetic inputs for draft-tree verification.

This package only draws random numbers and lays out arrays: model weights as
bf16 bit patterns, context token ids, random KV-cache contents and draft-tree
shapes.  It contains none of the method's arithmetic and imports neither the
CPU oracle nor the GPU library; both consume its outputs.  `logits` holds
the seeded logit rows of the distillation-loss kernel.
"""
from .model import (ModelDims, TINY, V7B, V13B, bf16_bits_from_f32,
                    f32_from_bf16_bits, normal_bf16, layer_weights,
                    final_weights, adapter_weights, embedding, random_kv_context,
                    context_tokens, random_hidden, MATRIX_IDS)
from .trees import (chain_tree, complete_binary_tree, random_tree,
                    product_tree_pruned, chain_with_corrections,
                    distinct_sibling_tokens, is_valid_tree,
                    all_parent_arrays, relabel_topological)
from .logits import lm_like_logits, special_rows, position_mask

__all__ = [n for n in dir() if not n.startswith("_")]
