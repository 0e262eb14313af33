"""Seeded synthetic inputs for the tree-verification workloads.

This module only draws random numbers, lays out arrays and converts number
formats.  It holds none of the verification method's arithmetic (no attention,
no masks, no softmax, no acceptance rule), so that both the CPU oracle and the
HIP library can be fed bit-identical inputs from one place without sharing any
of the method's code.

Notation follows the paper (Section 3.1): T draft-tree nodes, C contemplate
rows, M = T + C query rows, P cached prefix length of which the first s rows
are soft-prompt slots, V vocabulary size.
"""
from .trees import (
    random_tree,
    tiny_tree_root3,
    chain_tree,
    append_contemplates_chained,
    interleave_contemplates_per_node,
)
from .tensors import (
    f32_to_bf16_bits,
    bf16_bits_to_f32,
    AttnInputs,
    AcceptInputs,
    make_attention_inputs,
    make_accept_inputs,
)
from .workloads import WORKLOADS, Workload, attention_case, accept_case

__all__ = [
    "random_tree",
    "tiny_tree_root3",
    "chain_tree",
    "append_contemplates_chained",
    "interleave_contemplates_per_node",
    "f32_to_bf16_bits",
    "bf16_bits_to_f32",
    "AttnInputs",
    "AcceptInputs",
    "make_attention_inputs",
    "make_accept_inputs",
    "WORKLOADS",
    "Workload",
    "attention_case",
    "accept_case",
]
