"""The synthetic workloads (shapes of the paper's evaluation: Llama-3.2-3B,
Llama-3.1-8B and Qwen3-4B targets, 60-node draft trees; Section 4) plus helpers that
build one attention case / one acceptance case for a workload.

Index 0 is the tiny fp32 case the CPU oracle finishes instantly; the others take
their head geometry and vocabulary from the named model families.  "N(0, x)" is
read as standard deviation x.  Seeds: 1000 + workload index for tensors, and
seed + 1 + sequence index for each sequence's tree.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

from . import tensors, trees


@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str
    B: int
    Hq: int
    Hkv: int
    D: int
    prefix: object            # int, or (lo, hi) for ragged lengths drawn per sequence
    T: int
    C: int
    max_depth: int
    max_children: int
    n_layers: int
    V: int
    logit_std: float
    qkv_std: float
    accept_modes: Sequence    # tuples (temperature, rule)
    seed: int


_SQ = 1.0 / np.sqrt(128.0)

WORKLOADS = [
    Workload("tiny-fp32", "f32", 1, 8, 2, 64, 128, 7, 2, 3, 3, 1, 1000, 2.0, 1.0,
             ((1.0, tensors.RULE_DRAFT_WOR), (1.0, tensors.RULE_DETERMINISTIC)), 1000),
    Workload("llama3.2-3b-layer", "bf16", 1, 24, 8, 128, 2048, 60, 4, 8, 8, 1, 128256, 3.0, _SQ,
             ((1.0, tensors.RULE_DRAFT_WOR),), 1001),
    Workload("llama3.1-8b-32layers", "bf16", 1, 32, 8, 128, 4096, 60, 4, 8, 8, 32, 128256, 3.0, _SQ,
             ((0.0, tensors.RULE_GREEDY), (1.0, tensors.RULE_DETERMINISTIC)), 1002),
    Workload("llama3.1-8b-batch8-ragged", "bf16", 8, 32, 8, 128, (512, 8192), 60, 4, 8, 8, 1, 128256, 3.0, _SQ,
             ((1.0, tensors.RULE_DETERMINISTIC),), 1003),
    Workload("qwen3-4b-long", "bf16", 1, 32, 8, 128, 16384, 60, 4, 10, 8, 1, 151936, 3.0, _SQ,
             ((1.0, tensors.RULE_DRAFT_WOR),), 1004),
    # the paper's own verification layout (Section 3.1): one contemplate row per draft node (C = T, 2T = 120 rows,
    # interleaved) and 16 soft-prompt slots at the head of the cache; Llama-3.1-8B head geometry
    Workload("llama3.1-8b-contemplate-per-node", "bf16", 1, 32, 8, 128, 4096 + 16, 60, 60, 8, 8, 32, 128256, 3.0, _SQ,
             ((1.0, tensors.RULE_DETERMINISTIC),), 1005),
]

PAPER_SOFT_LEN = 16      # soft-prompt slots named in Section 3.1


def _trees_for(w: Workload, B: int):
    parents = []
    for b in range(B):
        trng = np.random.default_rng(w.seed + 1 + b)
        if w.name == "tiny-fp32":
            parents.append(trees.tiny_tree_root3(trng, w.T))
        else:
            parents.append(trees.random_tree(trng, w.T, w.max_depth, w.max_children))
    return np.stack(parents)


def prefix_lengths(w: Workload) -> np.ndarray:
    if isinstance(w.prefix, tuple):
        lrng = np.random.default_rng(w.seed + 500)
        return lrng.integers(w.prefix[0], w.prefix[1] + 1, size=w.B).astype(np.int32)
    return np.full(w.B, int(w.prefix), dtype=np.int32)


def attention_case(index: int, *, layer: int = 0, soft_len: int = 0, peaked: bool = False,
                   prefix_override: Optional[object] = None) -> tensors.AttnInputs:
    """One layer's attention inputs for workload `index`.  `peaked` draws Q and K
    with unit variance so scaled scores have unit spread (a meaningful test of the
    tolerance: the default 1/sqrt(D) draws give near-uniform attention)."""
    w = WORKLOADS[index]
    node_parent = _trees_for(w, w.B)
    par, kin = [], []
    for b in range(w.B):
        if w.C == w.T:
            p, k, _, _ = trees.interleave_contemplates_per_node(node_parent[b])
        else:
            p, k, _ = trees.append_contemplates_chained(node_parent[b], w.C, anchor=0)
        par.append(p)
        kin.append(k)
    rng = np.random.default_rng([w.seed, layer, int(peaked), soft_len])
    plen = prefix_lengths(w) if prefix_override is None else np.atleast_1d(np.asarray(prefix_override, np.int32))
    std_q = 1.0 if peaked else w.qkv_std
    std_kv = 1.0 if peaked else w.qkv_std
    return tensors.make_attention_inputs(
        rng, dtype=w.dtype, Hq=w.Hq, Hkv=w.Hkv, D=w.D, prefix_len=plen,
        parent=np.stack(par), kind=np.stack(kin), soft_len=soft_len,
        q_std=std_q, kv_std=std_kv, scale=1.0 / np.sqrt(w.D),
        pool_pad_tokens=0,
    )


def accept_case(index: int, mode: int = 0, *, draft_target_corr: float = 0.0, child_boost: float = 0.0,
                V_override: Optional[int] = None) -> tensors.AcceptInputs:
    """Acceptance inputs of workload `index`.  The defaults are the plain recipe (independent
    Gaussian logits: most walks stop at the root); `draft_target_corr` and `child_boost` are the
    realism knobs that bring the accepted length into the range the paper reports (Tables 1-3)."""
    w = WORKLOADS[index]
    temperature, rule = w.accept_modes[mode]
    node_parent = _trees_for(w, w.B)
    rng = np.random.default_rng([w.seed, 77, mode])
    if w.C == w.T:      # one contemplate row per node: row c predicts the future of node c
        con_anchor = np.tile(np.arange(w.C, dtype=np.int32), (w.B, 1))
    else:               # a few contemplate rows, all anchored at the root
        con_anchor = np.zeros((w.B, w.C), dtype=np.int32)
    return tensors.make_accept_inputs(
        rng, parent=node_parent, V=int(V_override or w.V), temperature=temperature, rule=rule,
        logit_std=w.logit_std, con_anchor=con_anchor, draft_target_corr=draft_target_corr,
        child_boost=child_boost,
    )
