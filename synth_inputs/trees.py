"""Draft-tree shapes and contemplate-row placement (pure index bookkeeping).

A tree is a parent array over its rows: parent[0] = -1 (the root, i.e. the last
committed token) and parent[i] < i for every other row, so rows are listed in
the order the draft model proposed them and the children of a node, read in
increasing row index, are in proposal order.
"""
from __future__ import annotations

import numpy as np

KIND_NODE = 0
KIND_CONTEMPLATE = 1


def depths_of(parent: np.ndarray) -> np.ndarray:
    d = np.zeros(len(parent), dtype=np.int32)
    for i in range(1, len(parent)):
        d[i] = d[parent[i]] + 1
    return d


def random_tree(rng: np.random.Generator, T: int, max_depth: int, max_children: int) -> np.ndarray:
    """T-node tree grown by attaching each new node to a uniformly chosen
    existing node that still has depth < max_depth and fewer than max_children
    children (depth = number of edges from the root)."""
    if T < 1:
        raise ValueError("a tree has at least its root")
    parent = np.full(T, -1, dtype=np.int32)
    depth = np.zeros(T, dtype=np.int32)
    nchild = np.zeros(T, dtype=np.int32)
    for i in range(1, T):
        ok = np.flatnonzero((depth[:i] < max_depth) & (nchild[:i] < max_children))
        if ok.size == 0:
            raise ValueError("tree budget cannot be met with these limits")
        p = int(ok[rng.integers(0, ok.size)])
        parent[i] = p
        depth[i] = depth[p] + 1
        nchild[p] += 1
    return parent


def tiny_tree_root3(rng: np.random.Generator, T: int = 7) -> np.ndarray:
    """The tiny fp32 case: a root with exactly 3 children and depth exactly 3;
    whatever nodes remain are attached at random below the root's children."""
    if T < 6:
        raise ValueError("needs at least 6 nodes for 3 children and depth 3")
    parent = np.full(T, -1, dtype=np.int32)
    parent[1:4] = 0
    parent[4] = int(rng.integers(1, 4))   # depth 2
    parent[5] = 4                          # depth 3
    depth = depths_of(parent[:6]).tolist()
    for i in range(6, T):
        ok = [j for j in range(1, i) if depth[j] < 3]   # never the root: it keeps 3 children
        p = int(ok[rng.integers(0, len(ok))])
        parent[i] = p
        depth.append(depth[p] + 1)
    return parent


def chain_tree(T: int) -> np.ndarray:
    """Degenerate tree: every node has one child (linear speculation)."""
    return np.arange(-1, T - 1, dtype=np.int32)


def append_contemplates_chained(parent_nodes: np.ndarray, C: int, anchor: int = 0):
    """Rows [0, T) are the draft nodes; C contemplate rows are appended after
    them, the first hanging off `anchor`, each next one off the previous
    contemplate row (so they see the anchor's path and each other causally).

    Returns (parent[M], kind[M], con_anchor[C]).
    """
    T = len(parent_nodes)
    parent = np.concatenate([parent_nodes.astype(np.int32), np.zeros(C, dtype=np.int32)])
    kind = np.concatenate([np.zeros(T, dtype=np.uint8), np.ones(C, dtype=np.uint8)])
    for c in range(C):
        parent[T + c] = anchor if c == 0 else T + c - 1
    con_anchor = np.full(C, anchor, dtype=np.int32)
    return parent, kind, con_anchor


def interleave_contemplates_per_node(parent_nodes: np.ndarray):
    """The paper's verification layout (Section 3.1, Figure 4): one contemplate
    row inserted right after each draft node, 2T rows in all.  Row 2i is node i,
    row 2i+1 its contemplate row, whose parent is row 2i.

    Returns (parent[2T], kind[2T], con_anchor[T], node_rows[T]).
    """
    T = len(parent_nodes)
    parent = np.empty(2 * T, dtype=np.int32)
    kind = np.empty(2 * T, dtype=np.uint8)
    for i in range(T):
        p = int(parent_nodes[i])
        parent[2 * i] = -1 if p < 0 else 2 * p
        kind[2 * i] = KIND_NODE
        parent[2 * i + 1] = 2 * i
        kind[2 * i + 1] = KIND_CONTEMPLATE
    con_anchor = np.arange(T, dtype=np.int32)
    node_rows = np.arange(0, 2 * T, 2, dtype=np.int32)
    return parent, kind, con_anchor, node_rows
