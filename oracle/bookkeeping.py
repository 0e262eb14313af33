"""CPU oracle for the two small steps around the verification pass: committing the accepted
path to the KV cache, and the mixture-of-experts embedding of a contemplate token.

TEST INFRASTRUCTURE ONLY (imported by tests/ and the smoke check).  Plain numpy / Python loops
in the order of the definitions; fp64 for the arithmetic.  Shares no code with the GPU library.

What it follows:
 - commit: a rejected draft token and everything after it are discarded, the longest accepted
   path of the tree is kept (paper, Section 2, step 3 and the tree-of-candidates paragraph); the
   future prediction handed to the next drafting round is the one of the last accepted token
   (Section 3.1).
 - embedding: a linear layer maps the hidden state of the most recently accepted token to
   logits over the experts, a softmax normalises them, the top K experts are selected and their
   embeddings are combined with those softmax scores as weights (Section 3.2).
"""
from __future__ import annotations

import numpy as np

STATUS_BAD_PATH = 32


def path_is_valid(path_row, n_accepted: int, node_row_row, T: int, M: int) -> bool:
    """A path is the root followed by strictly increasing node indices (a child's index exceeds its
    parent's); every node must map to one of this step's M rows, and these rows increase along the
    path too: the rows are the ones the tree attention of the step ran over, where a row comes after
    its parent's row (Section 2, tree attention), and consecutive path entries are parent and child."""
    if n_accepted + 1 > T:
        return False
    prev = prev_row = -1
    for j in range(n_accepted + 1):
        node = int(path_row[j])
        if node < 0 or node >= T or node <= prev:
            return False
        if j == 0 and node != 0:
            return False
        row = node if node_row_row is None else int(node_row_row[node])
        if row < 0 or row >= M or row <= prev_row:
            return False
        prev, prev_row = node, row
    return True


def commit_kv(k_pool: np.ndarray, v_pool: np.ndarray, kv_offset, prefix_len, path, n_accepted, node_row, M: int):
    """k_pool, v_pool: [L, rows, Hkv, D].  Returns (new_k, new_v, new_prefix_len, status): for every
    layer and sequence the rows of the accepted path's nodes are copied, in path order, to the rows
    right behind the old prefix.  All copies read the OLD pool."""
    B, T = path.shape
    new_k, new_v = k_pool.copy(), v_pool.copy()
    new_len = np.array(prefix_len, dtype=np.int32).copy()
    status = np.zeros(B, dtype=np.int32)
    for b in range(B):
        n = int(n_accepted[b])
        if n < 0:
            continue
        nr = None if node_row is None else node_row[b]
        if not path_is_valid(path[b], n, nr, T, M):
            status[b] = STATUS_BAD_PATH
            continue
        base = int(kv_offset[b]) + int(prefix_len[b])
        for j in range(n + 1):
            node = int(path[b, j])
            src = base + (node if nr is None else int(nr[node]))
            dst = base + j
            for l in range(k_pool.shape[0]):
                new_k[l, dst] = k_pool[l, src]
                new_v[l, dst] = v_pool[l, src]
        new_len[b] = int(prefix_len[b]) + n + 1
    return new_k, new_v, new_len, status


def gather_future(hidden: np.ndarray, con_row, selected_con):
    """hidden [B, M, d]: f[b] = hidden[b, con_row[b][selected_con[b]]], zeros when nothing is selected."""
    B, _, d = hidden.shape
    f = np.zeros((B, d), dtype=hidden.dtype)
    for b in range(B):
        c = int(selected_con[b])
        if c >= 0:
            f[b] = hidden[b, int(con_row[b][c])]
    return f


def contemplate_embed(h: np.ndarray, router_w: np.ndarray, expert_emb: np.ndarray, k_expert: int):
    """h [B, d_in], router_w [n_expert, d_in], expert_emb [n_expert, d_out] (any float type; widened to
    fp64).  Returns (out [B, d_out], gates [B, n_expert], chosen [B, k_expert])."""
    h = np.asarray(h, dtype=np.float64)
    w = np.asarray(router_w, dtype=np.float64)
    e = np.asarray(expert_emb, dtype=np.float64)
    B, n_expert = h.shape[0], w.shape[0]
    out = np.zeros((B, e.shape[1]))
    gates = np.zeros((B, n_expert))
    chosen = np.zeros((B, k_expert), dtype=np.int32)
    for b in range(B):
        logits = np.array([float(np.dot(w[x], h[b])) for x in range(n_expert)])
        ex = np.exp(logits - logits.max())
        g = ex / ex.sum()
        gates[b] = g
        left = list(range(n_expert))
        for r in range(k_expert):               # the K largest scores, best first, lowest index on ties
            best = left[0]
            for x in left[1:]:
                if g[x] > g[best]:
                    best = x
            left.remove(best)
            chosen[b, r] = best
            out[b] += g[best] * e[best]
    return out, gates, chosen
