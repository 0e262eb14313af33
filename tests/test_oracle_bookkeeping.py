"""Pins of the bookkeeping oracle (oracle/bookkeeping.py): the KV commit of the accepted path
(Section 2, step 3; Section 3.1) and the mixture-of-experts contemplate embedding (Section 3.2),
against hand-written examples, library routines and the attention oracle."""
import numpy as np
import pytest
from scipy.special import softmax as scipy_softmax

import oracle
from oracle import bookkeeping as bk
from synth_inputs import trees


def _labelled_pool(L, rows, Hkv, D):
    """Every (layer, row, head) holds its own coordinates, so a moved row can be recognised."""
    k = np.zeros((L, rows, Hkv, D))
    for l in range(L):
        for r in range(rows):
            for g in range(Hkv):
                k[l, r, g, :] = 1000 * l + 10 * r + g
    return k, -k


def test_commit_hand_example_appended_layout():
    """P = 5, T = 7 nodes followed by 2 contemplate rows (M = 9).  Accepted path 0 -> 2 -> 5: the cache must
    end with the old rows 5 (node 0), 7 (node 2), 10 (node 5) at rows 5, 6, 7.  Written out by hand."""
    L, P, M, Hkv, D = 2, 5, 9, 2, 4
    k, v = _labelled_pool(L, P + M, Hkv, D)
    path = np.array([[0, 2, 5, -1, -1, -1, -1]], dtype=np.int32)
    nk, nv, nl, st = bk.commit_kv(k, v, [0], [P], path, [2], None, M)
    assert st[0] == 0 and nl[0] == 8
    for l in range(L):
        for g in range(Hkv):
            assert nk[l, 5, g, 0] == 1000 * l + 10 * 5 + g
            assert nk[l, 6, g, 0] == 1000 * l + 10 * 7 + g
            assert nk[l, 7, g, 0] == 1000 * l + 10 * 10 + g
            assert nv[l, 7, g, 0] == -(1000 * l + 10 * 10 + g)
    assert np.array_equal(nk[:, :5], k[:, :5])          # the prefix is untouched
    assert np.array_equal(nk[:, 8:], k[:, 8:])          # rows behind the new end are left as they were


def test_commit_hand_example_interleaved_layout_and_overlapping_moves():
    """One contemplate row after each node (node i is new row 2i).  Path 0 -> 1 -> 2: sources are new rows
    0, 2, 4 and destinations 0, 1, 2 - destination 2 is the source of the second move, so every copy must read
    the old cache."""
    L, P, T, Hkv, D = 1, 3, 4, 1, 2
    M = 2 * T
    k, v = _labelled_pool(L, P + M, Hkv, D)
    node_row = np.arange(0, 2 * T, 2, dtype=np.int32)[None]
    path = np.array([[0, 1, 2, -1]], dtype=np.int32)
    nk, _, nl, st = bk.commit_kv(k, v, [0], [P], path, [2], node_row, M)
    assert st[0] == 0 and nl[0] == P + 3
    assert [nk[0, P + j, 0, 0] for j in range(3)] == [10 * (P + 0), 10 * (P + 2), 10 * (P + 4)]


def test_commit_full_chain_acceptance_is_a_no_op():
    T, P = 6, 4
    k, v = _labelled_pool(2, P + T, 2, 4)
    path = np.arange(T, dtype=np.int32)[None]
    nk, nv, nl, st = bk.commit_kv(k, v, [0], [P], path, [T - 1], None, T)
    assert np.array_equal(nk, k) and np.array_equal(nv, v) and nl[0] == P + T and st[0] == 0


def test_commit_rejects_malformed_paths_and_skips_failed_sequences():
    T, P = 5, 2
    k, v = _labelled_pool(1, 3 * (P + T), 1, 2)
    off = [0, P + T, 2 * (P + T)]
    path = np.array([[0, 3, 2, -1, -1], [1, 2, -1, -1, -1], [0, 1, -1, -1, -1]], dtype=np.int32)
    nk, _, nl, st = bk.commit_kv(k, v, off, [P] * 3, path, [2, 1, -1], None, T)
    assert st[0] == bk.STATUS_BAD_PATH and st[1] == bk.STATUS_BAD_PATH and st[2] == 0
    assert np.array_equal(nk, k) and list(nl) == [P, P, P]


def test_commit_rejects_a_row_map_that_puts_a_child_before_its_parent():
    """The rows of a path are parent and child rows of the tree the attention ran over, so they increase along it;
    a map that swaps two of them is flagged and nothing moves, the identity and the interleaved map pass."""
    T, P, M = 4, 3, 8
    k, v = _labelled_pool(1, P + M, 1, 2)
    path = np.array([[0, 1, 3, -1]], dtype=np.int32)
    for rows, ok in (([0, 2, 4, 6], True), ([0, 1, 2, 3], True), ([0, 6, 4, 2], False), ([0, 2, 4, 2], False)):
        nk, _, nl, st = bk.commit_kv(k, v, [0], [P], path, [2], np.array([rows], dtype=np.int32), M)
        assert (st[0] == 0) == ok and nl[0] == (P + 3 if ok else P)
        if not ok:
            assert np.array_equal(nk, k)


def test_committed_cache_reproduces_the_accepted_nodes_attention():
    """Ties the commit to the attention oracle: the last accepted node attended to the prefix and to its own
    path under the tree mask; plain causal attention of the same query over the committed cache (prefix +
    accepted rows, nothing else) must give the same output."""
    rng = np.random.default_rng(5)
    T, P, Hq, Hkv, D = 12, 20, 4, 2, 8
    parent_nodes = trees.random_tree(rng, T, 4, 3)
    parent, kind, _ = trees.append_contemplates_chained(parent_nodes, 2, anchor=0)
    M = len(parent)
    q = rng.standard_normal((M, Hq, D))
    k = rng.standard_normal((P + M, Hkv, D))
    v = rng.standard_normal((P + M, Hkv, D))
    ref = oracle.tree_attention(q, k, v, parent, kind, soft_len=0, scale=0.3)
    # a root-to-node path
    node = T - 1
    path = [node]
    while parent_nodes[path[-1]] >= 0:
        path.append(int(parent_nodes[path[-1]]))
    path = path[::-1]
    prow = np.full((1, T), -1, dtype=np.int32)
    prow[0, :len(path)] = path
    nk, nv, nl, st = bk.commit_kv(k[None], v[None], [0], [P], prow, [len(path) - 1], None, M)
    assert st[0] == 0
    Lc = int(nl[0])
    for h in range(Hq):
        g = h // (Hq // Hkv)
        s = 0.3 * nk[0, :Lc, g] @ q[node, h]
        w = np.exp(s - s.max())
        w /= w.sum()
        assert np.allclose(w @ nv[0, :Lc, g], ref[node, h], atol=1e-12)


def test_gather_future_picks_the_selected_contemplate_row():
    hidden = np.arange(2 * 6 * 3, dtype=np.float64).reshape(2, 6, 3)
    con_row = np.array([[4, 5], [1, 3]], dtype=np.int32)
    f = bk.gather_future(hidden, con_row, [1, -1])
    assert np.array_equal(f[0], hidden[0, 5]) and np.all(f[1] == 0)


# ---- mixture-of-experts embedding -----------------------------------------------------------------------
def test_embed_hand_example():
    """Two experts, logits (ln 3, 0): scores (3/4, 1/4).  K = 1 keeps expert 0 with weight 3/4 (not 1)."""
    h = np.array([[1.0, 0.0]])
    w = np.array([[np.log(3.0), 5.0], [0.0, -2.0]])
    e = np.array([[4.0, 8.0], [100.0, 100.0]])
    out, g, ch = bk.contemplate_embed(h, w, e, 1)
    assert np.allclose(g, [[0.75, 0.25]]) and ch[0, 0] == 0
    assert np.allclose(out, [[3.0, 6.0]])
    out2, _, ch2 = bk.contemplate_embed(h, w, e, 2)
    assert np.allclose(out2, [[3.0 + 25.0, 6.0 + 25.0]]) and list(ch2[0]) == [0, 1]


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_embed_all_experts_equals_library_softmax_times_embeddings(seed):
    rng = np.random.default_rng(seed)
    B, d_in, d_out, n = 3, 40, 24, 7
    h, w, e = rng.standard_normal((B, d_in)), rng.standard_normal((n, d_in)), rng.standard_normal((n, d_out))
    out, g, ch = bk.contemplate_embed(h, w, e, n)
    g_ref = scipy_softmax(h @ w.T, axis=1)
    assert np.allclose(g, g_ref, atol=1e-14) and np.allclose(out, g_ref @ e, atol=1e-12)
    for b in range(B):
        assert list(ch[b]) == list(np.argsort(-g_ref[b], kind="stable"))


def test_embed_top_k_matches_sorting_and_ties_take_the_lowest_index():
    rng = np.random.default_rng(9)
    B, d_in, d_out, n, k = 4, 16, 8, 10, 3
    h, w, e = rng.standard_normal((B, d_in)), rng.standard_normal((n, d_in)), rng.standard_normal((n, d_out))
    w[7] = w[2]                                         # experts 2 and 7 always tie
    out, g, ch = bk.contemplate_embed(h, w, e, k)
    for b in range(B):
        order = sorted(range(n), key=lambda x: (-g[b, x], x))[:k]
        assert list(ch[b]) == order
        assert np.allclose(out[b], sum(g[b, x] * e[x] for x in order))
        if 7 in ch[b]:
            assert 2 in ch[b] and list(ch[b]).index(2) < list(ch[b]).index(7)
    assert np.all(g.sum(axis=1) > 0.999999)
