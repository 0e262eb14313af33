"""Pins of the attention oracle against things other than itself: library causal
attention, per-path brute force, closed forms and invariants (CPU only)."""
import json
import os

import numpy as np
import pytest
import torch

import oracle
from synth_inputs import trees

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rand_case(seed, M_nodes, C, Hq, Hkv, D, P, s=0, interleaved=False, max_depth=4, max_children=3):
    rng = np.random.default_rng(seed)
    pn = trees.random_tree(rng, M_nodes, max_depth, max_children)
    if interleaved:
        parent, kind, _, _ = trees.interleave_contemplates_per_node(pn)
    else:
        parent, kind, _ = trees.append_contemplates_chained(pn, C, anchor=int(rng.integers(0, M_nodes)) if C else 0)
    M = len(parent)
    q = rng.standard_normal((M, Hq, D))
    k = rng.standard_normal((P + M, Hkv, D))
    v = rng.standard_normal((P + M, Hkv, D))
    return parent, kind, q, k, v


def _path_rows(parent, i):
    rows = []
    j = i
    while j >= 0:
        rows.append(j)
        j = int(parent[j])
    return sorted(rows)


def _softmax_attend(qvec, K, V, scale):
    """Unmasked single-query attention over the given keys (textbook form)."""
    sc = scale * (K @ qvec)
    w = np.exp(sc - sc.max())
    w /= w.sum()
    return w @ V, sc.max() + np.log(np.exp(sc - sc.max()).sum())


def test_row_count_identities_from_paper():
    """Section 3.1: prefill context t+s+1, verification processes 2T rows."""
    with open(os.path.join(GOLDEN, "paper_row_counts.json")) as f:
        g = json.load(f)
    for ex in g["examples"]:
        t, s, T = ex["t"], ex["s"], ex["T"]
        # prefill: one root row plus one contemplate row on top of s + t cached rows: the
        # contemplate row sees everything cached, the root and itself
        parent, kind, _ = trees.append_contemplates_chained(np.array([-1], dtype=np.int32), 1)
        vis = oracle.visibility_matrix(parent, kind, P=s + t - 1, s=s)   # root = last prompt token
        assert int(vis[1].sum()) == ex["prefill_context"]
        # verification: one contemplate per node
        pn = trees.random_tree(np.random.default_rng(T), T, 8, 8)
        parent, kind, con_anchor, node_rows = trees.interleave_contemplates_per_node(pn)
        assert len(parent) == ex["verify_rows"] == 2 * T
        assert int(kind.sum()) == T


def test_single_node_is_plain_decode_attention():
    """T=1, C=0: the only row attends to all P cached rows and itself."""
    rng = np.random.default_rng(3)
    Hq, Hkv, D, P = 8, 2, 64, 50
    q = rng.standard_normal((1, Hq, D))
    k = rng.standard_normal((P + 1, Hkv, D))
    v = rng.standard_normal((P + 1, Hkv, D))
    scale = 1.0 / np.sqrt(D)
    out, lse = oracle.tree_attention(q, k, v, [-1], [0], soft_len=0, scale=scale, return_lse=True)
    G = Hq // Hkv
    for h in range(Hq):
        ref, ref_lse = _softmax_attend(q[0, h], k[:, h // G], v[:, h // G], scale)
        np.testing.assert_allclose(out[0, h], ref, rtol=0, atol=1e-13)
        assert abs(lse[h, 0] - ref_lse) < 1e-12
    # and against the library's causal attention on the full sequence, last row
    tq = torch.from_numpy(np.concatenate([np.zeros((P, Hq, D)), q])).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None].repeat_interleave(G, dim=1)
    tv = torch.from_numpy(v).permute(1, 0, 2)[None].repeat_interleave(G, dim=1)
    sd = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    np.testing.assert_allclose(out[0], sd[0, :, -1].numpy(), rtol=0, atol=1e-13)


@pytest.mark.parametrize("Hq,Hkv", [(8, 2), (6, 2), (4, 4)])
def test_chain_tree_is_causal_attention(Hq, Hkv):
    """parent[i] = i-1: the last M rows of ordinary causal attention over P+M tokens,
    computed by the library routine (heads expanded the grouped-query way)."""
    rng = np.random.default_rng(11)
    D, P, M = 32, 37, 9
    G = Hq // Hkv
    q = rng.standard_normal((M, Hq, D))
    k = rng.standard_normal((P + M, Hkv, D))
    v = rng.standard_normal((P + M, Hkv, D))
    scale = 0.2
    out = oracle.tree_attention(q, k, v, trees.chain_tree(M), np.zeros(M, np.uint8), soft_len=0, scale=scale)
    tq = torch.from_numpy(np.concatenate([rng.standard_normal((P, Hq, D)), q])).permute(1, 0, 2)[None]
    tk = torch.from_numpy(k).permute(1, 0, 2)[None].repeat_interleave(G, dim=1)
    tv = torch.from_numpy(v).permute(1, 0, 2)[None].repeat_interleave(G, dim=1)
    sd = torch.nn.functional.scaled_dot_product_attention(tq, tk, tv, is_causal=True, scale=scale)
    ref = sd[0, :, P:].permute(1, 0, 2).numpy()
    np.testing.assert_allclose(out, ref, rtol=0, atol=1e-13)


@pytest.mark.parametrize("seed,interleaved,s", [(0, False, 0), (1, False, 5), (2, True, 0), (3, True, 16)])
def test_per_path_brute_force(seed, interleaved, s):
    """Row by row: gather exactly the keys on the row's own path (plus the cached rows
    it may see) and run unmasked attention."""
    Hq, Hkv, D, P = 4, 2, 16, 40
    parent, kind, q, k, v = _rand_case(seed, 11, 3, Hq, Hkv, D, P, s, interleaved)
    M = len(parent)
    scale = 1.0 / np.sqrt(D)
    out, lse = oracle.tree_attention(q, k, v, parent, kind, soft_len=s, scale=scale, return_lse=True)
    G = Hq // Hkv
    for i in range(M):
        first = 0 if kind[i] == 1 else s
        keys = list(range(first, P)) + [P + j for j in _path_rows(parent, i)]
        for h in range(Hq):
            ref, ref_lse = _softmax_attend(q[i, h], k[keys, h // G], v[keys, h // G], scale)
            np.testing.assert_allclose(out[i, h], ref, rtol=0, atol=1e-12)
            assert abs(lse[h, i] - ref_lse) < 1e-12


def test_zero_query_gives_mean_of_visible_values_and_counts():
    """Q = 0 makes every visible weight 1/|vis(i)|; |vis(i)| = P - s*[node] + depth(i) + 1.
    Checks the visible SET, not just the arithmetic."""
    Hq, Hkv, D, P, s = 2, 1, 8, 30, 7
    parent, kind, q, k, v = _rand_case(5, 12, 4, Hq, Hkv, D, P, s)
    M = len(parent)
    q[:] = 0.0
    out, lse = oracle.tree_attention(q, k, v, parent, kind, soft_len=s, scale=1.0, return_lse=True)
    depth = trees.depths_of(parent)
    for i in range(M):
        n_vis = P - (s if kind[i] == 0 else 0) + depth[i] + 1
        assert abs(np.exp(lse[0, i]) - n_vis) < 1e-9
        first = 0 if kind[i] == 1 else s
        keys = list(range(first, P)) + [P + j for j in _path_rows(parent, i)]
        assert len(keys) == n_vis
        np.testing.assert_allclose(out[i, 0], v[keys, 0].mean(axis=0), rtol=0, atol=1e-13)


def test_indicator_values_expose_individual_weights():
    """V[k] = one-hot(k) (D >= number of keys): the output IS the weight vector, which must
    be zero off the path, positive on it and sum to one."""
    Hq, Hkv, P = 2, 2, 6
    parent, kind, q, k, v = _rand_case(8, 7, 2, Hq, Hkv, 4, P)
    M = len(parent)
    L = P + M
    qd = np.random.default_rng(1).standard_normal((M, Hq, L))
    kd = np.random.default_rng(2).standard_normal((L, Hkv, L))
    vd = np.zeros((L, Hkv, L))
    for t in range(L):
        vd[t, :, t] = 1.0
    out = oracle.tree_attention(qd, kd, vd, parent, kind, soft_len=0, scale=0.3)
    vis = oracle.visibility_matrix(parent, kind, P, 0)
    for i in range(M):
        for h in range(Hq):
            w = out[i, h]
            assert abs(w.sum() - 1.0) < 1e-13
            assert np.all(w[vis[i] == 0] == 0.0)
            assert np.all(w[vis[i] == 1] > 0.0)
            sc = 0.3 * kd[:, h] @ qd[i, h]
            ref = np.where(vis[i] == 1, np.exp(sc - sc[vis[i] == 1].max()), 0.0)
            np.testing.assert_allclose(w, ref / ref.sum(), rtol=0, atol=1e-14)


def test_equal_values_pass_through():
    parent, kind, q, k, v = _rand_case(9, 10, 3, 4, 2, 8, 20)
    row = np.arange(8, dtype=np.float64) - 3.5
    v[:] = row
    out = oracle.tree_attention(q, k, v, parent, kind, soft_len=0, scale=0.5)
    np.testing.assert_allclose(out, np.broadcast_to(row, out.shape), rtol=0, atol=1e-13)


def test_invisible_keys_do_not_matter_bitwise():
    """Changing K/V of any key a row cannot see leaves that row bit-identical."""
    Hq, Hkv, D, P, s = 4, 2, 16, 25, 4
    parent, kind, q, k, v = _rand_case(21, 13, 3, Hq, Hkv, D, P, s)
    M = len(parent)
    base = oracle.tree_attention(q, k, v, parent, kind, soft_len=s, scale=0.25)
    vis = oracle.visibility_matrix(parent, kind, P, s)
    rng = np.random.default_rng(99)
    for i in range(M):
        k2, v2 = k.copy(), v.copy()
        hidden = np.flatnonzero(vis[i] == 0)
        assert hidden.size > 0
        k2[hidden] = rng.standard_normal((hidden.size, Hkv, D)) * 50
        v2[hidden] = rng.standard_normal((hidden.size, Hkv, D)) * 50
        out = oracle.tree_attention(q, k2, v2, parent, kind, soft_len=s, scale=0.25)
        assert np.array_equal(out[i], base[i])
    # and a visible key does matter
    k2 = k.copy()
    k2[P] += 1.0      # the root is on every path
    assert not np.array_equal(oracle.tree_attention(q, k2, v, parent, kind, soft_len=s, scale=0.25), base)


def test_soft_prompts_touch_contemplate_rows_only():
    """Section 3.1: only contemplate rows attend to the soft-prompt slots."""
    Hq, Hkv, D, P = 4, 2, 16, 30
    parent, kind, q, k, v = _rand_case(31, 9, 3, Hq, Hkv, D, P)
    M = len(parent)
    s = 16
    with_s = oracle.tree_attention(q, k, v, parent, kind, soft_len=s, scale=0.25)
    # the same rows with the first s cache rows removed: what a model without soft prompts sees
    without = oracle.tree_attention(q, k[s:], v[s:], parent, kind, soft_len=0, scale=0.25)
    nodes = np.flatnonzero(kind == 0)
    cons = np.flatnonzero(kind == 1)
    np.testing.assert_allclose(with_s[nodes], without[nodes], rtol=0, atol=1e-14)
    assert np.abs(with_s[cons] - without[cons]).max() > 1e-3


def test_relabelling_siblings_permutes_outputs():
    """Outputs follow the rows: renumbering rows (keeping parents before children) permutes them."""
    Hq, Hkv, D, P = 2, 1, 8, 10
    parent = np.array([-1, 0, 0, 1, 2, 2], dtype=np.int32)
    kind = np.zeros(6, np.uint8)
    rng = np.random.default_rng(4)
    q = rng.standard_normal((6, Hq, D))
    k = rng.standard_normal((P + 6, Hkv, D))
    v = rng.standard_normal((P + 6, Hkv, D))
    base = oracle.tree_attention(q, k, v, parent, kind, soft_len=0, scale=0.3)
    perm = np.array([0, 2, 1, 4, 5, 3])      # new row r holds old row perm[r]
    inv = np.argsort(perm)
    parent2 = np.array([-1 if parent[o] < 0 else inv[parent[o]] for o in perm], dtype=np.int32)
    assert all(parent2[i] < i for i in range(6))
    k2, v2 = k.copy(), v.copy()
    k2[P:], v2[P:] = k[P:][perm], v[P:][perm]
    out = oracle.tree_attention(q[perm], k2, v2, parent2, kind, soft_len=0, scale=0.3)
    np.testing.assert_allclose(out, base[perm], rtol=0, atol=1e-13)


def test_contemplate_rows_are_invisible_to_nodes_and_other_branches():
    pn = np.array([-1, 0, 0, 1], dtype=np.int32)
    parent, kind, _, rows = trees.interleave_contemplates_per_node(pn)
    anc = oracle.ancestor_matrix(parent, kind)
    for i in range(len(parent)):
        for j in range(len(parent)):
            if kind[j] == 1 and j != i:
                assert anc[i, j] == 0      # nobody but itself sees a per-node contemplate row
    # chained contemplates see each other causally
    parent, kind, _ = trees.append_contemplates_chained(pn, 3, anchor=1)
    anc = oracle.ancestor_matrix(parent, kind)
    assert anc[6].tolist() == [1, 1, 0, 0, 1, 1, 1]


@pytest.mark.parametrize("parent,kind", [
    ([-1, 1], [0, 0]),          # self parent
    ([-1, 2, 0], [0, 0, 0]),    # forward reference
    ([-2, 0], [0, 0]),
    ([-1, 0, 1], [0, 1, 0]),    # draft node hanging off a contemplate row
    ([-1, 0], [0, 2]),          # unknown kind
])
def test_malformed_trees_are_rejected(parent, kind):
    with pytest.raises(oracle.OracleError):
        oracle.ancestor_matrix(parent, kind)


def test_scale_and_gqa_mapping_matter():
    """Guards against a silently ignored scale or a wrong head-to-KV-head map: distinct KV
    heads, compare against explicitly expanded heads."""
    rng = np.random.default_rng(17)
    Hq, Hkv, D, P = 6, 3, 8, 12
    parent, kind, q, k, v = _rand_case(17, 8, 2, Hq, Hkv, D, P)
    out = oracle.tree_attention(q, k, v, parent, kind, soft_len=0, scale=0.7)
    kx = np.repeat(k, Hq // Hkv, axis=1)     # head h uses kv head h // G
    vx = np.repeat(v, Hq // Hkv, axis=1)
    out_x = oracle.tree_attention(q, kx, vx, parent, kind, soft_len=0, scale=0.7)
    np.testing.assert_allclose(out, out_x, rtol=0, atol=0)
    assert np.abs(out - oracle.tree_attention(q, k, v, parent, kind, soft_len=0, scale=0.1)).max() > 1e-3
