"""GPU parity: tree_verify_attention (HIP, through the C ABI) against the fp64 CPU oracle on
identical seeded inputs.  Tolerances (max-abs on the attention output): 1e-5 on the fp32 path,
2e-2 on the bf16 path; the bf16 cases also bound the error relative to the largest oracle
output, because the 1/sqrt(D)-scaled draws give outputs far smaller than 2e-2."""
import numpy as np
import pytest

import oracle
import synth_inputs as si
from synth_inputs import trees
from tests import harness as H

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}
# bf16 output rounding is 2^-9 relative to the value; inputs are exact; P is rounded to bf16 before
# the PV product (2^-9 relative per weight, averaging down over many keys)
REL_TOL_BF16 = 1.5e-2


def _check(inp, out, lse, status, *, seqs=None, rel=True):
    worst = 0.0
    for b in (range(inp.B) if seqs is None else seqs):
        assert status[b] == 0
        ref, ref_lse = H.oracle_attention(inp, b)
        err = np.abs(out[b] - ref).max()
        assert np.isfinite(out[b]).all()
        assert err <= TOL[inp.dtype], f"seq {b}: max-abs {err:.3e}"
        if inp.dtype == "bf16" and rel:
            assert err <= REL_TOL_BF16 * np.abs(ref).max(), f"seq {b}: {err:.3e} vs scale {np.abs(ref).max():.3e}"
        if lse is not None:
            lerr = np.abs(lse[b] - ref_lse).max()
            # bf16 path: scores come from exact bf16 inputs with fp32 accumulation and the row sums are kept in fp32
            # (only the weights handed to the PV product are rounded), so the log-sum-exp is good to fp32 level
            assert lerr <= (1e-5 * max(1.0, np.abs(ref_lse).max()) if inp.dtype == "f32" else 1e-3), f"lse err {lerr:.3e}"
        worst = max(worst, err)
    return worst


def _case(seed, *, dtype, Hq, Hkv, D, P, T, C=4, s=0, layout="appended", q_std=1.0, kv_std=1.0, B=1,
          max_depth=8, max_children=8, pad=0):
    rng = np.random.default_rng(seed)
    par, kin = [], []
    for b in range(B):
        pn = trees.random_tree(rng, T, max_depth, max_children)
        if layout == "interleaved":
            p, k, _, _ = trees.interleave_contemplates_per_node(pn)
        else:
            p, k, _ = trees.append_contemplates_chained(pn, C, anchor=int(rng.integers(0, T)))
        par.append(p)
        kin.append(k)
    return si.make_attention_inputs(rng, dtype=dtype, Hq=Hq, Hkv=Hkv, D=D, prefix_len=P, parent=np.stack(par),
                                    kind=np.stack(kin), soft_len=s, q_std=q_std, kv_std=kv_std,
                                    pool_pad_tokens=pad)


# ---- fp32 path ----------------------------------------------------------------------------------------
@pytest.mark.parametrize("s", [0, 16])
def test_tiny_fp32_workload(s):
    inp = si.attention_case(0, soft_len=s)
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st)


@pytest.mark.parametrize("D,Hq,Hkv,M_T,P", [(64, 8, 2, 29, 77), (128, 6, 2, 17, 130), (64, 4, 4, 60, 0),
                                             (128, 3, 1, 1, 5)])
def test_fp32_shapes(D, Hq, Hkv, M_T, P):
    inp = _case(5, dtype="f32", Hq=Hq, Hkv=Hkv, D=D, P=P, T=M_T, C=3, s=min(P, 3))
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st)


def test_fp32_paper_layout_two_rows_per_node():
    inp = _case(6, dtype="f32", Hq=8, Hkv=2, D=64, P=100, T=30, layout="interleaved", s=16)
    assert inp.M == 60
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st)


# ---- bf16 MFMA path -------------------------------------------------------------------------------------
@pytest.mark.parametrize("Hq,Hkv,T,C,P,s", [
    (8, 2, 60, 4, 300, 0),        # G=4, M=64: one query head per row block, ragged last tile
    (6, 2, 60, 4, 517, 16),       # G=3: three row blocks
    (8, 2, 33, 4, 200, 5),        # G*M = 148: ragged last row block, heads straddle blocks
    (4, 1, 7, 2, 64, 0),          # 36 packed rows in one block
    (8, 8, 20, 1, 1000, 40),      # G=1 (multi-head attention), soft prompts longer than a tile
    (16, 1, 5, 3, 96, 0),         # G=16
])
@pytest.mark.parametrize("peaked", [False, True])
@pytest.mark.parametrize("wg", [1, 2, 4])
def test_bf16_shapes(Hq, Hkv, T, C, P, s, peaked, wg):
    """wg = 64-row blocks sharing one key stream per workgroup (the three kernel instantiations)."""
    std = 1.0 if peaked else 1.0 / np.sqrt(128)
    inp = _case(11, dtype="bf16", Hq=Hq, Hkv=Hkv, D=128, P=P, T=T, C=C, s=s, q_std=std, kv_std=std)
    out, lse, st = H.run_attention(inp, wg_row_blocks=wg)
    _check(inp, out, lse, st)
    out, lse, st = H.run_attention(inp, wg_row_blocks=wg, num_splits=3)
    _check(inp, out, lse, st)


def test_bf16_paper_layout_120_rows_and_soft_prompts():
    """One contemplate row per node (2T = 120 rows, two mask words) and s = 16 soft-prompt slots."""
    inp = _case(12, dtype="bf16", Hq=8, Hkv=2, D=128, P=700, T=60, layout="interleaved", s=16)
    assert inp.M == 120
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st)
    inp = _case(13, dtype="bf16", Hq=4, Hkv=2, D=128, P=90, T=64, layout="interleaved", s=16)
    assert inp.M == 128
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st)


@pytest.mark.parametrize("P", [0, 1, 31, 32, 33, 160])
@pytest.mark.parametrize("splits", [0, 1, 2, 5])
def test_bf16_short_prefixes_and_forced_splits(P, splits):
    inp = _case(14 + P, dtype="bf16", Hq=8, Hkv=2, D=128, P=P, T=60, C=4, q_std=1.0, kv_std=1.0)
    for wg in (1, 2, 4):
        out, lse, st = H.run_attention(inp, num_splits=splits, wg_row_blocks=wg)
        _check(inp, out, lse, st)


def test_bf16_split_counts_agree_closely():
    inp = _case(15, dtype="bf16", Hq=8, Hkv=2, D=128, P=2048, T=60, C=4, q_std=1.0, kv_std=1.0)
    o1, l1, _ = H.run_attention(inp, num_splits=1)
    for n in (2, 3, 8, 16):
        on, ln, st = H.run_attention(inp, num_splits=n)
        _check(inp, on, ln, st)
        assert np.abs(on - o1).max() <= 2e-2


def test_bf16_ragged_batch_with_poisoned_padding():
    """Sequences of different length in one pool; the unused rows between them hold huge values,
    so any read past a sequence's last row shows up in the output."""
    inp = _case(16, dtype="bf16", Hq=8, Hkv=2, D=128, P=[70, 1, 333, 0, 129], T=20, C=3, B=5, pad=3,
                q_std=1.0, kv_std=1.0)
    big = si.f32_to_bf16_bits(np.full((3, 2, 128), 3e38, np.float32))
    for b in range(inp.B):
        end = int(inp.kv_offset[b]) + int(inp.prefix_len[b]) + inp.M
        inp.k_pool[end:end + 3] = big
        inp.v_pool[end:end + 3] = big
    for splits in (0, 1, 3):
        for wg in (1, 2, 4):
            out, lse, st = H.run_attention(inp, num_splits=splits, wg_row_blocks=wg)
            _check(inp, out, lse, st)


def test_bf16_many_sequences_and_largest_tree():
    """48 sequences in one call (the second grid dimension, the planner's many-sequence branch) and a tree of
    the largest size the library takes (128 rows: both mask words, two 64-row blocks per query head)."""
    rng = np.random.default_rng(31)
    P = [int(x) for x in rng.integers(0, 400, size=48)]
    inp = _case(31, dtype="bf16", Hq=4, Hkv=2, D=128, P=P, T=12, C=2, B=48, q_std=1.0, kv_std=1.0)
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st, seqs=range(0, 48, 5))
    inp = _case(32, dtype="bf16", Hq=4, Hkv=4, D=128, P=[150, 33], T=120, C=8, B=2, max_depth=30, max_children=3,
                q_std=1.0, kv_std=1.0)
    assert inp.M == 128
    for wg in (0, 2):
        out, lse, st = H.run_attention(inp, wg_row_blocks=wg)
        _check(inp, out, lse, st)


def test_bf16_invisible_keys_do_not_change_the_output_bitwise():
    inp = _case(17, dtype="bf16", Hq=8, Hkv=2, D=128, P=100, T=30, C=2, s=8, q_std=1.0, kv_std=1.0)
    base, _, _ = H.run_attention(inp, num_splits=2)
    vis = oracle.visibility_matrix(inp.parent[0], inp.kind[0], 100, 8)
    rng = np.random.default_rng(0)
    # change the soft-prompt slots: node rows must not move at all, contemplate rows must
    k2 = inp.k_pool.copy()
    v2 = inp.v_pool.copy()
    k2[:8] = si.f32_to_bf16_bits(rng.standard_normal((8, 2, 128)).astype(np.float32) * 4)
    v2[:8] = si.f32_to_bf16_bits(rng.standard_normal((8, 2, 128)).astype(np.float32) * 4)
    inp2 = si.AttnInputs(**{**inp.__dict__, "k_pool": k2, "v_pool": v2})
    out2, _, _ = H.run_attention(inp2, num_splits=2)
    nodes = np.flatnonzero(inp.kind[0] == 0)
    cons = np.flatnonzero(inp.kind[0] == 1)
    assert np.array_equal(out2[0, nodes], base[0, nodes])
    assert not np.array_equal(out2[0, cons], base[0, cons])
    # change one leaf's K/V: only that row may move
    leaf = max(i for i in nodes if not any(inp.parent[0][j] == i for j in range(inp.M)))
    k3, v3 = inp.k_pool.copy(), inp.v_pool.copy()
    k3[100 + leaf] = si.f32_to_bf16_bits(rng.standard_normal((2, 128)).astype(np.float32) * 4)
    v3[100 + leaf] = si.f32_to_bf16_bits(rng.standard_normal((2, 128)).astype(np.float32) * 4)
    out3, _, _ = H.run_attention(si.AttnInputs(**{**inp.__dict__, "k_pool": k3, "v_pool": v3}), num_splits=2)
    others = [i for i in range(inp.M) if vis[i, 100 + leaf] == 0]
    assert np.array_equal(out3[0, others], base[0, others])
    assert not np.array_equal(out3[0, leaf], base[0, leaf])


def test_results_are_run_to_run_identical():
    inp = _case(18, dtype="bf16", Hq=8, Hkv=2, D=128, P=900, T=60, C=4, q_std=1.0, kv_std=1.0)
    a, la, _ = H.run_attention(inp)
    b, lb, _ = H.run_attention(inp)
    assert np.array_equal(a, b) and np.array_equal(la, lb)


def test_bf16_sequences_are_served_once_whatever_their_lengths():
    """The bf16 kernel hands its workgroups to the sequences by decreasing prefix length: equal lengths, empty
    prefixes, a length outside the bound, and more sequences than a wave has lanes (served in index order) must
    each still be answered exactly once, in their own output rows."""
    import paper_2603_08899_amd as tv
    P = [64, 64, 0, 200, 64, 0, 200, 64, 1]
    inp = _case(41, dtype="bf16", Hq=4, Hkv=2, D=128, P=P, T=10, C=2, B=len(P), q_std=1.0, kv_std=1.0)
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st)
    out, lse, st = H.run_attention(inp, max_prefix_len=100)      # sequences 3 and 6 exceed the bound
    for b in range(len(P)):
        if P[b] > 100:
            assert st[b] & tv.TV_STATUS_BAD_PREFIX and np.all(out[b] == 0)
        else:
            assert st[b] == 0
    _check(inp, out, lse, st, seqs=[b for b in range(len(P)) if P[b] <= 100])
    rng = np.random.default_rng(42)
    P = [int(x) for x in rng.integers(0, 150, size=70)]
    inp = _case(42, dtype="bf16", Hq=4, Hkv=2, D=128, P=P, T=8, C=2, B=70, q_std=1.0, kv_std=1.0)
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st, seqs=range(0, 70, 7))
    assert np.all(st == 0) and np.all(np.isfinite(lse))
    # more sequences than lanes AND several key ranges (one KV head, one row block: few workgroups per sequence)
    import paper_2603_08899_amd as tv
    P = [int(x) for x in rng.integers(0, 2000, size=70)]
    inp = _case(43, dtype="bf16", Hq=1, Hkv=1, D=128, P=P, T=8, C=2, B=70, q_std=1.0, kv_std=1.0)
    assert tv.tv_attention_plan(tv.make_attn_desc(dtype=tv.TV_DTYPE_BF16, B=70, M=inp.M, Hq=1, Hkv=1, D=128, soft_len=0,
                                                  max_prefix_len=max(P), softmax_scale=inp.scale))[1] > 1
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st, seqs=range(0, 70, 9))
    assert np.all(st == 0) and np.all(np.isfinite(lse))


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
@pytest.mark.parametrize("P,s", [(16, 16), (48, 48), (64, 64), (100, 96), (33, 32), (400, 399)])
def test_soft_prompt_slots_up_to_the_whole_prefix(dtype, D, P, s):
    """soft_len up to P itself: draft nodes then see no cached row at all (only their tree ancestors), contemplate
    rows see everything; slot ranges that end inside a tile, on a tile edge, and several tiles long."""
    inp = _case(55, dtype=dtype, Hq=4, Hkv=2, D=D, P=P, T=14, C=3, s=s, q_std=1.0, kv_std=1.0)
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st)
    if dtype == "bf16":
        out, lse, st = H.run_attention(inp, max_prefix_len=4096, num_splits=4)      # the slots spread over key ranges
        _check(inp, out, lse, st)


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_pool_strides_head_major_and_padded_rows(dtype, D):
    """The same K/V values in three pool layouts - token-major (the default strides), head-major
    [Hkv][rows][D], and token-major with padded rows and padded heads - give the same output bit for bit."""
    import torch
    inp = _case(54, dtype=dtype, Hq=8, Hkv=2, D=D, P=[300, 47], T=12, C=2, B=2, q_std=1.0, kv_std=1.0)
    q = H.to_device_storage(inp.q, dtype)
    k = H.to_device_storage(inp.k_pool, dtype)            # [rows, Hkv, D]
    v = H.to_device_storage(inp.v_pool, dtype)
    rows = k.shape[0]
    ref, ref_lse, st = H.run_attention(inp, device_inputs=(q, k, v))
    _check(inp, ref, ref_lse, st)
    kh, vh = k.permute(1, 0, 2).contiguous(), v.permute(1, 0, 2).contiguous()
    out, lse, st = H.run_attention(inp, device_inputs=(q, kh, vh), kv_token_stride=D, kv_head_stride=rows * D)
    assert np.array_equal(out, ref) and np.array_equal(lse, ref_lse) and np.all(st == 0)
    hs, ts = D + 16, 2 * (D + 16) + 8                     # padded heads, padded rows (multiples of 8 elements)
    kp = torch.full((rows, ts), float("nan"), device="cuda", dtype=k.dtype)
    vp = torch.full((rows, ts), float("nan"), device="cuda", dtype=k.dtype)
    for g in range(2):
        kp[:, g * hs:g * hs + D] = k[:, g]
        vp[:, g * hs:g * hs + D] = v[:, g]
    out, lse, st = H.run_attention(inp, device_inputs=(q, kp, vp), kv_token_stride=ts, kv_head_stride=hs)
    assert np.array_equal(out, ref) and np.array_equal(lse, ref_lse) and np.all(st == 0)


@pytest.mark.parametrize("wg", [0, 1, 2, 4])
def test_bf16_fewer_tiles_than_key_streams(wg):
    """The launch is sized from max_prefix_len; a sequence far shorter than that bound leaves whole key streams, and
    whole workgroups, without a tile.  They must contribute nothing (small-magnitude scores, so that a stray
    contribution with weight 2^0 would show)."""
    import paper_2603_08899_amd as tv
    for P, bound in ((40, 4096), (0, 4096), (300, 16384), (1000, 65536)):
        inp = _case(52, dtype="bf16", Hq=8, Hkv=2, D=128, P=P, T=20, C=2, q_std=0.3, kv_std=0.3)
        out, lse, st = H.run_attention(inp, max_prefix_len=bound, wg_row_blocks=wg)
        _check(inp, out, lse, st)
    P = [40, 2000, 0, 700, 5, 64]
    inp = _case(53, dtype="bf16", Hq=8, Hkv=2, D=128, P=P, T=20, C=2, B=len(P), q_std=0.3, kv_std=0.3)
    out, lse, st = H.run_attention(inp, max_prefix_len=8192, wg_row_blocks=wg)
    _check(inp, out, lse, st)
    rb, n = tv.tv_attention_plan(tv.make_attn_desc(dtype=tv.TV_DTYPE_BF16, B=len(P), M=inp.M, Hq=8, Hkv=2, D=128,
                                                   soft_len=0, max_prefix_len=8192, softmax_scale=inp.scale,
                                                   wg_row_blocks=wg))
    assert n * (4 // rb) > (40 + inp.M + 31) // 32        # more key streams than the short sequences have tiles


def test_bf16_length_hint_changes_the_launch_not_the_answer():
    """sum_prefix_len only sizes the launch: with the true sum, with the sum of a batch of equal lengths and
    without it the outputs meet the same bound (the split of the keys may differ, so not bit for bit)."""
    import paper_2603_08899_amd as tv
    P = [700, 90, 1500, 333, 2048, 64]
    inp = _case(51, dtype="bf16", Hq=8, Hkv=2, D=128, P=P, T=16, C=2, B=len(P), q_std=1.0, kv_std=1.0)
    plans = set()
    for hint in (0, sum(P), len(P) * max(P)):
        out, lse, st = H.run_attention(inp, sum_prefix_len=hint)
        _check(inp, out, lse, st)
        plans.add(tv.tv_attention_plan(tv.make_attn_desc(dtype=tv.TV_DTYPE_BF16, B=len(P), M=inp.M, Hq=8, Hkv=2, D=128,
                                                          soft_len=0, max_prefix_len=max(P), softmax_scale=inp.scale,
                                                          sum_prefix_len=hint)))
    print("plans", plans)


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
def test_malformed_sequences_are_flagged_and_zeroed(dtype, D):
    import paper_2603_08899_amd as tv
    inp = _case(19, dtype=dtype, Hq=4, Hkv=2, D=D, P=[50, 60, 70, 80], T=10, C=2, B=4, q_std=1.0, kv_std=1.0)
    inp.parent[1, 5] = 7                 # forward reference
    inp.kind[2, 3] = 1                   # a draft node now hangs off a contemplate row (if it has children)
    kids = [j for j in range(inp.M) if inp.parent[2, j] == 3 and inp.kind[2, j] == 0]
    for splits in (1, 2):
        out, lse, st = H.run_attention(inp, num_splits=splits, max_prefix_len=75)   # sequence 3 exceeds the bound
        assert st[0] == 0
        assert st[1] & tv.TV_STATUS_BAD_PARENT
        assert (st[2] & tv.TV_STATUS_BAD_KIND) if kids else st[2] == 0
        assert st[3] & tv.TV_STATUS_BAD_PREFIX
        for b in (1, 3):
            assert np.all(out[b] == 0)
        _check(inp, out, lse, st, seqs=[0])


@pytest.mark.parametrize("dtype,D,Hq,Hkv,T,C,P,s,layout,wg,splits", [
    ("bf16", 128, 8, 2, 60, 4, [700], 0, "appended", 1, 0),
    ("bf16", 128, 8, 2, 60, 4, [700], 16, "appended", 1, 3),
    ("bf16", 128, 8, 2, 60, 60, [300], 16, "interleaved", 0, 0),          # 120 rows: both mask words
    ("bf16", 128, 6, 2, 37, 3, [0, 900, 64, 5], 0, "appended", 2, 2),
    ("bf16", 128, 4, 1, 60, 4, [2000, 100], 8, "appended", 4, 0),
    ("f32", 64, 8, 2, 20, 2, [90, 10], 4, "appended", 0, 0),               # the fp32 path builds its own masks
])
def test_prepared_tree_changes_nothing_bitwise(dtype, D, Hq, Hkv, T, C, P, s, layout, wg, splits):
    """Section 3.1 / Figure 4: the mask belongs to the step.  Handing a layer call the record tv_prepare_tree wrote
    for the same trees must give the same bits as letting the call check the trees and walk the ancestors itself."""
    inp = _case(4100 + T + len(P), dtype=dtype, Hq=Hq, Hkv=Hkv, D=D, P=P if len(P) > 1 else P[0], T=T, C=C, s=s,
                layout=layout, B=len(P))
    a = H.run_attention(inp, wg_row_blocks=wg, num_splits=splits)
    b = H.run_attention(inp, wg_row_blocks=wg, num_splits=splits, prepare=True)
    assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1]) and np.array_equal(a[2], b[2])
    _check(inp, *b)


@pytest.mark.parametrize("splits", [1, 2])
def test_prepared_malformed_trees_are_flagged_and_zeroed(splits):
    import paper_2603_08899_amd as tv
    inp = _case(23, dtype="bf16", Hq=4, Hkv=2, D=128, P=[50, 60, 70, 80], T=10, C=2, B=4)
    inp.parent[1, 5] = 7                 # forward reference
    inp.kind[2, 4] = 3                   # unknown kind
    out, lse, st = H.run_attention(inp, num_splits=splits, max_prefix_len=75, prepare=True)   # sequence 3 exceeds the bound
    assert st[0] == 0
    assert st[1] == tv.TV_STATUS_BAD_PARENT and st[2] == tv.TV_STATUS_BAD_KIND and st[3] == tv.TV_STATUS_BAD_PREFIX
    for b in (1, 2, 3):
        assert np.all(out[b] == 0) and np.all(lse[b] == 0)
    _check(inp, out, lse, st, seqs=[0])


@pytest.mark.parametrize("wg,splits", [(1, 0), (2, 3), (4, 1)])
def test_bf16_relabelling_rows_permutes_the_output(wg, splits):
    """Outputs follow the rows: renumbering the rows of a tree (parents still before children; siblings swapped,
    whole subtrees moved) only permutes the rows of the result.  Each row's keys are then met in another order and
    in other tiles, so the match is to rounding, not bitwise."""
    rng = np.random.default_rng(77)
    inp = _case(78, dtype="bf16", Hq=8, Hkv=2, D=128, P=333, T=48, C=0)
    M, P = inp.M, int(inp.prefix_len[0])
    parent = inp.parent[0]
    # a random relabelling that keeps every parent in front of its children: visit the tree with children in random order
    kids = [[] for _ in range(M)]
    for i in range(1, M):
        kids[parent[i]].append(i)
    order, stack = [], [0]
    while stack:
        x = stack.pop(int(rng.integers(0, len(stack))))       # any visited-parent-first order
        order.append(x)
        stack.extend(kids[x])
    perm = np.array(order)                                     # new row r holds old row perm[r]
    assert not np.array_equal(perm, np.arange(M))
    inv = np.argsort(perm)
    parent2 = np.array([-1 if parent[o] < 0 else inv[parent[o]] for o in perm], dtype=np.int32)
    assert all(parent2[i] < i for i in range(M))
    import dataclasses
    k2, v2 = inp.k_pool.copy(), inp.v_pool.copy()
    k2[P:P + M], v2[P:P + M] = inp.k_pool[P:P + M][perm], inp.v_pool[P:P + M][perm]
    inp2 = dataclasses.replace(inp, q=inp.q[:, perm].copy(), k_pool=k2, v_pool=v2, parent=parent2[None].copy(),
                               kind=inp.kind[:, perm].copy())
    out1, lse1, st1 = H.run_attention(inp, wg_row_blocks=wg, num_splits=splits)
    out2, lse2, st2 = H.run_attention(inp2, wg_row_blocks=wg, num_splits=splits)
    assert st1[0] == 0 and st2[0] == 0
    _check(inp2, out2, lse2, st2)
    scale = np.abs(out1).max()
    assert np.abs(out2[0] - out1[0][perm]).max() <= 2 ** -7 * scale          # two bf16 roundings apart at most
    assert np.abs(lse2[0] - lse1[0][:, perm]).max() <= 1e-4


@pytest.mark.parametrize("seed", range(48))
def test_bf16_random_configurations(seed):
    """Seeded random draws over everything the launch depends on at once: batch size, head grouping, tree size
    and layout, prefix lengths (some empty, some far below the bound), soft-prompt slots, a loose max_prefix_len,
    forced or free workgroup shape and range count.  Each draw is checked against the oracle like the hand-picked
    cases above."""
    rng = np.random.default_rng(9000 + seed)
    B = int(rng.choice([1, 1, 2, 3, 5, 9]))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 3, 4, 8]))
    layout = "interleaved" if rng.random() < 0.3 else "appended"
    T = int(rng.integers(1, 61))
    C = int(rng.integers(0, 5))
    if layout == "appended" and T + C > 128: C = 0
    top = int(rng.choice([40, 300, 1500, 5000]))
    P = [int(x) for x in rng.integers(0, top + 1, size=B)]
    if rng.random() < 0.3: P[int(rng.integers(0, B))] = 0
    s_len = int(rng.integers(0, min(P) + 1)) if rng.random() < 0.4 and min(P) > 0 else 0
    s_len = min(s_len, 70)
    bound = max(P) * int(rng.choice([1, 1, 2, 8])) + int(rng.choice([0, 0, 33]))
    wg = int(rng.choice([0, 0, 1, 2, 4]))
    splits = int(rng.choice([0, 0, 0, 1, 2, 3, 7]))
    std = float(rng.choice([0.3, 1.0]))
    inp = _case(9100 + seed, dtype="bf16", Hq=G * Hkv, Hkv=Hkv, D=128, P=P if B > 1 else P[0], T=T, C=C, s=s_len,
                layout=layout, B=B, q_std=std, kv_std=std, max_depth=int(rng.integers(6, 13)),
                max_children=int(rng.integers(2, 9)))
    print(f"[random] seed {seed}: B={B} Hq={G * Hkv} Hkv={Hkv} M={inp.M} P={P} s={s_len} bound={bound} wg={wg} splits={splits}",
          flush=True)
    out, lse, st = H.run_attention(inp, max_prefix_len=bound, wg_row_blocks=wg, num_splits=splits, prepare=bool(seed % 2))
    _check(inp, out, lse, st)


@pytest.mark.parametrize("seed", range(24))
def test_fp32_random_configurations(seed):
    rng = np.random.default_rng(9500 + seed)
    B = int(rng.choice([1, 2, 5]))
    Hkv = int(rng.choice([1, 2, 4]))
    G = int(rng.choice([1, 2, 3, 8]))
    D = int(rng.choice([64, 128]))
    layout = "interleaved" if rng.random() < 0.3 else "appended"
    T = int(rng.integers(1, 61))
    C = int(rng.integers(0, 5))
    P = [int(x) for x in rng.integers(0, int(rng.choice([40, 300, 1200])) + 1, size=B)]
    s_len = min(int(rng.integers(0, min(P) + 1)), 70) if rng.random() < 0.4 and min(P) > 0 else 0
    inp = _case(9600 + seed, dtype="f32", Hq=G * Hkv, Hkv=Hkv, D=D, P=P if B > 1 else P[0], T=T, C=C, s=s_len,
                layout=layout, B=B, max_depth=int(rng.integers(6, 13)), max_children=int(rng.integers(2, 9)))
    print(f"[random] seed {seed}: B={B} Hq={G * Hkv} Hkv={Hkv} D={D} M={inp.M} P={P} s={s_len}", flush=True)
    out, lse, st = H.run_attention(inp, max_prefix_len=max(P) * int(rng.choice([1, 4])) + 5)
    _check(inp, out, lse, st)


# ---- the named workloads at full size -----------------------------------------------------------------------
@pytest.mark.parametrize("index,peaked", [(1, False), (1, True), (2, False), (2, True)])
def test_full_size_single_sequence_workloads(index, peaked):
    """Llama-3.2-3B-shaped (G=3, P=2048) and Llama-3.1-8B-shaped (G=4, P=4096) layers, all outputs."""
    inp = si.attention_case(index, peaked=peaked)
    for wg in (0, 1, 4):
        out, lse, st = H.run_attention(inp, wg_row_blocks=wg)
        _check(inp, out, lse, st)


def test_full_size_long_context_all_heads():
    """Qwen3-4B-shaped, P=16384: every row of every head, in the launch shape the library picks."""
    inp = si.attention_case(4, peaked=True)
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st)


@pytest.mark.parametrize("peaked", [False, True])
def test_full_size_contemplate_row_per_node(peaked):
    """The paper's verification layout at Llama-3.1-8B size (Section 3.1): 60 nodes each followed by its
    contemplate row (120 rows, two mask words), 16 soft-prompt slots, prefix 4096: all outputs."""
    inp = si.attention_case(5, soft_len=16, peaked=peaked)
    assert inp.M == 120 and inp.soft_len == 16
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st)


def test_full_size_ragged_batch_all_heads():
    """Eight sequences, prefix lengths 512..8192, one pool: every row of every head of every sequence."""
    inp = si.attention_case(3, peaked=True)
    out, lse, st = H.run_attention(inp)
    _check(inp, out, lse, st)


@pytest.mark.parametrize("seed", range(8))
def test_bf16_random_large_configurations(seed):
    """Random draws at sizes where the planner leaves the single-sequence, 64-row default: long contexts, batches
    of unequal lengths, with and without the length hint.  Checked on two heads of every sequence."""
    rng = np.random.default_rng(9800 + seed)
    B = int(rng.choice([1, 2, 4, 12]))
    Hkv, G = int(rng.choice([2, 8])), int(rng.choice([2, 4]))
    top = int(rng.choice([9000, 20000, 45000])) if B <= 2 else int(rng.choice([3000, 9000]))
    P = [int(x) for x in rng.integers(top // 16, top + 1, size=B)]
    T = int(rng.integers(20, 61))
    layout = "interleaved" if rng.random() < 0.3 else "appended"
    inp = _case(9900 + seed, dtype="bf16", Hq=G * Hkv, Hkv=Hkv, D=128, P=P if B > 1 else P[0], T=T, C=4, layout=layout, B=B,
                s=int(rng.choice([0, 16])), q_std=1.0, kv_std=1.0)
    hint = sum(P) if rng.random() < 0.5 else 0
    import paper_2603_08899_amd as tv
    plan = tv.tv_attention_plan(tv.make_attn_desc(dtype=tv.TV_DTYPE_BF16, B=B, M=inp.M, Hq=G * Hkv, Hkv=Hkv, D=128,
                                                  soft_len=inp.soft_len, max_prefix_len=max(P), softmax_scale=inp.scale,
                                                  sum_prefix_len=hint))
    print(f"[random] seed {seed}: B={B} Hq={G * Hkv} Hkv={Hkv} M={inp.M} P={P} s={inp.soft_len} hint={hint} plan={plan}", flush=True)
    out, _, st = H.run_attention(inp, want_lse=False, sum_prefix_len=hint)
    assert np.all(st == 0)
    for b in range(B):
        ref = H.oracle_attention_rows(inp, b, range(inp.M), heads=[(3 * b) % (G * Hkv), G * Hkv - 1])
        for (i, h), r in ref.items():
            assert np.abs(out[b, i, h] - r).max() <= 2e-2
            assert np.abs(out[b, i, h] - r).max() <= REL_TOL_BF16 * np.abs(r).max() + 1e-4


def test_layers_from_one_pool_back_to_back():
    """Several layers' K/V in one allocation, one launch per layer on one stream without host
    synchronisation in between (the 32-layer benchmark configuration, shortened)."""
    import torch
    import paper_2603_08899_amd as tv
    w = si.WORKLOADS[2]
    layers = [si.attention_case(2, layer=l, peaked=True) for l in range(3)]
    L0 = layers[0]
    rows = L0.k_pool.shape[0]
    kpool = torch.stack([H.to_device_storage(x.k_pool, "bf16") for x in layers])
    vpool = torch.stack([H.to_device_storage(x.v_pool, "bf16") for x in layers])
    qs = [H.to_device_storage(x.q, "bf16") for x in layers]
    desc = tv.make_attn_desc(dtype=tv.TV_DTYPE_BF16, B=1, M=L0.M, Hq=w.Hq, Hkv=w.Hkv, D=128, soft_len=0,
                             max_prefix_len=int(L0.prefix_len[0]), softmax_scale=L0.scale)
    ws = torch.empty(max(tv.tv_attention_workspace_bytes(desc), 256), device="cuda", dtype=torch.uint8)
    kv_off = torch.zeros(1, dtype=torch.int64, device="cuda")
    plen = torch.from_numpy(L0.prefix_len).cuda()
    parent = torch.from_numpy(L0.parent).cuda()
    kind = torch.from_numpy(L0.kind).cuda()
    outs = [torch.empty_like(qs[0]) for _ in layers]
    status = torch.zeros(1, dtype=torch.int32, device="cuda")
    for l in range(len(layers)):
        tv.tree_verify_attention(desc, qs[l], kpool[l], vpool[l], kv_off, plen, parent, kind, outs[l], None,
                                 status, ws)
    torch.cuda.synchronize()
    assert rows == kpool.shape[1]
    for l, inp in enumerate(layers):
        ref = H.oracle_attention(inp, 0, want_lse=False)
        got = outs[l].float().cpu().numpy()[0].astype(np.float64)
        assert np.abs(got - ref).max() <= 2e-2
        assert np.abs(got - ref).max() <= REL_TOL_BF16 * np.abs(ref).max()


def test_host_only_call_before_torch_leaves_the_gpu_usable():
    """A fresh process that asks the library for a launch plan (a host-only call that reads the device's CU count)
    before anything has imported torch must still get a working torch.cuda afterwards, and a correct result: the
    binding has to make the library and PyTorch share one HIP runtime whichever is touched first."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = r'''
import sys
sys.path.insert(0, %r)
import paper_2603_08899_amd as tv
d = tv.make_attn_desc(dtype=tv.TV_DTYPE_F32, B=1, M=4, Hq=2, Hkv=1, D=64, soft_len=0, max_prefix_len=8, softmax_scale=0.125)
print("plan", tv.tv_attention_plan(d), flush=True)
import torch
q = torch.ones((1, 4, 2, 64), device="cuda"); k = torch.ones((12, 1, 64), device="cuda"); v = 2 * torch.ones((12, 1, 64), device="cuda")
out = torch.zeros_like(q); st = torch.zeros(1, dtype=torch.int32, device="cuda")
tv.tree_verify_attention(d, q, k, v, torch.zeros(1, dtype=torch.int64, device="cuda"), torch.full((1,), 8, dtype=torch.int32, device="cuda"),
                         torch.tensor([[-1, 0, 1, 2]], dtype=torch.int32, device="cuda"), torch.zeros((1, 4), dtype=torch.uint8, device="cuda"),
                         out, None, st, None)
torch.cuda.synchronize()
print("status", int(st[0]), "out", float(out.min()), float(out.max()), flush=True)
''' % root
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=110)
    assert r.returncode == 0, r.stderr[-800:]
    assert "plan (1, 1)" in r.stdout and "status 0 out 2.0 2.0" in r.stdout, r.stdout
