"""GPU test of the entry point for callers that cannot allocate: tree_verify_attention_noalloc, called through the
C ABI, against tree_verify_attention on the same inputs - the same kernels and launch shape, so the same bits -
on two calls in a row, the second with a smaller input (the fixed scratch array keeps the first call's contents)."""
import numpy as np
import pytest

import synth_inputs as si
from synth_inputs import trees
from tests import harness as H

pytestmark = pytest.mark.gpu


def _case(seed, B, P, T, C, s):
    rng = np.random.default_rng(seed)
    par, kin = [], []
    for b in range(B):
        pn = trees.random_tree(rng, T, 8, 8)
        p, k, _ = trees.append_contemplates_chained(pn, C, anchor=0)
        par.append(p)
        kin.append(k)
    return si.make_attention_inputs(rng, dtype="bf16", Hq=8, Hkv=2, D=128, prefix_len=P, parent=np.stack(par),
                                    kind=np.stack(kin), soft_len=s, q_std=1.0, kv_std=1.0, pool_pad_tokens=0)


def _both(inp, **kw):
    import torch
    import paper_2603_08899_amd as tv
    ref = H.run_attention(inp, **kw)
    got = H.run_attention(inp, noalloc=True, **kw)
    assert np.array_equal(ref[2], got[2])
    assert np.array_equal(ref[0], got[0]) and np.array_equal(ref[1], got[1])
    return got


def test_noalloc_entry_point_matches_the_workspace_one_twice_in_a_row():
    import paper_2603_08899_amd as tv
    big = _case(5, 3, [3000, 1500, 700], 60, 4, 16)        # several key ranges: the scratch array is used
    desc = tv.make_attn_desc(dtype=tv.TV_DTYPE_BF16, B=3, M=64, Hq=8, Hkv=2, D=128, soft_len=16, max_prefix_len=3000,
                             softmax_scale=big.scale)
    assert 0 < tv.tv_attention_workspace_bytes(desc) <= tv.TV_NOALLOC_SCRATCH_BYTES
    out, lse, st = _both(big)
    for b in range(3):
        ref, ref_lse = H.oracle_attention(big, b)
        assert st[b] == 0 and np.abs(out[b] - ref).max() <= 2e-2 and np.abs(lse[b] - ref_lse).max() <= 1e-3
    small = _case(6, 1, 900, 20, 2, 0)                       # smaller input, fewer partial results
    out, lse, st = _both(small, num_splits=3)
    ref, ref_lse = H.oracle_attention(small, 0)
    assert st[0] == 0 and np.abs(out[0] - ref).max() <= 2e-2 and np.abs(lse[0] - ref_lse).max() <= 1e-3


def test_noalloc_entry_point_refuses_what_does_not_fit():
    import torch
    import paper_2603_08899_amd as tv
    desc = tv.make_attn_desc(dtype=tv.TV_DTYPE_BF16, B=64, M=128, Hq=32, Hkv=8, D=128, soft_len=0, max_prefix_len=8192,
                             softmax_scale=0.1, num_splits=8)
    assert tv.tv_attention_workspace_bytes(desc) > tv.TV_NOALLOC_SCRATCH_BYTES
    dummy = torch.zeros(64, device="cuda", dtype=torch.int64)
    with pytest.raises(tv.ConfuVerifyError) as e:
        tv.tree_verify_attention_noalloc(desc, dummy, dummy, dummy, dummy, dummy, dummy, dummy, dummy, None, dummy)
    assert e.value.code == tv.TV_ERR_WORKSPACE
