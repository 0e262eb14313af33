"""CPU-side checks of the C-ABI library: it loads, exports every symbol the header declares,
its host helpers agree with the oracle, and host-detectable errors are reported without a GPU."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
import paper_2603_08899_amd as tv
from synth_inputs import trees

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "confu_verify.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"^\s*(?:int|const char\*)\s+(\w+)\s*\(", text, flags=re.M))
    return names


def test_library_loads_and_exports_every_declared_symbol():
    l = tv.lib()
    declared = _declared_functions()
    assert declared == set(tv.EXPORTED_SYMBOLS), declared ^ set(tv.EXPORTED_SYMBOLS)
    for name in declared:
        assert getattr(l, name) is not None
    assert l.tv_version() >= 100
    assert l.tv_error_string(0) == b"ok"


def test_struct_layouts_match_header_sizes():
    # the library checks struct_size itself: a wrong python-side layout is rejected
    d = tv.make_attn_desc(dtype=tv.TV_DTYPE_BF16, B=1, M=64, Hq=32, Hkv=8, D=128, soft_len=0,
                          max_prefix_len=4096, softmax_scale=0.1)
    assert tv.tv_attention_workspace_bytes(d) > 0
    d.struct_size += 4
    with pytest.raises(tv.ConfuVerifyError):
        tv.tv_attention_workspace_bytes(d)
    a = tv.make_accept_desc(B=1, T=60, V=128256, C=4, rule=tv.TV_RULE_DRAFT_WOR, temperature=1.0)
    assert tv.tv_accept_workspace_bytes(a) > 0


@pytest.mark.parametrize("seed", range(6))
def test_host_mask_builder_matches_oracle_ancestor_matrix(seed):
    rng = np.random.default_rng(seed)
    T = int(rng.integers(1, 61))
    pn = trees.random_tree(rng, T, 8, 8)
    if seed % 2:
        parent, kind, _, _ = trees.interleave_contemplates_per_node(pn)
    else:
        parent, kind, _ = trees.append_contemplates_chained(pn, 4, anchor=int(rng.integers(0, T)))
    bits = tv.tv_build_mask_host(parent, kind)
    anc = oracle.ancestor_matrix(parent, kind)
    M = len(parent)
    for i in range(M):
        for j in range(M):
            assert ((int(bits[i, j // 64]) >> (j % 64)) & 1) == anc[i, j]


@pytest.mark.parametrize("parent,kind,bit", [
    ([-1, 1], [0, 0], tv.TV_STATUS_BAD_PARENT),
    ([-1, 2, 0], [0, 0, 0], tv.TV_STATUS_BAD_PARENT),
    ([-1, 0, 1], [0, 1, 0], tv.TV_STATUS_BAD_KIND),
    ([-1, 0], [0, 3], tv.TV_STATUS_BAD_KIND),
])
def test_host_mask_builder_rejects_what_the_oracle_rejects(parent, kind, bit):
    with pytest.raises(tv.ConfuVerifyError) as e:
        tv.tv_build_mask_host(parent, kind)
    assert e.value.code == -bit
    with pytest.raises(oracle.OracleError):
        oracle.ancestor_matrix(parent, kind)


@pytest.mark.parametrize("kw", [
    dict(M=0), dict(M=129), dict(Hq=7), dict(D=96), dict(softmax_scale=0.0), dict(soft_len=-1),
    dict(max_prefix_len=3, soft_len=16), dict(kv_head_stride=100), dict(kv_token_stride=1028), dict(B=0),
    dict(B=65536), dict(dtype=5), dict(sum_prefix_len=4097), dict(sum_prefix_len=-1),
])
def test_attention_descriptor_errors_on_host(kw):
    base = dict(dtype=tv.TV_DTYPE_BF16, B=1, M=64, Hq=32, Hkv=8, D=128, soft_len=0, max_prefix_len=4096,
                softmax_scale=0.1)
    base.update(kw)
    with pytest.raises(tv.ConfuVerifyError) as e:
        tv.tv_attention_workspace_bytes(tv.make_attn_desc(**base))
    assert e.value.code in (tv.TV_ERR_INVALID_ARG, tv.TV_ERR_UNSUPPORTED)


@pytest.mark.parametrize("kw", [dict(T=0), dict(T=129), dict(V=0), dict(rule=9), dict(temperature=0.0),
                                dict(logits_row_stride=5), dict(B=2000), dict(logits_dtype=7), dict(C=-1)])
def test_accept_descriptor_errors_on_host(kw):
    base = dict(B=1, T=60, V=1000, C=0, rule=tv.TV_RULE_DETERMINISTIC, temperature=1.0)
    base.update(kw)
    with pytest.raises(tv.ConfuVerifyError):
        tv.tv_accept_workspace_bytes(tv.make_accept_desc(**base))


def test_null_pointers_are_rejected_before_any_launch():
    # no device work is enqueued: the checks run on host scalars and pointer values only
    d = tv.make_attn_desc(dtype=tv.TV_DTYPE_F32, B=1, M=4, Hq=2, Hkv=1, D=64, soft_len=0,
                          max_prefix_len=8, softmax_scale=0.1)
    rc = tv.lib().tree_verify_attention(ctypes.byref(d), *([None] * 12), 0, None)
    assert rc == tv.TV_ERR_INVALID_ARG
    a = tv.make_accept_desc(B=1, T=4, V=10, C=0, rule=tv.TV_RULE_GREEDY, temperature=0.0)
    rc = tv.lib().tree_accept(ctypes.byref(a), *([None] * 14), 0, None)
    assert rc == tv.TV_ERR_INVALID_ARG


def test_workspace_grows_with_split_count():
    mk = lambda n: tv.tv_attention_workspace_bytes(tv.make_attn_desc(
        dtype=tv.TV_DTYPE_BF16, B=1, M=64, Hq=32, Hkv=8, D=128, soft_len=0, max_prefix_len=4096,
        softmax_scale=0.1, num_splits=n))
    assert mk(1) == 0 and mk(2) > 0 and mk(4) == 2 * mk(2)


def _plan(**kw):
    base = dict(dtype=tv.TV_DTYPE_BF16, B=1, M=64, Hq=32, Hkv=8, D=128, soft_len=0, max_prefix_len=4096,
                softmax_scale=0.1)
    base.update(kw)
    return tv.tv_attention_plan(tv.make_attn_desc(**base))


def test_attention_planner_choices_on_a_256_cu_device():
    """Host logic only (without a GPU the library assumes the MI355X's 256 CUs).  The shapes below are the ones the
    planner's cost model was fitted on; each expectation is the configuration measured fastest there (or, for a
    batch, the one its uniform/ragged hedge is documented to take)."""
    assert _plan() == (1, 8)                                     # the benchmark layer: one 64-row workgroup per CU
    assert _plan(max_prefix_len=1024) == (1, 4)                  # ranges keep at least eight tiles
    assert _plan(max_prefix_len=8192) == (1, 8)                  # 23.1 us against 25.2 with 128-row workgroups
    assert _plan(max_prefix_len=16384) in ((1, 8), (2, 16))      # measured equal (38.6 us both)
    assert _plan(max_prefix_len=32768) == (2, 16)                # long context: 128-row workgroups
    assert _plan(max_prefix_len=65536)[0] in (2, 4)
    assert _plan(B=4, max_prefix_len=1024) == (1, 2)             # short batch: one wave of workgroups, not two
    assert _plan(B=8, max_prefix_len=8192) == (2, 4)             # long batch: twice the CU count, for ragged lengths
    assert _plan(B=64, max_prefix_len=512)[1] == 1               # enough sequences: no split of the keys
    # the hint: the same batch shape sized for equal lengths, and for the ragged lengths of the batch-of-8 workload
    assert _plan(B=16, max_prefix_len=4096) == (2, 2) and _plan(B=16, max_prefix_len=4096, sum_prefix_len=16 * 4096) == (2, 1)
    wgs = lambda plan: 8 * 8 * (4 // plan[0]) * plan[1]           # B * Hkv * row groups * ranges
    assert wgs(_plan(B=8, max_prefix_len=8192, sum_prefix_len=8 * 8192)) == 256      # equal lengths: one per CU
    assert wgs(_plan(B=8, max_prefix_len=8192, sum_prefix_len=34868)) > 256          # ragged: more, smaller ones
    assert _plan(B=8, max_prefix_len=8192) == (2, 4)                                   # unknown: the compromise
    # what the caller fixes is kept
    assert _plan(num_splits=3) == (1, 3) and _plan(wg_row_blocks=4)[0] == 4
    assert _plan(num_splits=50)[1] == 16                         # capped: 130 tiles, at least eight per range
    assert _plan(dtype=tv.TV_DTYPE_F32, D=64) == (1, 1)
    # every workgroup count the planner can produce fits the grid
    for B in (1, 3, 17, 1000, 65535):
        for P in (0, 100, 5000, 200000):
            rb, n = _plan(B=B, max_prefix_len=P)
            assert rb in (1, 2, 4) and 1 <= n <= 64
            assert 8 * (4 // rb) * n < 2 ** 31


def test_a_plain_c_client_links_and_calls_the_host_entry_points(tmp_path):
    """The boundary is a C ABI: a C99 translation unit that includes the header, links the library and calls the
    host-only entry points (no device work) must build and agree with the Python binding."""
    import os, shutil, subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    src = tmp_path / "client.c"
    src.write_text(r'''
#include <stdio.h>
#include <string.h>
#include "confu_verify.h"
int main(void) {
    tv_attn_desc d;
    memset(&d, 0, sizeof d);
    d.struct_size = sizeof d; d.dtype = TV_DTYPE_BF16; d.B = 1; d.M = 64; d.Hq = 32; d.Hkv = 8; d.D = 128;
    d.max_prefix_len = 4096; d.softmax_scale = 0.088f;
    size_t bytes = 0; int32_t rb = 0, n = 0;
    int rc1 = tv_attention_workspace_bytes(&d, &bytes);
    int rc2 = tv_attention_plan(&d, &rb, &n);
    int32_t parent[3] = {-1, 0, 1}; uint8_t kind[3] = {0, 0, 1}; uint64_t bits[6];
    int rc3 = tv_build_mask_host(parent, kind, 3, bits);
    printf("%d %d %d %d %zu %d %d %llu %s\n", tv_version(), rc1, rc2, rc3, bytes, (int)rb, (int)n,
           (unsigned long long)bits[4], tv_error_string(TV_ERR_WORKSPACE));
    return 0;
}
''')
    exe = tmp_path / "client"
    libdir = os.path.dirname(tv.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(root, "include"), str(src), "-o", str(exe),
                           "-L", libdir, "-l:" + os.path.basename(tv.LIB_PATH), "-Wl,-rpath," + libdir])
    out = subprocess.check_output([str(exe)], text=True).split(None, 8)
    d = tv.make_attn_desc(dtype=tv.TV_DTYPE_BF16, B=1, M=64, Hq=32, Hkv=8, D=128, soft_len=0, max_prefix_len=4096,
                          softmax_scale=0.088)
    assert int(out[0]) == tv.lib().tv_version() and out[1:4] == ["0", "0", "0"]
    assert int(out[4]) == tv.tv_attention_workspace_bytes(d)
    assert (int(out[5]), int(out[6])) == tv.tv_attention_plan(d)
    assert int(out[7]) == 0b111                       # row 2 sees rows 0, 1 and itself
    assert out[8].strip() == "workspace missing or too small"
