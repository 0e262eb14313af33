"""GPU parity: tree_commit (bit-exact row moves) and contemplate_embed (fp32 sums of bf16/fp32
inputs) against oracle/bookkeeping.py on identical seeded inputs, through the C ABI."""
import numpy as np
import pytest

import synth_inputs as si
from oracle import bookkeeping as bk
from synth_inputs import trees
from tests import harness as H

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def _random_paths(rng, B, T, max_depth, max_children):
    """Root-to-node paths of random trees, -1 padded, with some sequences marked as failed (n = -1)."""
    path = np.full((B, T), -1, dtype=np.int32)
    n_acc = np.zeros(B, dtype=np.int32)
    for b in range(B):
        parent = trees.random_tree(rng, T, max_depth, max_children)
        node = int(rng.integers(0, T))
        p = [node]
        while parent[p[-1]] >= 0:
            p.append(int(parent[p[-1]]))
        p = p[::-1]
        path[b, :len(p)] = p
        n_acc[b] = len(p) - 1
    return path, n_acc


def _run_commit(dtype, L, B, T, M, Hkv, D, plen, path, n_acc, node_row, *, pad_tokens=0, head_major=False,
                hidden=None, con_row=None, selected=None, seed=0):
    import paper_2603_08899_amd as tv
    torch = _torch()
    rng = np.random.default_rng(seed)
    rows_b = [int(p) + M for p in plen]
    kv_off = np.concatenate([[0], np.cumsum(rows_b)[:-1]]).astype(np.int64)
    rows = int(sum(rows_b)) + pad_tokens
    shape = (L, Hkv, rows, D) if head_major else (L, rows, Hkv, D)
    if dtype == "bf16":
        kbits = rng.integers(0, 0x7F80, size=shape).astype(np.uint16)        # finite bf16 patterns
        vbits = rng.integers(0, 0x7F80, size=shape).astype(np.uint16)
        k64, v64 = si.bf16_bits_to_f32(kbits).astype(np.float64), si.bf16_bits_to_f32(vbits).astype(np.float64)
        kd, vd = H.to_device_storage(kbits, "bf16"), H.to_device_storage(vbits, "bf16")
        dt = tv.TV_DTYPE_BF16
    else:
        k64, v64 = rng.standard_normal(shape), rng.standard_normal(shape)
        k64, v64 = k64.astype(np.float32).astype(np.float64), v64.astype(np.float32).astype(np.float64)
        kd, vd = H.to_device_storage(k64, "f32"), H.to_device_storage(v64, "f32")
        dt = tv.TV_DTYPE_F32
    if head_major:
        ts, hs = D, rows * D
        k_ref, v_ref = k64.transpose(0, 2, 1, 3), v64.transpose(0, 2, 1, 3)
    else:
        ts, hs = Hkv * D, D
        k_ref, v_ref = k64, v64
    d_model = 0 if hidden is None else hidden.shape[2]
    C = 0 if con_row is None else con_row.shape[1]
    desc = tv.make_commit_desc(dtype=dt, B=B, T=T, M=M, Hkv=Hkv, D=D, n_layers=L,
                               kv_layer_stride=(Hkv * rows * D), kv_token_stride=ts, kv_head_stride=hs,
                               C=C, d_model=d_model)
    i32 = lambda x: None if x is None else torch.from_numpy(np.ascontiguousarray(x, dtype=np.int32)).cuda()
    new_len = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    status = torch.full((B,), -7, dtype=torch.int32, device="cuda")
    hid_d = f_d = None
    if hidden is not None:
        hid_d = H.to_device_storage(hidden if dtype == "f32" else si.f32_to_bf16_bits(hidden.astype(np.float32)), dtype)
        f_d = torch.full((B, d_model), 7.0, device="cuda", dtype=hid_d.dtype)
    tv.tree_commit(desc, kd, vd, torch.from_numpy(kv_off).cuda(), i32(plen), i32(path), i32(n_acc), i32(node_row),
                   hid_d, i32(con_row), i32(selected), f_d, new_len, status)
    torch.cuda.synchronize()
    nk, nv, nl, st = bk.commit_kv(k_ref, v_ref, kv_off, plen, path, n_acc, node_row, M)
    got_k = kd.float().cpu().numpy().astype(np.float64)
    got_v = vd.float().cpu().numpy().astype(np.float64)
    if head_major:
        got_k, got_v = got_k.transpose(0, 2, 1, 3), got_v.transpose(0, 2, 1, 3)
    assert np.array_equal(new_len.cpu().numpy(), nl)
    assert np.array_equal(status.cpu().numpy(), st)
    assert np.array_equal(got_k, nk) and np.array_equal(got_v, nv)          # moves are bit-exact
    return f_d, nl, st


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("layout", ["appended", "interleaved"])
def test_commit_random_paths_small(dtype, layout):
    rng = np.random.default_rng(31)
    B, T, Hkv, D, L = 5, 12, 2, 64 if dtype == "f32" else 128, 3
    M = 2 * T if layout == "interleaved" else T + 3
    node_row = np.tile(np.arange(0, 2 * T, 2, dtype=np.int32), (B, 1)) if layout == "interleaved" else None
    path, n_acc = _random_paths(rng, B, T, 6, 3)
    n_acc[3] = -1                                              # a sequence tree_accept flagged
    plen = rng.integers(0, 40, size=B).astype(np.int32)
    _run_commit(dtype, L, B, T, M, Hkv, D, plen, path, n_acc, node_row, seed=1)


def test_commit_overlapping_moves_and_full_chain():
    """Path 0 -> 1 -> 2 -> ... in the interleaved layout: every destination is an earlier entry's source."""
    T = 40
    path = np.arange(T, dtype=np.int32)[None]
    node_row = np.arange(0, 2 * T, 2, dtype=np.int32)[None]
    _run_commit("bf16", 2, 1, T, 2 * T, 8, 128, [100], path, [T - 1], node_row, seed=2)
    # the same chain with nodes first: nothing moves
    _run_commit("bf16", 2, 1, T, T + 4, 8, 128, [100], path, [T - 1], None, seed=3)


def test_commit_malformed_paths_are_flagged_and_nothing_moves():
    T = 8
    path = np.array([[0, 3, 2, -1, -1, -1, -1, -1], [1, 2, -1, -1, -1, -1, -1, -1], [0, 9, -1, -1, -1, -1, -1, -1],
                     [0, 2, 5, -1, -1, -1, -1, -1]], dtype=np.int32)
    _, nl, st = _run_commit("bf16", 1, 4, T, T, 2, 128, [5, 6, 7, 8], path, [2, 1, 1, 2], None, seed=4)
    assert list(st) == [bk.STATUS_BAD_PATH] * 3 + [0] and list(nl) == [5, 6, 7, 11]


def test_commit_rows_that_do_not_increase_along_the_path_are_flagged():
    """A row map under which a child's row comes before its parent's contradicts the tree the attention ran over:
    flagged, nothing moves (the path spans several chunks of the move)."""
    T = 40
    path = np.arange(T, dtype=np.int32)[None].repeat(2, axis=0)
    node_row = np.tile(np.arange(T, dtype=np.int32), (2, 1))
    node_row[0, 20], node_row[0, 21] = 21, 20                 # sequence 0: two neighbours of the path swapped
    _, nl, st = _run_commit("bf16", 2, 2, T, T + 4, 8, 128, [10, 12], path, [T - 1, T - 1], node_row, seed=6)
    assert list(st) == [bk.STATUS_BAD_PATH, 0] and list(nl) == [10, 12 + T]


def test_commit_padded_and_head_major_pools():
    rng = np.random.default_rng(33)
    B, T = 3, 20
    path, n_acc = _random_paths(rng, B, T, 7, 4)
    _run_commit("bf16", 2, B, T, T + 4, 4, 128, [64, 0, 130], path, n_acc, None, pad_tokens=5, seed=5)
    _run_commit("bf16", 2, B, T, T + 4, 4, 128, [64, 0, 130], path, n_acc, None, head_major=True, seed=6)


def test_commit_llama8b_shape_all_layers_with_future_gather():
    """32 layers of the benchmark shape (Hkv 8, D 128, P 4096, 60 nodes + 4 contemplate rows) in one call, fed by
    tree_accept's own outputs; the future prediction of the selected contemplate row is gathered."""
    acc = si.accept_case(2, 1, child_boost=5.0)
    got = H.run_accept(acc)
    T, C = acc.T, acc.C
    M = T + C
    rng = np.random.default_rng(7)
    hidden = rng.standard_normal((1, M, 4096)).astype(np.float32)
    con_row = (T + np.arange(C, dtype=np.int32))[None]
    f_d, nl, st = _run_commit("bf16", 32, 1, T, M, 8, 128, [4096], got["path"], got["n_accepted"], None,
                              hidden=hidden, con_row=con_row, selected=got["selected_con"], seed=8)
    assert st[0] == 0 and nl[0] == 4096 + got["n_accepted"][0] + 1
    hid_bf = si.bf16_bits_to_f32(si.f32_to_bf16_bits(hidden)).astype(np.float64)
    f_ref = bk.gather_future(hid_bf, con_row, got["selected_con"])
    assert np.array_equal(f_d.float().cpu().numpy().astype(np.float64), f_ref)


# ---- contemplate_embed --------------------------------------------------------------------------------------
def _run_embed(dtype, B, d_in, d_out, n_expert, k_expert, seed, tie=False):
    import paper_2603_08899_amd as tv
    torch = _torch()
    rng = np.random.default_rng(seed)
    h = rng.standard_normal((B, d_in)).astype(np.float32)
    w = (rng.standard_normal((n_expert, d_in)) / np.sqrt(d_in)).astype(np.float32) * 2.0
    e = rng.standard_normal((n_expert, d_out)).astype(np.float32)
    if tie and n_expert > 3:
        w[3] = w[1]
    if dtype == "bf16":
        hb, wb, eb = (si.f32_to_bf16_bits(x) for x in (h, w, e))
        h, w, e = (si.bf16_bits_to_f32(x) for x in (hb, wb, eb))
        hd, wd, ed = (H.to_device_storage(x, "bf16") for x in (hb, wb, eb))
        out = torch.full((B, d_out), 7.0, device="cuda", dtype=torch.bfloat16)
        dt = tv.TV_DTYPE_BF16
    else:
        hd, wd, ed = (H.to_device_storage(x, "f32") for x in (h, w, e))
        out = torch.full((B, d_out), 7.0, device="cuda", dtype=torch.float32)
        dt = tv.TV_DTYPE_F32
    gates = torch.full((B, n_expert), -1.0, device="cuda", dtype=torch.float32)
    chosen = torch.full((B, k_expert), -1, device="cuda", dtype=torch.int32)
    desc = tv.make_embed_desc(dtype=dt, B=B, d_in=d_in, d_out=d_out, n_expert=n_expert, k_expert=k_expert)
    ws = torch.empty(tv.tv_embed_workspace_bytes(desc), device="cuda", dtype=torch.uint8)
    tv.contemplate_embed(desc, hd, wd, ed, out, gates, chosen, ws)
    torch.cuda.synchronize()
    ref_out, ref_g, ref_ch = bk.contemplate_embed(h, w, e, k_expert)
    g = gates.cpu().numpy().astype(np.float64)
    ch = chosen.cpu().numpy()
    o = out.float().cpu().numpy().astype(np.float64)
    # gates: fp32 dot products and exponentials of exact inputs
    assert np.abs(g - ref_g).max() <= 1e-5
    for b in range(B):
        # the selection may differ from the oracle's only between experts whose scores are closer than the gate error
        srt = np.sort(ref_g[b])[::-1]
        clear = all(abs(srt[i] - srt[i + 1]) > 1e-5 for i in range(min(k_expert, n_expert - 1)))
        if clear or tie:
            assert list(ch[b]) == list(ref_ch[b]), (ch[b], ref_ch[b])
        mine = sum(ref_g[b, x] * e[x].astype(np.float64) for x in ch[b])
        tol = 1e-5 if dtype == "f32" else 2.0 ** -8 * max(1.0, np.abs(mine).max())
        assert np.abs(o[b] - mine).max() <= tol
        if clear:
            assert np.abs(o[b] - ref_out[b]).max() <= tol
    return o


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("n_expert,k_expert", [(1, 1), (8, 2), (16, 16), (64, 4), (37, 5)])
def test_embed_small(dtype, n_expert, k_expert):
    _run_embed(dtype, 3, 64, 40, n_expert, k_expert, seed=40 + n_expert)


def test_embed_ties_take_the_lowest_index():
    _run_embed("f32", 4, 128, 64, 8, 3, seed=50, tie=True)


def test_embed_llama8b_widths():
    """The target-side module of an 8B model: input = three concatenated hidden states (3 x 4096), output width
    4096; and the draft-side module (4096 -> 4096); 64 experts, top 4."""
    _run_embed("bf16", 1, 3 * 4096, 4096, 64, 4, seed=60)
    _run_embed("bf16", 8, 4096, 4096, 64, 4, seed=61)


@pytest.mark.parametrize("seed", range(24))
def test_commit_random_configurations(seed):
    """Everything tree_commit's launch depends on drawn together: type, layers, batch, tree size and row layout,
    head count and width, prefix lengths (some zero), pool padding or a head-major pool, flagged sequences."""
    rng = np.random.default_rng(5000 + seed)
    dtype = str(rng.choice(["bf16", "f32"]))
    L, B, T = int(rng.integers(1, 6)), int(rng.choice([1, 2, 6, 33])), int(rng.integers(1, 41))
    Hkv = int(rng.choice([1, 2, 8]))
    D = int(rng.choice([64, 128])) if dtype == "f32" else int(rng.choice([64, 128, 256]))
    interleaved = bool(rng.random() < 0.4)
    M = 2 * T if interleaved else T + int(rng.integers(0, 5))
    node_row = np.tile(np.arange(0, 2 * T, 2, dtype=np.int32), (B, 1)) if interleaved else None
    path, n_acc = _random_paths(rng, B, T, int(rng.integers(6, 13)), int(rng.integers(2, 9)))
    if B > 1 and rng.random() < 0.5:
        n_acc[int(rng.integers(0, B))] = -1
    plen = rng.integers(0, 70, size=B).astype(np.int32)
    if rng.random() < 0.3:
        plen[int(rng.integers(0, B))] = 0
    head_major = bool(rng.random() < 0.3)
    pad = 0 if head_major else int(rng.choice([0, 0, 3]))
    print(f"[random] seed {seed}: {dtype} L={L} B={B} T={T} M={M} Hkv={Hkv} D={D} head_major={head_major} pad={pad}", flush=True)
    _run_commit(dtype, L, B, T, M, Hkv, D, plen, path, n_acc, node_row, pad_tokens=pad, head_major=head_major, seed=seed)


@pytest.mark.parametrize("seed", range(24))
def test_embed_random_configurations(seed):
    rng = np.random.default_rng(5500 + seed)
    dtype = str(rng.choice(["f32", "bf16"]))
    B = int(rng.choice([1, 2, 5, 19]))
    d_in = 8 * int(rng.integers(1, 200))
    d_out = 8 * int(rng.integers(1, 200))
    n_expert = int(rng.integers(1, 65))
    k_expert = int(rng.integers(1, n_expert + 1))
    print(f"[random] seed {seed}: {dtype} B={B} d_in={d_in} d_out={d_out} experts={n_expert} top={k_expert}", flush=True)
    _run_embed(dtype, B, d_in, d_out, n_expert, k_expert, seed=5600 + seed)
