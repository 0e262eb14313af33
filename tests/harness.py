"""Glue for the GPU parity tests: feeds one set of seeded inputs to the HIP library (through
its C ABI binding) and to the CPU oracle, and compares."""
from __future__ import annotations

import numpy as np

import oracle
from synth_inputs import AttnInputs, AcceptInputs, bf16_bits_to_f32


def _torch():
    import torch
    return torch


def to_device_storage(arr: np.ndarray, dtype: str):
    torch = _torch()
    if dtype == "bf16":
        return torch.from_numpy(np.ascontiguousarray(arr).view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(arr, dtype=np.float32)).cuda()


def run_attention(inp: AttnInputs, *, want_lse: bool = True, num_splits: int = 0, max_prefix_len=None,
                  device_inputs=None, wg_row_blocks: int = 0, sum_prefix_len: int = 0,
                  kv_token_stride: int = 0, kv_head_stride: int = 0, prepare: bool = False, noalloc: bool = False):
    """Returns (out float64 [B,M,Hq,D], lse float64 [B,Hq,M] or None, status int32 [B]).
    prepare=True: the trees go through tv_prepare_tree first and the call is handed the prepared record."""
    import paper_2603_08899_amd as tv
    torch = _torch()
    dt = tv.TV_DTYPE_BF16 if inp.dtype == "bf16" else tv.TV_DTYPE_F32
    mp = int(inp.prefix_len.max()) if max_prefix_len is None else int(max_prefix_len)
    desc = tv.make_attn_desc(dtype=dt, B=inp.B, M=inp.M, Hq=inp.Hq, Hkv=inp.Hkv, D=inp.D,
                             soft_len=inp.soft_len, max_prefix_len=mp, softmax_scale=inp.scale,
                             num_splits=num_splits, wg_row_blocks=wg_row_blocks, sum_prefix_len=sum_prefix_len,
                             kv_token_stride=kv_token_stride, kv_head_stride=kv_head_stride)
    if device_inputs is None:
        q = to_device_storage(inp.q, inp.dtype)
        k = to_device_storage(inp.k_pool, inp.dtype)
        v = to_device_storage(inp.v_pool, inp.dtype)
    else:
        q, k, v = device_inputs
    kv_off = torch.from_numpy(inp.kv_offset.astype(np.int64)).cuda()
    plen = torch.from_numpy(inp.prefix_len.astype(np.int32)).cuda()
    parent = torch.from_numpy(np.ascontiguousarray(inp.parent, dtype=np.int32)).cuda()
    kind = torch.from_numpy(np.ascontiguousarray(inp.kind, dtype=np.uint8)).cuda()
    out = torch.full((inp.B, inp.M, inp.Hq, inp.D), float("nan"), device="cuda",
                     dtype=torch.bfloat16 if inp.dtype == "bf16" else torch.float32)
    lse = torch.full((inp.B, inp.Hq, inp.M), float("nan"), device="cuda", dtype=torch.float32) if want_lse else None
    status = torch.full((inp.B,), -7, device="cuda", dtype=torch.int32)
    wsb = tv.tv_attention_workspace_bytes(desc)
    ws = torch.empty(max(wsb, 256), device="cuda", dtype=torch.uint8)
    prepared = None
    if prepare:
        prepared = torch.full((inp.B * tv.TV_PREPARED_TREE_BYTES,), 0xA5, device="cuda", dtype=torch.uint8)
        tv.tv_prepare_tree(parent, kind, prepared)
    if noalloc:      # the entry point that keeps its partial results in the library's own fixed array
        tv.tree_verify_attention_noalloc(desc, q, k, v, kv_off, plen, parent, kind, out, lse, status, prepared_tree=prepared)
    else:
        tv.tree_verify_attention(desc, q, k, v, kv_off, plen, parent, kind, out, lse, status, ws, prepared_tree=prepared)
    torch.cuda.synchronize()
    o = out.float().cpu().numpy().astype(np.float64)
    l = None if lse is None else lse.cpu().numpy().astype(np.float64)
    return o, l, status.cpu().numpy()


def oracle_attention(inp: AttnInputs, b: int, want_lse: bool = True):
    return oracle.tree_attention(inp.q_f64(b), inp.k_f64(b), inp.v_f64(b), inp.parent[b], inp.kind[b],
                                 soft_len=inp.soft_len, scale=inp.scale, return_lse=want_lse)


def oracle_attention_rows(inp: AttnInputs, b: int, rows, heads):
    """Oracle output for a few (row, head) pairs only: every other query is replaced by zeros is NOT
    done - instead the oracle runs on a sub-problem with just those heads (exact, since heads are
    independent) and all rows (rows of a tree are independent too, but the mask needs the full tree)."""
    q = inp.q_f64(b)
    k = inp.k_f64(b)
    v = inp.v_f64(b)
    G = inp.Hq // inp.Hkv
    outs = {}
    for h in heads:
        g = h // G
        o = oracle.tree_attention(q[:, h:h + 1], k[:, g:g + 1], v[:, g:g + 1], inp.parent[b], inp.kind[b],
                                  soft_len=inp.soft_len, scale=inp.scale)
        for i in rows:
            outs[(i, h)] = o[i, 0]
    return outs


def logits_rounded_to_bf16(inp: AcceptInputs) -> AcceptInputs:
    """The same case with both logits matrices rounded to bf16 values (kept as float32): what the oracle is
    given when the HIP path reads bf16 logits, so that both sides see identical numbers."""
    import dataclasses
    from synth_inputs import f32_to_bf16_bits

    def rnd(a):
        return None if a is None else bf16_bits_to_f32(f32_to_bf16_bits(np.asarray(a, dtype=np.float32)))
    return dataclasses.replace(inp, target_logits=rnd(inp.target_logits), draft_logits=rnd(inp.draft_logits))


def run_accept(inp: AcceptInputs, *, row_stride: int = 0, logits_dtype: str = "f32"):
    """logits_dtype 'bf16': the logits (which must hold bf16 values, see logits_rounded_to_bf16) are handed
    over as bf16."""
    import paper_2603_08899_amd as tv
    torch = _torch()
    bf16 = logits_dtype == "bf16"
    desc = tv.make_accept_desc(B=inp.B, T=inp.T, V=inp.V, C=inp.C, rule=inp.rule,
                               temperature=inp.temperature, logits_row_stride=row_stride,
                               logits_dtype=tv.TV_DTYPE_BF16 if bf16 else tv.TV_DTYPE_F32)
    ldt = torch.bfloat16 if bf16 else torch.float32

    def logits_dev(a):
        if a is None:
            return None
        x = torch.from_numpy(np.ascontiguousarray(a)).cuda()
        if bf16:
            assert torch.equal(x.to(ldt).to(torch.float32), x), "logits are not bf16 values"
        if row_stride:
            buf = torch.full((inp.B, inp.T, row_stride), float("nan"), device="cuda", dtype=ldt)
            buf[:, :, :inp.V] = x.to(ldt)
            return buf
        return x.to(ldt)

    tl = logits_dev(inp.target_logits)
    dl = logits_dev(inp.draft_logits)
    token = torch.from_numpy(inp.token).cuda()
    parent = torch.from_numpy(inp.parent).cuda()
    un = torch.from_numpy(inp.uniforms).cuda()
    ca = None if inp.con_anchor is None else torch.from_numpy(inp.con_anchor).cuda()
    i32 = dict(device="cuda", dtype=torch.int32)
    path = torch.full((inp.B, inp.T), -9, **i32)
    outs = {k: torch.full((inp.B,), -9, **i32) for k in
            ("n_accepted", "final_token", "final_kind", "last_node", "selected_con", "status")}
    ws = torch.empty(max(tv.tv_accept_workspace_bytes(desc), 256), device="cuda", dtype=torch.uint8)
    tv.tree_accept(desc, tl, dl, token, parent, un, ca, path, outs["n_accepted"], outs["final_token"],
                   outs["final_kind"], outs["last_node"], outs["selected_con"], outs["status"], ws)
    torch.cuda.synchronize()
    res = {k: v.cpu().numpy() for k, v in outs.items()}
    res["path"] = path.cpu().numpy()
    return res


def oracle_accept(inp: AcceptInputs, b: int) -> dict:
    return oracle.tree_accept(inp.target_logits[b], None if inp.draft_logits is None else inp.draft_logits[b],
                              inp.token[b], inp.parent[b], inp.uniforms[b], temperature=inp.temperature,
                              rule=inp.rule, con_anchor=None if inp.con_anchor is None else inp.con_anchor[b])


def _softmax64(z, temp):
    z = z.astype(np.float64) / temp
    e = np.exp(z - z.max())
    return e / e.sum()


def decision_margins(inp: AcceptInputs, b: int, ref: dict) -> float:
    """Smallest distance to its threshold of any comparison made along the oracle's walk
    (accept tests in probability units, final draw as |CDF - u|); fp64, numpy.  Used only to
    classify a GPU/oracle disagreement as 'within 1e-6 of a threshold'."""
    if inp.rule == oracle.RULE_GREEDY:
        return np.inf
    T = inp.T
    un = inp.uniforms[b]
    parent, token = inp.parent[b], inp.token[b]
    margin = np.inf
    path = ref["path"][:ref["n_accepted"] + 1]
    p = None
    if inp.rule == oracle.RULE_SAMPLE_MATCH:
        # one inverse-CDF draw at every visited node
        for cur in path:
            cdf = np.cumsum(_softmax64(inp.target_logits[b, cur], inp.temperature))
            margin = min(margin, float(np.abs(cdf - float(un[T + cur])).min()))
        return margin
    for step, cur in enumerate(path):
        p = _softmax64(inp.target_logits[b, cur], inp.temperature)
        q = None if inp.draft_logits is None else _softmax64(inp.draft_logits[b, cur], inp.temperature)
        for c in range(cur + 1, T):
            if parent[c] != cur:
                continue
            x = token[c]
            if inp.rule == oracle.RULE_DETERMINISTIC:
                margin = min(margin, abs(float(un[c]) - p[x]))
                acc = float(un[c]) < p[x]
            else:
                margin = min(margin, abs(float(un[c]) * q[x] - p[x]))
                acc = float(un[c]) * q[x] < p[x]
            if acc:
                break
            if inp.rule == oracle.RULE_DETERMINISTIC:
                p[x] = 0
                p = p / p.sum()
            else:
                r = np.maximum(p - q, 0)
                if r.sum() > 0:
                    p = r / r.sum()
                if inp.rule == oracle.RULE_DRAFT_WOR:
                    q[x] = 0
                    q = q / q.sum()
    cdf = np.cumsum(p)
    margin = min(margin, float(np.abs(cdf - float(un[T + path[-1]])).min()))
    return margin


def compare_accept(inp: AcceptInputs, got: dict):
    """Returns (exact matches, near-threshold disagreements).  Raises on any other disagreement."""
    exact = near = 0
    for b in range(inp.B):
        ref = oracle_accept(inp, b)
        assert got["status"][b] == 0, f"status {got['status'][b]} for sequence {b}"
        same = (got["n_accepted"][b] == ref["n_accepted"] and got["final_token"][b] == ref["final_token"]
                and got["final_kind"][b] == ref["final_kind"] and got["last_node"][b] == ref["last_node"]
                and got["selected_con"][b] == ref["selected_con"]
                and np.array_equal(got["path"][b], ref["path"]))
        if same:
            exact += 1
            continue
        mg = decision_margins(inp, b, ref)
        if mg < 1e-6:
            near += 1
            continue
        raise AssertionError(
            f"sequence {b}: GPU path {got['path'][b][:8]} n={got['n_accepted'][b]} tok={got['final_token'][b]} "
            f"kind={got['final_kind'][b]} vs oracle path {ref['path'][:8]} n={ref['n_accepted']} "
            f"tok={ref['final_token']} kind={ref['final_kind']} (closest threshold margin {mg:.3e})")
    return exact, near
