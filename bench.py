#!/usr/bin/env python3
"""Benchmark of the tree-verification hot path on one MI355X.

A step is one verification pass of the Llama-3.1-8B-shaped workload: tree_verify_attention
for all 32 layers back to back from one KV pool (batch 1, 32 query / 8 KV heads, head dim 128,
prefix 4096, 60 draft nodes + 4 contemplate rows, bf16) followed by one tree_accept over a
128256-entry vocabulary at temperature 1.0.  Inputs are seeded and synthetic and resident in
HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--no-graph] [--no-cpu-baseline]
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E
WORKLOAD_INDEX = 2              # llama3.1-8b-32layers
PAPER_LAYOUT_INDEX = 5          # the same model shape with one contemplate row per draft node
OTHER_WORKLOADS = (0, 1, 3, 4)  # the other named configurations: parity cases, timed for information
DEEP_WALK_BOOST = 7.5           # child_boost of the acceptance inputs whose walk accepts about four nodes


TRAFFIC_FILE = os.path.join(ROOT, "profiles", "attn_bf16_kernel_llama8b_hbm_traffic.txt")


def measured_traffic(library_version):
    """(HBM bytes per attention launch, stamp) from the committed counter summary: the lines
    `traffic_bytes_per_launch = N` and `library_version = V`.  The bytes are None when the summary is absent or
    was taken with another version of the library than the one that is running."""
    traffic, stamp = None, None
    try:
        for line in open(TRAFFIC_FILE):
            if line.startswith("traffic_bytes_per_launch"):
                traffic = int(float(line.split("=")[1].split()[0]))
            elif line.startswith("library_version"):
                stamp = int(line.split("=")[1].split()[0])
    except OSError:
        pass
    if stamp != library_version:
        traffic = None
    return traffic, stamp


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (debugging)")
    ap.add_argument("--splits", type=int, default=0, help="key ranges per sequence (0 = library decides)")
    ap.add_argument("--wg-row-blocks", type=int, default=0, help="row blocks sharing a key stream (0 = library decides)")
    ap.add_argument("--no-paper-layout", action="store_true",
                    help="skip the extra measurements of the paper's 120-row layout and of the head-major pool")
    ap.add_argument("--others", default=",".join(str(i) for i in OTHER_WORKLOADS),
                    help="indices of the other named workloads to time (comma separated; empty: none)")
    ap.add_argument("--calibration-copy-mib", type=int, default=0,
                    help="also run three plain device copies of this many MiB before the timed region "
                         "(a kernel of known traffic, to scale hardware counters of a profiler run)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build measures one GPU only (the path has no multi-GPU part); run with --gpus 1",
              file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import paper_2603_08899_amd as tv
    import synth_inputs as si

    def to_device_bf16(bits):
        """uint16 bf16 bit patterns (numpy) -> bfloat16 tensor on the device."""
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = si.WORKLOADS[WORKLOAD_INDEX]
    L = args.layers or w.n_layers

    # ---- inputs, resident in HBM -------------------------------------------------------------------
    t0 = time.time()
    def attention_setup(index, soft_len=0, head_major=False, n_layers=None):
        """n_layers layers of workload `index` (all of the benchmark's by default) in one KV pool on the device, and
        a function that launches them.  The pool is [L, tokens, Hkv, D] (the workload's layout: the sequences of a
        batch one after the other); head_major=True holds the same rows as [L, Hkv, tokens, D] and hands the strides
        over in the descriptor."""
        wk = si.WORKLOADS[index]
        n_layers = n_layers or L
        first = si.attention_case(index, layer=0, soft_len=soft_len)
        bf16 = first.dtype == "bf16"
        tdt = torch.bfloat16 if bf16 else torch.float32
        to_dev = to_device_bf16 if bf16 else (lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).cuda())
        B, m, p = first.B, first.M, int(first.prefix_len.max())
        tokens = first.k_pool.shape[0]
        kp = torch.empty((n_layers, tokens, wk.Hkv, wk.D), device="cuda", dtype=tdt)
        vp = torch.empty_like(kp)
        q = torch.empty((n_layers, B, m, wk.Hq, wk.D), device="cuda", dtype=tdt)
        for l in range(n_layers):
            x = first if l == 0 else si.attention_case(index, layer=l, soft_len=soft_len)
            kp[l].copy_(to_dev(x.k_pool).reshape(tokens, wk.Hkv, wk.D))
            vp[l].copy_(to_dev(x.v_pool).reshape(tokens, wk.Hkv, wk.D))
            q[l].copy_(to_dev(x.q).reshape(B, m, wk.Hq, wk.D))
        strides = {}
        if head_major:
            kp = kp.permute(0, 2, 1, 3).contiguous()
            vp = vp.permute(0, 2, 1, 3).contiguous()
            strides = dict(kv_token_stride=wk.D, kv_head_stride=tokens * wk.D)
        o = torch.empty_like(q)
        off = torch.from_numpy(first.kv_offset.astype(np.int64)).cuda()
        pl = torch.from_numpy(first.prefix_len.astype(np.int32)).cuda()
        par = torch.from_numpy(np.ascontiguousarray(first.parent, dtype=np.int32)).cuda()
        kin = torch.from_numpy(np.ascontiguousarray(first.kind, dtype=np.uint8)).cuda()
        st = torch.zeros(B, dtype=torch.int32, device="cuda")
        desc = tv.make_attn_desc(dtype=tv.TV_DTYPE_BF16 if bf16 else tv.TV_DTYPE_F32, B=B, M=m, Hq=wk.Hq, Hkv=wk.Hkv,
                                 D=wk.D, soft_len=soft_len, max_prefix_len=p, softmax_scale=first.scale,
                                 num_splits=args.splits, wg_row_blocks=args.wg_row_blocks, **strides)
        ws = torch.empty(max(tv.tv_attention_workspace_bytes(desc), 256), device="cuda", dtype=torch.uint8)
        prep = torch.zeros(B * tv.TV_PREPARED_TREE_BYTES, device="cuda", dtype=torch.uint8)

        def run():
            # the tree is checked and its masks are built once per step, for all layers (Section 3.1 / Figure 4)
            if bf16:
                tv.tv_prepare_tree(par, kin, prep)
            for l in range(n_layers):
                tv.tree_verify_attention(desc, q[l], kp[l], vp[l], off, pl, par, kin, o[l], None, st, ws,
                                         prepared_tree=prep if bf16 else None)

        elem = 2 if bf16 else 4
        keys = [int(x) + m for x in first.prefix_len]
        bytes_layer = sum(2 * k * wk.Hkv * wk.D * elem for k in keys) + 2 * B * m * wk.Hq * wk.D * elem
        flops_layer = sum(4 * m * wk.Hq * k * wk.D for k in keys)
        rb, n_ranges = tv.tv_attention_plan(desc)
        return {"run": run, "first": first, "out": o, "M": m, "P": p, "bytes": bytes_layer, "flops": flops_layer,
                "layers": n_layers, "status": st,
                "plan": {"rows_per_workgroup": 64 * rb if bf16 else 16, "key_ranges": n_ranges},
                "keep": (kp, vp, q, off, pl, par, kin, st, ws, prep)}

    main_attn = attention_setup(WORKLOAD_INDEX)
    layer0, outs, M, P = main_attn["first"], main_attn["out"], main_attn["M"], main_attn["P"]
    attention_layers = main_attn["run"]

    acc = si.accept_case(WORKLOAD_INDEX, 1, child_boost=5.0)      # temperature 1.0, no draft logits
    cdesc = tv.make_accept_desc(B=1, T=acc.T, V=acc.V, C=acc.C, rule=acc.rule, temperature=acc.temperature)
    tl = torch.from_numpy(acc.target_logits).cuda()
    token = torch.from_numpy(acc.token).cuda()
    aparent = torch.from_numpy(acc.parent).cuda()
    un = torch.from_numpy(acc.uniforms).cuda()
    ca = torch.from_numpy(acc.con_anchor).cuda()
    i32 = dict(device="cuda", dtype=torch.int32)
    path = torch.zeros((1, acc.T), **i32)
    o_n, o_tok, o_kind, o_last, o_con, o_st = (torch.zeros(1, **i32) for _ in range(6))
    cws = torch.empty(max(tv.tv_accept_workspace_bytes(cdesc), 256), device="cuda", dtype=torch.uint8)
    gacc = si.accept_case(WORKLOAD_INDEX, 0, child_boost=5.0)     # temperature 0
    gdesc = tv.make_accept_desc(B=1, T=gacc.T, V=gacc.V, C=gacc.C, rule=gacc.rule, temperature=0.0)
    gtl = torch.from_numpy(gacc.target_logits).cuda()
    gtoken = torch.from_numpy(gacc.token).cuda()
    setup_s = time.time() - t0

    def accept():
        tv.tree_accept(cdesc, tl, None, token, aparent, un, ca, path, o_n, o_tok, o_kind, o_last, o_con, o_st, cws)

    def accept_greedy():
        tv.tree_accept(gdesc, gtl, None, gtoken, aparent, None, ca, path, o_n, o_tok, o_kind, o_last, o_con, o_st, cws)

    # the same call with the logits handed over as bf16 (the LM head's output type in a bf16 model)
    bdesc = tv.make_accept_desc(B=1, T=acc.T, V=acc.V, C=acc.C, rule=acc.rule, temperature=acc.temperature,
                                logits_dtype=tv.TV_DTYPE_BF16)
    tl16 = tl.to(torch.bfloat16)

    def accept_bf16():
        tv.tree_accept(bdesc, tl16, None, token, aparent, un, ca, path, o_n, o_tok, o_kind, o_last, o_con, o_st, cws)

    def full_step():
        attention_layers()
        accept()

    stream = torch.cuda.Stream()          # default priority

    if args.calibration_copy_mib > 0:
        # a plain elementwise kernel (out = in + 0, fp32): reads n bytes and writes n bytes
        n = args.calibration_copy_mib << 20
        src = torch.ones(n // 4, device="cuda", dtype=torch.float32)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.add(src, 0.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    def timed(fn, steps, warmup, calls_per_launch=1):
        """Average milliseconds per call of fn over `steps` launches, HIP events on the launch stream.  A launch
        is calls_per_launch calls of fn back to back (one graph when graphs are on): a call of one or two short
        kernels is timed like a layer of the 32-layer attention graph, without a graph launch of its own."""
        def several():
            for _ in range(calls_per_launch):
                fn()
        with torch.cuda.stream(stream):
            runner = several
            if not args.no_graph:
                fn()                      # first call sets kernel attributes outside the capture
                torch.cuda.synchronize()
                g = torch.cuda.CUDAGraph()
                with torch.cuda.graph(g, stream=stream):
                    several()
                runner = g.replay
            for _ in range(warmup):
                runner()
            torch.cuda.synchronize()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(steps):
                runner()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / (steps * calls_per_launch)

    ms_step = timed(full_step, args.steps, args.warmup)
    ms_attn = timed(attention_layers, args.steps, args.warmup)
    ms_accept = timed(accept, args.steps, args.warmup, 16)
    ms_greedy = timed(accept_greedy, args.steps, args.warmup, 16)
    ms_accept16 = timed(accept_bf16, args.steps, args.warmup, 16)

    # the same call on inputs whose walk is about as deep as the accepted lengths the paper reports (tau 3.5 - 5.3)
    dacc = si.accept_case(WORKLOAD_INDEX, 1, child_boost=DEEP_WALK_BOOST)
    dtl = torch.from_numpy(dacc.target_logits).cuda()
    dtoken = torch.from_numpy(dacc.token).cuda()
    dun = torch.from_numpy(dacc.uniforms).cuda()
    d_n = torch.zeros(1, **i32)

    def accept_deep():
        tv.tree_accept(cdesc, dtl, None, dtoken, aparent, dun, ca, path, d_n, o_tok, o_kind, o_last, o_con, o_st, cws)

    ms_accept_deep = timed(accept_deep, args.steps, args.warmup, 16)
    torch.cuda.synchronize()
    deep_tau = int(d_n[0]) + 1
    us_layer = ms_attn * 1e3 / L

    # ---- the steps around the pass: commit of the accepted path (all layers, one call), contemplate embedding -----
    kp_all, vp_all = main_attn["keep"][0], main_attn["keep"][1]
    cm_desc = tv.make_commit_desc(dtype=tv.TV_DTYPE_BF16, B=1, T=acc.T, M=M, Hkv=w.Hkv, D=w.D, n_layers=L,
                                  kv_layer_stride=kp_all.stride(0), C=acc.C, d_model=4096)
    hidden = torch.randn((1, M, 4096), device="cuda").to(torch.bfloat16)
    con_row = (acc.T + torch.arange(acc.C, device="cuda", dtype=torch.int32)).reshape(1, -1).contiguous()
    f_out = torch.empty((1, 4096), device="cuda", dtype=torch.bfloat16)
    new_len = torch.zeros(1, **i32)
    cm_status = torch.zeros(1, **i32)
    plen_d = main_attn["keep"][4]
    kv_off_d = main_attn["keep"][3]

    def commit():
        tv.tree_commit(cm_desc, kp_all, vp_all, kv_off_d, plen_d, path, o_n, None, hidden, con_row, o_con, f_out,
                       new_len, cm_status)

    em_desc = tv.make_embed_desc(dtype=tv.TV_DTYPE_BF16, B=1, d_in=3 * 4096, d_out=4096, n_expert=64, k_expert=4)
    em_h = torch.randn((1, 3 * 4096), device="cuda").to(torch.bfloat16)
    em_w = (torch.randn((64, 3 * 4096), device="cuda") * 0.02).to(torch.bfloat16)
    em_e = torch.randn((64, 4096), device="cuda").to(torch.bfloat16)
    em_out = torch.empty((1, 4096), device="cuda", dtype=torch.bfloat16)
    em_ws = torch.empty(tv.tv_embed_workspace_bytes(em_desc), device="cuda", dtype=torch.uint8)

    def embed():
        tv.contemplate_embed(em_desc, em_h, em_w, em_e, em_out, None, None, em_ws)

    with torch.cuda.stream(stream):
        accept()                          # path / n_accepted / selected_con for the commit
    torch.cuda.synchronize()
    ms_commit = timed(commit, args.steps, args.warmup, 16)      # (after the first call the moves are repeats)
    ms_embed = timed(embed, args.steps, args.warmup, 16)
    n_moved = int(o_n[0]) + 1
    around = {"tree_commit_us": round(ms_commit * 1e3, 2), "tree_commit_layers": L,
              "tree_commit_bytes_moved": 2 * 2 * L * n_moved * w.Hkv * w.D * 2,
              "contemplate_embed_us": round(ms_embed * 1e3, 2),
              "contemplate_embed_bytes_read": 2 * (64 * 3 * 4096 + 3 * 4096 + 4 * 4096),
              "contemplate_embed_shape": "d_in 12288, d_out 4096, 64 experts, top 4, bf16"}

    # ---- the paper's own layout (one contemplate row per node, 120 rows, 16 soft-prompt slots): MFMA-bound --------
    paper = None
    if not args.no_paper_layout:
        pa = attention_setup(PAPER_LAYOUT_INDEX, soft_len=16)
        us_paper = timed(pa["run"], max(args.steps // 2, 2), 2) * 1e3 / L
        paper_got = pa["out"][0].float().cpu().numpy()[0].astype(np.float64)
        paper_first, paper_rows = pa["first"], pa["M"]
        paper = {"workload": si.WORKLOADS[PAPER_LAYOUT_INDEX].name, "rows": pa["M"], "soft_len": 16, "prefix": pa["P"],
                 "us_per_layer": round(us_paper, 3),
                 "roofline": {"bound": "mfma", "achieved": round(pa["flops"] / (us_paper * 1e-6) / 1e12, 1),
                              "peak": 2500.0, "unit": "TFLOP/s",
                              "frac": round(pa["flops"] / (us_paper * 1e-6) / 2.5e15, 4), "traffic": None},
                 "hbm_gbps_on_algorithmic_bytes": round(pa["bytes"] / (us_paper * 1e-6) / 1e9, 1),
                 "max_abs_err_layer0_head3": None}        # filled in by the CPU-baseline leg
        del pa

    # ---- other shapes of the same kernel (information only; `value` stays the workload's own layout and size) ------
    other = None
    if not args.no_paper_layout:
        hm = attention_setup(WORKLOAD_INDEX, head_major=True)
        us_hm = timed(hm["run"], max(args.steps // 2, 2), 2) * 1e3 / L
        hm_same = bool(torch.equal(hm["out"][0], outs[0]))          # same rows, other strides: same bits
        del hm
        other = {"kv_head_major_pool_us_per_layer": round(us_hm, 3), "kv_head_major_output_identical": hm_same}

    # ---- the other named configurations, a few layers each (parity cases: timed for information only) ----------
    others = None
    other_indices = [int(x) for x in args.others.split(",") if x.strip() != ""]
    if other_indices:
        others = {}
        for idx in other_indices:
            wk = si.WORKLOADS[idx]
            # (enough layers for the pool to exceed the 256 MB last-level cache where the shape allows it)
            ow = attention_setup(idx, n_layers={0: 4, 1: 32, 3: 4, 4: 8}.get(idx, 8))
            us = timed(ow["run"], max(args.steps // 5, 3), 2) * 1e3 / ow["layers"]
            torch.cuda.synchronize()
            gbps = ow["bytes"] / (us * 1e-6) / 1e9
            ent = {"us_per_layer": round(us, 3), "batch": ow["first"].B, "max_prefix": ow["P"], "rows": ow["M"],
                   "dtype": ow["first"].dtype, "plan": ow["plan"], "status_ok": bool((ow["status"] == 0).all()),
                   "algorithmic_bytes_per_launch": ow["bytes"]}
            if ow["first"].dtype == "bf16":
                ent["roofline"] = {"bound": "hbm", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                                   "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None}
            else:       # the small fp32 case runs on the plain fp32 path
                tf = ow["flops"] / (us * 1e-6) / 1e12
                ent["roofline"] = {"bound": "alu", "achieved": round(tf, 3), "peak": 157.3, "unit": "TFLOP/s",
                                   "frac": round(tf / 157.3, 5), "traffic": None}
            others[wk.name] = ent
            del ow
            torch.cuda.empty_cache()

    # ---- what the CPU-baseline leg compares with the oracle (layer 0's output; the acceptance result) -----------
    torch.cuda.synchronize()
    got0 = outs[0].float().cpu().numpy()[0].astype(np.float64)
    with torch.cuda.stream(stream):
        accept()
    torch.cuda.synchronize()
    parity = None

    # ---- roofline of the dominant kernel (attention) ------------------------------------------------------
    bytes_layer, flops_layer = main_attn["bytes"], main_attn["flops"]
    lib_version = int(tv.lib().tv_version())
    traffic_bytes, traffic_stamp = measured_traffic(lib_version)
    achieved = bytes_layer / (us_layer * 1e-6) / 1e9
    roofline = {"bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": traffic_bytes,
                "traffic_profile_library_version": traffic_stamp, "library_version": lib_version,
                "kernel": "attn_bf16_kernel (+ combine), per layer launch",
                "algorithmic_bytes_per_launch": bytes_layer,
                "mfma_frac_of_bf16_peak": round(flops_layer / (us_layer * 1e-6) / 2.5e15, 4)}

    # ---- tree_accept: bytes moved (statistics of all T rows) and the visited-row (algorithmic) figure ------------
    n_visit = int(o_n[0]) + 1
    moved = acc.T * acc.V * 4
    accept_info = {
        "us_per_step": round(ms_accept * 1e3, 2), "bytes_moved": moved,
        "achieved_gbps_on_moved": round(moved / (ms_accept * 1e-3) / 1e9, 1),
        "visited_rows": n_visit, "algorithmic_bytes": n_visit * acc.V * 4,
        "frac_of_hbm_peak_on_algorithmic": round(n_visit * acc.V * 4 / (ms_accept * 1e-3) / 1e9 / HBM_PEAK_GBPS, 5),
        "greedy_us_per_step": round(ms_greedy * 1e3, 2),
        "bf16_logits_us_per_step": round(ms_accept16 * 1e3, 2), "bf16_logits_bytes_moved": moved // 2,
        "deep_walk": {"us_per_step": round(ms_accept_deep * 1e3, 2), "tau": deep_tau, "child_boost": DEEP_WALK_BOOST}}

    # ---- CPU oracle on the host cores, bounded sample (about 10 s of attention layers, 2 s of acceptance walks).
    #      The same leg compares what the GPU produced with what the oracle says (the only place the oracle is
    #      used). ------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        from tests import harness as H
        # layers of the benchmark pool, one after the other, until about ten seconds of oracle time are spent
        cpu_attn_s, n_cpu_layers, worst = 0.0, 0, 0.0
        while n_cpu_layers < L and cpu_attn_s < 10.0:
            x = layer0 if n_cpu_layers == 0 else si.attention_case(WORKLOAD_INDEX, layer=n_cpu_layers)
            q64, k64, v64 = x.q_f64(0), x.k_f64(0), x.v_f64(0)
            t1 = time.time()
            ref = oracle.tree_attention(q64, k64, v64, x.parent[0], x.kind[0], soft_len=0, scale=x.scale)
            cpu_attn_s += time.time() - t1
            got = got0 if n_cpu_layers == 0 else outs[n_cpu_layers].float().cpu().numpy()[0].astype(np.float64)
            worst = max(worst, float(np.abs(got - ref).max()))
            n_cpu_layers += 1
        t1 = time.time()
        n_walks = 0
        while n_walks < 3 or time.time() - t1 < 2.0:
            aref = H.oracle_accept(acc, 0)
            n_walks += 1
        cpu_accept_s = (time.time() - t1) / n_walks
        cpu = {"value": round(cpu_attn_s / n_cpu_layers * 1e6, 1), "unit": "us/layer", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"{n_cpu_layers} of the {L} layers (fp64, all rows and heads; {cpu_attn_s:.1f} s) and "
                         f"{n_walks} tree_accept walks ({cpu_accept_s * n_walks:.1f} s)",
               "tree_accept_steps_per_s": round(1.0 / cpu_accept_s, 2)}
        accept_ok = (int(o_tok[0]) == aref["final_token"] and int(o_n[0]) == aref["n_accepted"]
                     and np.array_equal(path.cpu().numpy()[0], aref["path"]))
        parity = {"attention_max_abs_err_all_rows_and_heads": worst, "attention_layers_compared": n_cpu_layers,
                  "accept_matches_oracle": bool(accept_ok)}
        if paper is not None:
            pref = H.oracle_attention_rows(paper_first, 0, range(paper_rows), heads=[3])
            paper["max_abs_err_layer0_head3"] = max(float(np.abs(paper_got[i, h] - r).max()) for (i, h), r in pref.items())

    line = {
        "metric": "verify-attn us/layer (60 nodes + 4 contemplate rows); tree_accept steps/sec reported alongside",
        "value": round(us_layer, 3), "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": w.name, "layers": L, "batch": 1, "Hq": w.Hq, "Hkv": w.Hkv, "D": w.D, "prefix": P,
                   "tree_nodes": w.T, "contemplate_rows": w.C, "vocab": w.V,
                   "launch": "eager" if args.no_graph else "hip-graph replay", "attention_plan": main_attn["plan"]},
        "tree_accept_steps_per_s": {"temp1.0_deterministic": round(1e3 / ms_accept, 1),
                                    "temp0_greedy": round(1e3 / ms_greedy, 1)},
        "tree_accept": accept_info,
        "contemplate_row_per_node": paper,
        "other_layouts": other,
        "other_workloads": others,
        "around_the_pass": around,
        "verify_steps_per_s": round(1e3 / ms_step, 2),
        "attention_tb_per_s": round(achieved / 1e3, 3),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "parity_sample": parity,
        "setup_seconds": round(setup_s, 1),
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
