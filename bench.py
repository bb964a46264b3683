#!/usr/bin/env python3
"""Benchmark of the sparse verification-attention step on one MI355X.

A "step" is one verification step of the whole model: for every layer, svf_verify_step with
retrieval (scores + top-N) on anchor layers and reuse of the anchor's block set elsewhere
(Sec. 3.3), i.e. cfg 3: 32 x verification attention + 16 x score/select at 32k context,
8 drafts, 2048-token budget, paged KV.  Block representatives are built once before the timed
region (they are maintained at prefill / cache growth, not per step) and timed separately.

Prints ONE JSON line (see the field list at the bottom).  Inputs are synthetic and resident in
HBM before the timed region; every layer has its own KV pool so no layer's KV is re-read from
cache between steps.
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

HBM_PEAK_GBPS = 8000.0          # MI355X HBM3E, published peak

TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "verify_attn_cfg3_hbm_traffic.md")
KERNEL_SOURCE = os.path.join(ROOT, "paper_2512_21911_amd", "csrc", "verify_attn_mfma.hip")


def measured_traffic(workload):
    """HBM bytes per reuse-layer attention launch from the rocprofv3 counter runs (FETCH_SIZE and
    WRITE_SIZE, scaled by a copy of known size), as recorded in the profile summary.  The summary
    carries the SHA-256 of the kernel source it was taken on; for any other source the figure is
    stale and None is reported."""
    import hashlib
    import re
    try:
        text = open(TRAFFIC_SUMMARY).read()
        sha = hashlib.sha256(open(KERNEL_SOURCE, "rb").read()).hexdigest()
    except OSError:
        return None
    m = re.search(r"traffic_bytes_per_launch\[(\w+)\]\s*=\s*(\d+)\s+kernel_source_sha256\s*=\s*([0-9a-f]{64})", text)
    if not m or m.group(1) != workload or m.group(3) != sha:
        return None
    return int(m.group(2))


def step_mode(cfg, layer):
    """Anchor layers retrieve; the others reuse the anchor's blocks and its gather list (all
    layers of a step share one page table and one set of sequence lengths)."""
    import paper_2512_21911_amd as S
    return S.SVF_STEP_ANCHOR if cfg.is_anchor(layer) else S.SVF_STEP_REUSE_GATHER


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--cfg", type=int, default=3, help="workload configuration (3 = the headline metric)")
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (0 = the config's)")
    ap.add_argument("--hnd", action="store_true",
                    help="store the cache pages head-major ([page][Hkv][slot][d]) instead of token-major "
                         "([page][slot][Hkv][d], the configurations' layout); same interface, through the strides")
    ap.add_argument("--tree", type=int, default=0,
                    help="verify a draft tree of this many nodes (depth 6; 60 = the paper's EAGLE-3 runs, Sec. 4.1) "
                         "instead of the configuration's drafts, over the same cache")
    ap.add_argument("--no-graph", action="store_true", help="time plain stream launches instead of a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-layers", type=int, default=32, help="layers the CPU oracle is timed on")
    ap.add_argument("--profile-only", default="", help="run only this many steps of the timed loop (for rocprofv3)")
    ap.add_argument("--mfma-vs-valu", action="store_true",
                    help="time the attention of the configuration's layers with the matrix-core kernel and with the "
                         "vector-ALU kernel (svf_diag_verify_attn) instead of the step; with --profile-only N just run "
                         "N passes of each for the profiler")
    ap.add_argument("--analytics", action="store_true",
                    help="time the retrieval analytics (per-draft block sets, overlap, Jaccard) instead of the step")
    ap.add_argument("--variants", action="store_true",
                    help="time the retrieval variants (min/max and bf16 summaries, group maximum, budget over all "
                         "KV heads) on the headline configuration instead of the step")
    ap.add_argument("--sffn", action="store_true",
                    help="time the sparse feed-forward verification (Sec. 3.4) on the 8B model's FFN shape instead of the step")
    ap.add_argument("--sffn-cfg", type=int, default=3, help="FFN workload (3: 8 tokens, 4: 60-node tree)")
    ap.add_argument("--rules", action="store_true",
                    help="time the per-token rules (expert skipping, Sec. 3.5; acceptance / resampling, Sec. 2.1) instead "
                         "of the step")
    return ap.parse_args()


def mfma_vs_valu(args):
    """The attention launch of every layer of the configuration (blocks already selected) with the kernel
    svf_verify_attn picks for the shape (matrix cores for bf16, d = 128) and with the vector-ALU kernel
    forced, each as one captured HIP graph over independent layers.  One JSON line."""
    import numpy as np
    import torch
    import paper_2512_21911_amd as S
    import workloads as W

    torch.cuda.set_device(0)
    S.lib()
    cfg = W.CONFIGS[args.cfg]
    n_layers = args.layers or (cfg.n_layers if cfg.n_layers > 1 else 16)
    layers = [W.make_layer(cfg, l, device="cuda") for l in range(n_layers)]
    x0 = layers[0]
    shape = S.make_shape(B=cfg.B, gamma=cfg.gamma, Hq=cfg.Hq, Hkv=cfg.Hkv, d=cfg.d, dtype=cfg.dtype,
                         block_size=cfg.block_size, max_seq_len=cfg.T, k_blocks=cfg.k_blocks, k_pool=x0["k_pool"],
                         page_size=cfg.page_size,
                         max_pages_per_seq=(x0["block_table"].shape[1] if x0["block_table"] is not None else 0))
    ws = S.new_workspace(shape)
    reps = torch.zeros(cfg.B, cfg.Hkv, cfg.nb_max, cfg.d, device="cuda")
    idx = [torch.zeros(cfg.B, cfg.Hkv, cfg.k_blocks, dtype=torch.int32, device="cuda") for _ in range(n_layers)]
    cnt = [torch.zeros(cfg.B, cfg.Hkv, dtype=torch.int32, device="cuda") for _ in range(n_layers)]
    for l, x in enumerate(layers):
        S.svf_block_reps(shape, x["k_pool"], x["block_table"], x["seq_lens"], reps)
        S.svf_score_select(shape, x["q"], reps, x["seq_lens"], idx[l], cnt[l], ws)
    torch.cuda.synchronize()
    outs = {k: torch.zeros(cfg.B, cfg.gamma, cfg.Hq, cfg.d, device="cuda", dtype=cfg.torch_dtype)
            for k in (S.SVF_KERNEL_AUTO, S.SVF_KERNEL_VECTOR_ALU)}
    wss = {k: S.new_diag_workspace(shape, k) for k in outs}

    def run(kernel):
        for l, x in enumerate(layers):
            S.svf_diag_verify_attn(shape, kernel, x["q"], x["k_pool"], x["v_pool"], x["block_table"], x["seq_lens"],
                                   x["k_draft"], x["v_draft"], x["draft_mask"], idx[l], cnt[l], outs[kernel], wss[kernel])

    if args.profile_only:
        for k in outs:
            for _ in range(int(args.profile_only)):
                run(k)
        torch.cuda.synchronize()
        print(json.dumps({"profile_only_passes": int(args.profile_only), "workload": cfg.name, "layers": n_layers}))
        return

    us = {}
    for k in outs:
        run(k)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            run(k)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        with torch.cuda.graph(graph):
            run(k)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(args.steps):
            graph.replay()
        b.record()
        torch.cuda.synchronize()
        us[k] = a.elapsed_time(b) / args.steps * 1e3 / n_layers
    diff = float((outs[S.SVF_KERNEL_AUTO].float() - outs[S.SVF_KERNEL_VECTOR_ALU].float()).abs().max())
    tol = 2e-2 if cfg.dtype == "bf16" else 1e-4
    if not diff <= tol:
        raise SystemExit(f"bench --mfma-vs-valu: the two kernels disagree on the last layer (max-abs {diff:.3e})")
    bytes_ = W.algorithmic_bytes(cfg, x0["seq_lens"].cpu())["verify_attn"]
    M = cfg.gamma * (cfg.Hq // cfg.Hkv)
    line = {"metric": f"verify-attn us/launch, matrix-core vs vector-ALU kernel ({cfg.name})",
            "value": round(us[S.SVF_KERNEL_AUTO], 3), "unit": "us/launch", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": round(us[S.SVF_KERNEL_AUTO] * 1e-3, 6), "higher_is_better": False,
            "scaling": "weak", "vs_baseline": None, "dtype": cfg.dtype, "data": "synthetic",
            "config": {"workload": cfg.name, "layers": n_layers, "query_rows_per_kv_head": M, "launch": "hipgraph"},
            "roofline": {"bound": "hbm", "kernel": "verify_attn_mfma_kernel (sel_idx resolved in the kernel)",
                         "achieved": round(bytes_ / (us[S.SVF_KERNEL_AUTO] * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBPS,
                         "unit": "GB/s", "frac": round(bytes_ / (us[S.SVF_KERNEL_AUTO] * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4),
                         "traffic": None, "algorithmic_bytes_per_launch": bytes_,
                         "avg_launch_us": round(us[S.SVF_KERNEL_AUTO], 3)},
            "cpu_baseline": None,
            "extra": {"matrix_core_kernel_us": round(us[S.SVF_KERNEL_AUTO], 3),
                      "vector_alu_kernels_us": round(us[S.SVF_KERNEL_VECTOR_ALU], 3),
                      "vector_alu_over_matrix_core": round(us[S.SVF_KERNEL_VECTOR_ALU] / us[S.SVF_KERNEL_AUTO], 2),
                      "max_abs_difference_of_outputs": diff}}
    print(json.dumps(line))


def analytics(args):
    """Retrieval analytics on a 60-draft tree (the shape Sec. 2.2 analyses) over cfg 3's cache:
    per-draft block sets of one layer, their overlap by positional distance, and the Jaccard counts of
    32 layers' first-draft masks.  One JSON line; the roofline object is for the per-draft retrieval
    (one pass over the fp32 representatives)."""
    import dataclasses
    import numpy as np
    import torch
    import paper_2512_21911_amd as S
    import workloads as W
    from oracle import svf_analytics_oracle as A
    from oracle import svf_oracle as O

    torch.cuda.set_device(0)
    S.lib()
    base = W.CONFIGS[3]
    cfg = dataclasses.replace(base, name="cfg3_cache_tree60", gamma=60, tree_depth=6, n_layers=1)
    n_rep = 16                                            # independent layers, so no launch re-reads a cached one
    layers = [W.make_layer(cfg, l, device="cuda") for l in range(n_rep)]
    x0 = layers[0]
    shape = S.make_shape(B=cfg.B, gamma=cfg.gamma, Hq=cfg.Hq, Hkv=cfg.Hkv, d=cfg.d, dtype=cfg.dtype,
                         block_size=cfg.block_size, max_seq_len=cfg.T, k_blocks=cfg.k_blocks, k_pool=x0["k_pool"],
                         page_size=cfg.page_size, max_pages_per_seq=x0["block_table"].shape[1],
                         n_sink=cfg.n_sink, n_local=cfg.n_local)
    Wd = S.svf_mask_words(shape)
    reps = [torch.zeros(cfg.B, cfg.Hkv, cfg.nb_max, cfg.d, device="cuda") for _ in range(n_rep)]
    for l, x in enumerate(layers):
        S.svf_block_reps(shape, x["k_pool"], x["block_table"], x["seq_lens"], reps[l])
    masks = [torch.zeros(cfg.B, cfg.Hkv, cfg.gamma, Wd, dtype=torch.int64, device="cuda") for _ in range(n_rep)]
    ws = S.new_analytics_workspace(shape)
    parents = W.draft_tree(cfg).tolist()
    pos = [0] * cfg.gamma
    for i, p in enumerate(parents):
        pos[i] = 0 if p < 0 else pos[p] + 1
    n_dist = max(pos) + 1
    pos_d = torch.tensor(pos, dtype=torch.int32, device="cuda")
    inter = torch.zeros(cfg.B, n_dist, dtype=torch.int64, device="cuda")
    n_jl = 32
    layer_masks = torch.stack([masks[l % n_rep][:, :, 0] for l in range(n_jl)]).contiguous()
    iu = torch.zeros(n_jl, 2, dtype=torch.int64, device="cuda")

    def timed(fn, iters, warm):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters * 1e3            # us per call of fn

    def select_all():
        for l, x in enumerate(layers):
            S.svf_select_per_draft(shape, x["q"], reps[l], x["seq_lens"], masks[l], ws)

    us_select = timed(select_all, args.steps, args.warmup) / n_rep
    us_overlap = timed(lambda: S.svf_overlap_by_distance(shape, masks[0], pos_d, n_dist, inter), args.steps, args.warmup)
    us_jaccard = timed(lambda: S.svf_jaccard_adjacent(shape, layer_masks, n_jl, iu), args.steps, args.warmup)

    # algorithmic bytes of the per-draft retrieval: representatives once, queries, masks out
    nb = cfg.nb_max
    bytes_select = (cfg.B * cfg.Hkv * nb * cfg.d * 4 + cfg.B * cfg.gamma * cfg.Hq * cfg.d * 2
                    + cfg.B * cfg.Hkv * cfg.gamma * Wd * 8)
    gbps = bytes_select / (us_select * 1e-6) / 1e9

    # CPU oracle on the same layer (CPU-generated tensors of the same recipe), checked against the GPU
    xc = W.make_layer(cfg, 0, device="cpu")
    w0, c0 = time.perf_counter(), time.process_time()
    reps_ref = O.block_reps(xc["k_pool"], xc["block_table"], xc["seq_lens"], cfg.block_size, cfg.nb_max)
    t_reps = time.perf_counter() - w0
    w1 = time.perf_counter()
    s_ref = A.per_draft_scores(xc["q"], reps_ref)
    m_ref = A.per_draft_masks(s_ref, xc["seq_lens"], cfg.block_size, cfg.k_blocks)
    inter_ref, pairs_ref, mean_ref = A.overlap_by_distance(m_ref, pos, xc["seq_lens"], cfg.block_size, cfg.k_blocks, n_dist)
    wall = time.perf_counter() - w1
    cpu_t = time.process_time() - c0
    xg = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in xc.items()}
    rg = torch.zeros_like(reps[0])
    mg = torch.zeros_like(masks[0])
    S.svf_block_reps(shape, xg["k_pool"], xg["block_table"], xg["seq_lens"], rg)
    S.svf_select_per_draft(shape, xg["q"], rg, xg["seq_lens"], mg, ws)
    S.svf_overlap_by_distance(shape, mg, pos_d, n_dist, inter)
    torch.cuda.synchronize()
    same_masks = bool(np.array_equal(mg.cpu().numpy().view(np.uint64), A.pack_masks(m_ref)))
    same_inter = bool(np.array_equal(inter.cpu().numpy(), inter_ref))
    if not (same_masks and same_inter):
        raise SystemExit("bench --analytics: GPU masks / overlap counts differ from the oracle on the sampled layer")
    line = {
        "metric": "per-draft retrieval us/layer (60-draft tree, 32k ctx)", "value": round(us_select, 2), "unit": "us/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(us_select * 1e-3, 5),
        "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "d": cfg.d, "T": cfg.T,
                   "block_size": cfg.block_size, "gamma": cfg.gamma, "tree_depth": cfg.tree_depth,
                   "k_blocks": cfg.k_blocks, "launch": "stream"},
        "roofline": {"bound": "hbm", "kernel": "block_scores_all_kernel + select_kernel", "achieved": round(gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": bytes_select, "avg_launch_us": round(us_select, 3)},
        "cpu_baseline": {"value": round(wall * 1e6, 1), "unit": "us/layer",
                         "cores": max(1, int(round(cpu_t / max(wall + t_reps, 1e-9)))), "kind": "oracle",
                         "sample": "oracle per-draft scores + masks + overlap on layer 0 (representatives excluded); "
                                   "GPU masks and overlap counts identical"},
        "extra": {"overlap_by_distance_us": round(us_overlap, 2), "jaccard_32_layers_us": round(us_jaccard, 2),
                  "mean_overlap_by_distance": [None if not np.isfinite(v) else round(float(v), 4) for v in mean_ref]},
    }
    print(json.dumps(line))


def variants(args):
    """Retrieval variants on cfg 3 (one layer's retrieval = summaries already in HBM -> scores -> kept
    blocks, then the attention over what was kept).  One JSON line: the headline value is the retrieval
    with bf16 min/max summaries, group maximum and the budget over all KV heads; `extra` has every
    combination timed, and the roofline object is the variant scores kernel (one pass over the summaries)."""
    import numpy as np
    import torch
    import paper_2512_21911_amd as S
    import workloads as W
    from oracle import svf_oracle as O
    from oracle import svf_variants_oracle as V

    torch.cuda.set_device(0)
    S.lib()
    cfg = W.CONFIGS[3]
    n_rep = 16
    layers = [W.make_layer(cfg, l, device="cuda") for l in range(n_rep)]
    x0 = layers[0]
    n_total = cfg.k_blocks * cfg.Hkv                       # Eq. 6: the budget counts all KV heads
    k_row = min(cfg.nb_max, n_total)

    def shape_with(k_blocks):
        return S.make_shape(B=cfg.B, gamma=cfg.gamma, Hq=cfg.Hq, Hkv=cfg.Hkv, d=cfg.d, dtype=cfg.dtype,
                            block_size=cfg.block_size, max_seq_len=cfg.T, k_blocks=k_blocks, k_pool=x0["k_pool"],
                            page_size=cfg.page_size, max_pages_per_seq=x0["block_table"].shape[1])

    def timed(fn, iters, warm):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters * 1e3 / n_rep    # us per layer

    names = {(0, 0): "mean_f32", (0, 1): "mean_bf16", (1, 0): "minmax_f32", (1, 1): "minmax_bf16"}
    combos = [(0, 0, 0, 0), (0, 1, 0, 0), (1, 0, 0, 0), (1, 1, 0, 0), (1, 1, 1, 0), (0, 0, 0, 1), (1, 1, 1, 1)]
    table = {}
    kept = {}
    for summary, sdt, group, budget in combos:
        shape = shape_with(k_row if budget else cfg.k_blocks)
        rt = S.SvfRetrieval(summary, sdt, group, budget, n_total if budget else 0)
        tdt = torch.bfloat16 if sdt else torch.float32
        summ = [torch.zeros(cfg.B, cfg.Hkv, cfg.nb_max, 2 if summary else 1, cfg.d, device="cuda", dtype=tdt)
                for _ in range(n_rep)]
        idx = [torch.zeros(cfg.B, cfg.Hkv, shape.k_blocks, dtype=torch.int32, device="cuda") for _ in range(n_rep)]
        cnt = [torch.zeros(cfg.B, cfg.Hkv, dtype=torch.int32, device="cuda") for _ in range(n_rep)]
        out = torch.zeros(cfg.B, cfg.gamma, cfg.Hq, cfg.d, device="cuda", dtype=cfg.torch_dtype)
        ws = S.new_workspace(shape)

        def do_summaries():
            for l, x in enumerate(layers):
                S.svf_block_summaries(shape, rt, x["k_pool"], x["block_table"], x["seq_lens"], summ[l])

        def do_retrieve():
            for l, x in enumerate(layers):
                S.svf_retrieve(shape, rt, x["q"], summ[l], x["seq_lens"], idx[l], cnt[l], ws)

        def do_attn():
            for l, x in enumerate(layers):
                S.svf_verify_attn(shape, x["q"], x["k_pool"], x["v_pool"], x["block_table"], x["seq_lens"],
                                  x["k_draft"], x["v_draft"], x["draft_mask"], idx[l], cnt[l], out, ws)

        us_sum = timed(do_summaries, max(2, args.steps // 10), 1)
        us_ret = timed(do_retrieve, args.steps, args.warmup)
        us_att = timed(do_attn, args.steps, args.warmup)
        key = f"{names[(summary, sdt)]}/{'group_max' if group else 'group_mean'}/{'global' if budget else 'per_head'}"
        sum_bytes = cfg.B * cfg.Hkv * cfg.nb_max * (2 if summary else 1) * cfg.d * (2 if sdt else 4)
        table[key] = {"summaries_us": round(us_sum, 2), "retrieve_us": round(us_ret, 2), "attention_us": round(us_att, 2),
                      "summary_bytes": sum_bytes,
                      "kept_per_head_min_max": [int(torch.stack(cnt).min()), int(torch.stack(cnt).max())]}
        kept[key] = (shape, rt, summ[0], idx[0], cnt[0], us_ret, sum_bytes)

    # CPU oracle of the headline variant on layer 0, and the GPU's kept blocks checked against it
    head = "minmax_bf16/group_max/global"
    shape, rt, _, _, _, us_head, sum_bytes = kept[head]
    xc = W.make_layer(cfg, 0, device="cpu")
    w0, c0 = time.perf_counter(), time.process_time()
    mn, mx = V.block_minmax(xc["k_pool"], xc["block_table"], xc["seq_lens"], cfg.block_size, cfg.nb_max)
    t_sum = time.perf_counter() - w0
    w1 = time.perf_counter()
    s_ref = V.group_scores(V.head_scores(xc["q"], mn=V.round_bf16(mn), mx=V.round_bf16(mx)), cfg.Hkv, V.GROUP_MAX)
    i_ref, c_ref = V.select_global(s_ref, xc["seq_lens"], cfg.block_size, n_total, k_row)
    wall = time.perf_counter() - w1
    cpu_t = time.process_time() - c0
    xg = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in xc.items()}
    sg = torch.zeros(cfg.B, cfg.Hkv, cfg.nb_max, 2, cfg.d, device="cuda", dtype=torch.bfloat16)
    ig = torch.zeros(cfg.B, cfg.Hkv, k_row, dtype=torch.int32, device="cuda")
    cg = torch.zeros(cfg.B, cfg.Hkv, dtype=torch.int32, device="cuda")
    wsg = S.new_workspace(shape)
    S.svf_block_summaries(shape, rt, xg["k_pool"], xg["block_table"], xg["seq_lens"], sg)
    S.svf_retrieve(shape, rt, xg["q"], sg, xg["seq_lens"], ig, cg, wsg)
    torch.cuda.synchronize()
    ig, cg = ig.cpu().numpy(), cg.cpu().numpy()
    excused = 0
    for b in range(cfg.B):
        got = {(h, int(j)) for h in range(cfg.Hkv) for j in ig[b, h, :cg[b, h]]}
        ref = {(h, int(j)) for h in range(cfg.Hkv) for j in i_ref[b, h, :c_ref[b, h]]}
        diff = got ^ ref
        nb = -(-int(xc["seq_lens"][b]) // cfg.block_size)
        if diff and not diff <= set(V.near_tie_pairs(s_ref[b], nb, i_ref[b], c_ref[b])):
            raise SystemExit("bench --variants: the GPU's kept blocks differ from the oracle's beyond near-ties")
        excused += len(diff)
    alg = sum_bytes + cfg.B * cfg.Hq * cfg.d * 2 + cfg.B * cfg.Hkv * cfg.nb_max * 4
    line = {
        "metric": "retrieval us/layer (bf16 min/max summaries, group max, budget over all KV heads; 32k ctx)",
        "value": round(us_head, 2), "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us_head * 1e-3, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "cfg3_long_batch_32k", "B": cfg.B, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "d": cfg.d, "T": cfg.T,
                   "block_size": cfg.block_size, "n_total_blocks": n_total, "launch": "stream"},
        "roofline": {"bound": "hbm", "kernel": "variant_scores_kernel + select_global_kernel",
                     "achieved": round(alg / (us_head * 1e-6) / 1e9, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(alg / (us_head * 1e-6) / 1e9 / HBM_PEAK_GBPS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": alg, "avg_launch_us": round(us_head, 3)},
        "cpu_baseline": {"value": round(wall * 1e6, 1), "unit": "us/layer",
                         "cores": max(1, int(round(cpu_t / max(wall + t_sum, 1e-9)))), "kind": "oracle",
                         "sample": f"oracle scores + global top-N on layer 0 (summaries excluded: {t_sum:.1f} s); "
                                   f"GPU kept blocks identical up to {excused} near-tie pairs"},
        "extra": table,
    }
    print(json.dumps(line))


def sffn(args):
    """Sparse feed-forward verification of one layer (gate -> threshold set -> up -> down) for the draft
    tokens of a step, on the feed-forward shape of the 8B target model, at the paper's thresholds.  Four
    independent layers are cycled so that no launch finds its weights in a cache.  One JSON line: the
    headline value is tau = 0.05; the roofline object prices the bytes that layer has to read (gate matrix,
    the up / down rows some token needs, x, y) against the HBM peak."""
    import numpy as np
    import torch
    import paper_2512_21911_amd as S
    from oracle import sffn_oracle as FO
    from workloads import ffn as WF

    torch.cuda.set_device(0)
    S.lib()
    cfg = WF.FFN_CONFIGS[args.sffn_cfg]
    n_rep = 4
    layers = [WF.make_ffn(cfg, l, device="cuda") for l in range(n_rep)]
    y = torch.zeros(cfg.M, cfg.d_model, device="cuda", dtype=torch.bfloat16)
    active = torch.zeros(cfg.d_ff, device="cuda", dtype=torch.int64)

    def timed(fn, iters, warm):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters * 1e3 / n_rep    # us per layer

    if args.profile_only:
        # for the profiler's byte counters: a few calls at tau = 0.05 (default walk), then plain copies of
        # known size to scale the counters with
        shape = S.make_ffn_shape(M=cfg.M, d_model=cfg.d_model, d_ff=cfg.d_ff, act=cfg.act, tau=0.05)
        ws = S.new_ffn_workspace(shape)
        for _ in range(int(args.profile_only)):
            for w in layers:
                S.svf_sparse_ffn(shape, w["x"], w["w_gate"], w["w_up"], w["w_down_t"], y, ws)
        torch.cuda.synchronize()
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"profile_only_steps": int(args.profile_only), "workload": cfg.name,
                          "calibration_copy_bytes": 256 << 20}))
        return

    row = cfg.d_model * 2
    table = {}
    for walk, tau in [(S.SVF_FFN_WALK_AUTO, t) for t in (0.0, 0.01, 0.05, 0.1)] + \
                     [(S.SVF_FFN_WALK_GATE_FIRST, t) for t in (0.0, 0.05, 0.1)]:
        shape = S.make_ffn_shape(M=cfg.M, d_model=cfg.d_model, d_ff=cfg.d_ff, act=cfg.act, tau=tau, walk=walk)
        ws = S.new_ffn_workspace(shape)

        def all_layers():
            for w in layers:
                S.svf_sparse_ffn(shape, w["x"], w["w_gate"], w["w_up"], w["w_down_t"], y, ws, w["b_gate"], w["b_up"],
                                 w["b_down"], active)

        us = timed(all_layers, max(3, args.steps // 2), max(1, args.warmup // 2))
        w = layers[-1]
        S.svf_sparse_ffn(shape, w["x"], w["w_gate"], w["w_up"], w["w_down_t"], y, ws, None, None, None, active)
        torch.cuda.synchronize()
        bits = active.cpu().numpy().view(np.uint64)
        rows = float((bits != 0).mean())
        per_tok = float(np.mean([((bits >> np.uint64(m)) & np.uint64(1)).mean() for m in range(cfg.M)]))
        alg = int(cfg.d_ff * row * (1 + 2 * rows) + 2 * cfg.M * row)
        key = f"tau={tau}" if walk == S.SVF_FFN_WALK_AUTO else f"gate_first tau={tau}"
        table[key] = {"us_per_layer": round(us, 2), "token_sparsity": round(1 - per_tok, 3),
                               "rows_read": round(rows, 3), "algorithmic_bytes": alg,
                               "GBps": round(alg / (us * 1e-6) / 1e9, 1)}
    head = table["tau=0.05"]

    # CPU oracle on layer 0 (CPU-generated tensors of the same recipe), and the GPU checked against it
    wc = WF.make_ffn(cfg, 0, device="cpu")
    toks = list(range(cfg.M)) if cfg.M <= 8 else [0, cfg.M // 2, cfg.M - 1]
    w0, c0 = time.perf_counter(), time.process_time()
    y_ref, a_ref, _ = FO.sparse_ffn(wc["x"][toks], wc["w_gate"], wc["w_up"], wc["w_down_t"], None, None, None, cfg.act, 0.05)
    wall, cpu_t = time.perf_counter() - w0, time.process_time() - c0
    shape = S.make_ffn_shape(M=cfg.M, d_model=cfg.d_model, d_ff=cfg.d_ff, act=cfg.act, tau=0.05)
    ws = S.new_ffn_workspace(shape)
    g = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in wc.items()}
    S.svf_sparse_ffn(shape, g["x"], g["w_gate"], g["w_up"], g["w_down_t"], y, ws, None, None, None, active)
    torch.cuda.synchronize()
    err = float(np.abs(y.double().cpu().numpy()[toks] - y_ref).max())
    if not err <= 2e-2 * max(1.0, float(np.abs(y_ref).max())):
        raise SystemExit(f"bench --sffn: GPU output differs from the oracle on the sampled layer (max-abs {err:.3e})")
    line = {
        "metric": f"sparse FFN verification us/layer (tau=0.05, {cfg.M} tokens, d_model={cfg.d_model}, d_ff={cfg.d_ff})",
        "value": head["us_per_layer"], "unit": "us/layer", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(head["us_per_layer"] * 1e-3, 5), "higher_is_better": False, "scaling": "weak",
        "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": cfg.name, "M": cfg.M, "d_model": cfg.d_model, "d_ff": cfg.d_ff, "act": cfg.act,
                   "tau": 0.05, "launch": "stream"},
        "roofline": {"bound": "hbm", "kernel": "ffn_gate_up_fused_kernel + ffn_down_kernel + ffn_reduce_kernel",
                     "achieved": head["GBps"], "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": round(head["GBps"] / HBM_PEAK_GBPS, 4),
                     # FETCH_SIZE + WRITE_SIZE of the three kernels, scaled (profiles/sparse_ffn_dense8b_hbm_traffic.md)
                     "traffic": 339.5e6 if cfg.name == "ffn3_dense_8b" else None,
                     "algorithmic_bytes_per_launch": head["algorithmic_bytes"], "avg_launch_us": head["us_per_layer"]},
        "cpu_baseline": {"value": round(wall * 1e6 * cfg.M / len(toks), 1), "unit": "us/layer",
                         "cores": max(1, int(round(cpu_t / max(wall, 1e-9)))), "kind": "oracle",
                         "sample": f"oracle sparse FFN of {len(toks)} of {cfg.M} tokens of layer 0 ({wall:.1f} s wall), "
                                   f"scaled to {cfg.M}; max-abs vs GPU {err:.2e}"},
        "extra": table,
    }
    print(json.dumps(line))


def rules(args):
    """The two per-token rules on the shapes of Sec. 4.3 (8 of 256 experts per token, draft length 4, a
    vocabulary of 129 280): acceptance / resampling of 64 sequences (headline), expert skipping of 4096
    tokens, calibration of one layer's thresholds on 65 536 tokens.  Small latency-bound kernels; the
    roofline object prices the bytes the acceptance kernel must read."""
    import numpy as np
    import torch
    import paper_2512_21911_amd as S
    from oracle import spec_rules_oracle as R
    from workloads import rules as WR

    torch.cuda.set_device(0)
    S.lib()

    def timed(fn, iters, warm):
        for _ in range(warm):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(iters):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters * 1e3

    B, gamma, V = 64, 4, 129280
    xc = WR.acceptance_inputs(B, gamma, V, seed=1)
    x = {k: v.cuda() for k, v in xc.items()}
    n_acc = torch.zeros(B, dtype=torch.int32, device="cuda")
    res = torch.zeros(B, dtype=torch.int32, device="cuda")
    call = lambda: S.svf_accept_resample(x["p_target"], x["p_draft"], x["draft_tokens"], x["u_accept"], x["u_resample"],
                                         n_acc, res)
    us_acc = timed(call, args.steps, args.warmup)
    w0, c0 = time.perf_counter(), time.process_time()
    n_ref, r_ref, _ = R.accept_resample(*(xc[k].numpy() for k in ("p_target", "p_draft", "draft_tokens", "u_accept",
                                                                   "u_resample")))
    wall, cpu_t = time.perf_counter() - w0, time.process_time() - c0
    same_n = bool(np.array_equal(n_acc.cpu().numpy(), n_ref))
    same_r = int((res.cpu().numpy() == r_ref).sum())
    if not same_n or same_r < B - 2:
        raise SystemExit("bench --rules: acceptance differs from the oracle on the timed batch")
    rejected = int((n_ref < gamma).sum())
    alg = rejected * 2 * V * 4 + B * gamma * 4 * 4

    T, k, m = 4096, 8, 3
    wc = WR.routing_weights(T, k, seed=2)
    cal = WR.routing_weights(65536, k, seed=3).cuda()
    beta = torch.zeros(k - 1, device="cuda")
    ws = torch.empty(int(S.lib().svf_moe_calibrate_workspace_bytes(65536, k)), dtype=torch.uint8, device="cuda")
    us_cal = timed(lambda: S.svf_moe_calibrate(cal, beta, ws), max(5, args.steps // 5), 2)
    wg = wc.cuda()
    n_skip = torch.zeros(T, dtype=torch.int32, device="cuda")
    mask = torch.zeros(T, dtype=torch.int32, device="cuda")
    us_skip = timed(lambda: S.svf_moe_skip(wg, m, beta, n_skip, mask), args.steps, args.warmup)
    t0 = time.perf_counter()
    n_skip_ref, _ = R.moe_skip(wc.numpy(), beta.cpu().double().numpy(), m)
    t_skip_cpu = time.perf_counter() - t0
    differ = int((n_skip.cpu().numpy() != n_skip_ref).sum())
    if differ > 4:
        raise SystemExit("bench --rules: expert skipping differs from the oracle on the timed batch")
    gbps = alg / (us_acc * 1e-6) / 1e9
    line = {
        "metric": f"acceptance + resampling us/step ({B} sequences, draft length {gamma}, vocabulary {V})",
        "value": round(us_acc, 2), "unit": "us/step", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(us_acc * 1e-3, 5), "higher_is_better": False, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32", "data": "synthetic",
        "config": {"workload": "rules_mtp4_vocab129k", "B": B, "gamma": gamma, "V": V, "launch": "stream"},
        "roofline": {"bound": "hbm", "kernel": "accept_kernel", "achieved": round(gbps, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(gbps / HBM_PEAK_GBPS, 4), "traffic": None,
                     "algorithmic_bytes_per_launch": alg, "avg_launch_us": round(us_acc, 3)},
        "cpu_baseline": {"value": round(wall * 1e6, 1), "unit": "us/step",
                         "cores": max(1, int(round(cpu_t / max(wall, 1e-9)))), "kind": "oracle",
                         "sample": f"oracle acceptance + resampling of the same {B} sequences ({rejected} rejected); "
                                   f"accepted counts identical, {same_r}/{B} resampled tokens identical"},
        "extra": {"moe_skip_us": round(us_skip, 2), "moe_skip_tokens": T, "moe_skip_k": k, "moe_skip_m": m,
                  "moe_skip_mean_skipped": round(float(n_skip_ref.mean()), 3),
                  "moe_skip_oracle_us": round(t_skip_cpu * 1e6, 1), "moe_skip_tokens_differing": differ,
                  "moe_calibrate_us": round(us_cal, 2), "moe_calibrate_tokens": 65536,
                  "mean_accepted": round(float(n_ref.mean()), 3)},
    }
    print(json.dumps(line))


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus must be 1 "
              "(the path shards over sequences / KV heads with no exchange)", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2512_21911_amd as S
    import workloads as W

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    if args.mfma_vs_valu:
        mfma_vs_valu(args)
        return
    if args.analytics:
        analytics(args)
        return
    if args.variants:
        variants(args)
        return
    if args.sffn:
        sffn(args)
        return
    if args.rules:
        rules(args)
        return
    S.lib()                      # fail loudly if the HIP library is missing
    torch.cuda.set_device(0)
    cfg = W.CONFIGS[args.cfg]
    if args.tree:
        import dataclasses
        cfg = dataclasses.replace(cfg, name=f"{cfg.name}_tree{args.tree}", gamma=args.tree, tree_depth=6)
    # single-layer configurations are replicated (independent seeds, every replica an anchor layer) so
    # that no launch re-reads a KV pool that is still in cache and the launch overhead is amortised
    n_layers = args.layers or (cfg.n_layers if cfg.n_layers > 1 else 16)
    t_setup = time.time()

    # ---- per-layer device inputs --------------------------------------------------------
    layers = []
    for l in range(n_layers):
        x = W.make_layer(cfg, l, device="cuda")
        if args.hnd and x["block_table"] is not None:
            for key in ("k_pool", "v_pool"):
                store = x[key].permute(0, 2, 1, 3).contiguous()     # storage [page][Hkv][slot][d]
                x[key] = store.permute(0, 2, 1, 3)                  # logical view: the strides carry the layout
        layers.append(x)
    x0 = layers[0]
    shape = S.make_shape(B=cfg.B, gamma=cfg.gamma, Hq=cfg.Hq, Hkv=cfg.Hkv, d=cfg.d, dtype=cfg.dtype,
                         block_size=cfg.block_size, max_seq_len=cfg.T, k_blocks=cfg.k_blocks, k_pool=x0["k_pool"],
                         page_size=cfg.page_size,
                         max_pages_per_seq=(x0["block_table"].shape[1] if x0["block_table"] is not None else 0),
                         n_sink=cfg.n_sink, n_local=cfg.n_local)
    ws = S.new_workspace(shape)
    dev = "cuda"
    reps = [torch.zeros(cfg.B, cfg.Hkv, cfg.nb_max, cfg.d, device=dev, dtype=torch.float32) for _ in range(n_layers)]
    outs = [torch.empty(cfg.B, cfg.gamma, cfg.Hq, cfg.d, device=dev, dtype=cfg.torch_dtype) for _ in range(n_layers)]
    sel_idx = torch.full((cfg.B, cfg.Hkv, cfg.k_blocks), -1, device=dev, dtype=torch.int32)
    sel_cnt = torch.zeros((cfg.B, cfg.Hkv), device=dev, dtype=torch.int32)
    # per-layer block sets, and one workspace per anchor (it holds that anchor's gather list), for
    # the loops that time one kind of launch at a time
    sel_idx_l = [torch.empty_like(sel_idx) for _ in range(n_layers)]
    sel_cnt_l = [torch.empty_like(sel_cnt) for _ in range(n_layers)]
    anchor_of = [max(a for a in range(l + 1) if cfg.is_anchor(a)) for l in range(n_layers)]
    ws_l = {a: S.new_workspace(shape) for a in set(anchor_of)}

    def ev():
        return torch.cuda.Event(enable_timing=True)

    # ---- block representatives: built once, timed on their own ---------------------------
    def reps_pass():
        for l, x in enumerate(layers):
            S.svf_block_reps(shape, x["k_pool"], x["block_table"], x["seq_lens"], reps[l])
    reps_pass()
    torch.cuda.synchronize()
    e0, e1 = ev(), ev()
    e0.record()
    reps_pass()
    e1.record()
    torch.cuda.synchronize()
    reps_ms = e0.elapsed_time(e1) / n_layers
    bytes_ = W.algorithmic_bytes(cfg, x0["seq_lens"].cpu())

    # ---- the step -----------------------------------------------------------------------
    def step():
        for l, x in enumerate(layers):
            S.svf_verify_step(shape, step_mode(cfg, l), x["q"], reps[l], x["k_pool"], x["v_pool"], x["block_table"],
                              x["seq_lens"], x["k_draft"], x["v_draft"], x["draft_mask"], sel_idx, sel_cnt,
                              outs[l], ws)

    def one_layer(l, mode):
        x, a = layers[l], anchor_of[l]
        S.svf_verify_step(shape, mode, x["q"], reps[l], x["k_pool"], x["v_pool"], x["block_table"],
                          x["seq_lens"], x["k_draft"], x["v_draft"], x["draft_mask"], sel_idx_l[a], sel_cnt_l[a],
                          outs[l], ws_l[a])

    def attn_only():
        """The attention launch of a reuse layer (the most frequent launch of a step), on every layer."""
        for l in range(n_layers):
            one_layer(l, S.SVF_STEP_REUSE_GATHER)

    def anchor_only():
        """The launch(es) of an anchor layer: retrieval + attention."""
        for l in range(n_layers):
            if cfg.is_anchor(l):
                one_layer(l, S.SVF_STEP_ANCHOR)

    def select_only():
        """Stand-alone block selection (svf_score_select without the scores output: one launch)."""
        for l, x in enumerate(layers):
            if cfg.is_anchor(l):
                S.svf_score_select(shape, x["q"], reps[l], x["seq_lens"], sel_idx, sel_cnt, ws)

    anchor_only()                      # block sets and gather lists for the attention-only loop
    torch.cuda.synchronize()
    setup_s = time.time() - t_setup

    def make_runner(fn):
        """Plain launches, or one captured HIP graph of the whole call sequence."""
        if args.no_graph:
            return fn
        fn()
        torch.cuda.synchronize()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            fn()
        return graph.replay

    def timed(run, iters, warm):
        for _ in range(warm):
            run()
        torch.cuda.synchronize()
        a, b = ev(), ev()
        a.record()
        for _ in range(iters):
            run()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / iters          # ms per call of run()

    run_step = make_runner(step)
    if args.profile_only:
        n = int(args.profile_only)
        for _ in range(n):
            run_step()
        torch.cuda.synchronize()
        # a plain copy of known size, for scaling the profiler's HBM byte counters
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(4):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"profile_only_steps": n, "workload": cfg.name, "calibration_copy_bytes": 256 << 20}))
        return

    ms_step = timed(run_step, args.steps, args.warmup)

    def per_replay(run, iters):
        """Each replay between its own pair of events (all enqueued back to back, one sync at the
        end): median / min / 90th percentile of a step in us."""
        evs = [ev() for _ in range(iters + 1)]
        evs[0].record()
        for i in range(iters):
            run()
            evs[i + 1].record()
        torch.cuda.synchronize()
        t = sorted(evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(iters))
        return {"median": round(t[len(t) // 2], 2), "min": round(t[0], 2), "p90": round(t[min(len(t) - 1, (9 * len(t)) // 10)], 2)}

    step_stats = per_replay(run_step, args.steps)
    run_attn = make_runner(attn_only)
    ms_attn = timed(run_attn, args.steps, args.warmup)
    run_anchor = make_runner(anchor_only)
    ms_anchor = timed(run_anchor, args.steps, args.warmup)
    run_sel = make_runner(select_only)
    ms_sel = timed(run_sel, args.steps, args.warmup)
    ms_step_eager = timed(step, max(3, args.steps // 5), 2)

    # What a plain device-to-device copy reaches when one launch moves as many bytes as one attention
    # launch has to (half read, half written), launches back to back on buffers that are not in cache:
    # the measured streaming ceiling for a problem of this size, beside the published peak.
    half = max(1 << 20, bytes_["verify_attn"] // 2 // 256 * 256)
    n_cp = max(8, min(64, (1 << 30) // (2 * half)))           # >= 1 GiB touched between reuses of a buffer
    srcs = [torch.empty(half, dtype=torch.uint8, device=dev) for _ in range(n_cp)]
    dsts = [torch.empty(half, dtype=torch.uint8, device=dev) for _ in range(n_cp)]

    def copies():
        for a_, b_ in zip(srcs, dsts):
            b_.copy_(a_)

    ms_copy = timed(make_runner(copies), max(3, args.steps // 2), 2)
    copy_us = ms_copy * 1e3 / n_cp
    copy_gbps = 2 * half / (copy_us * 1e-6) / 1e9
    del srcs, dsts

    n_anchor = sum(1 for l in range(n_layers) if cfg.is_anchor(l))
    attn_us = ms_attn * 1e3 / n_layers                        # average duration of one attention launch
    sel_us = ms_sel * 1e3 / max(1, n_anchor)
    anchor_us = ms_anchor * 1e3 / max(1, n_anchor)
    attn_gbps = bytes_["verify_attn"] / (attn_us * 1e-6) / 1e9
    step_bytes = n_layers * bytes_["verify_attn"] + n_anchor * bytes_["score_select"]

    # ---- sampled check against the oracle + CPU baseline (rank 0, N = 1) ------------------
    cpu_baseline = None
    near_ties = None
    if not args.no_cpu_baseline:
        from oracle import svf_oracle as O
        import numpy as np
        n_cpu = max(1, min(args.cpu_layers, n_layers))
        wall = 0.0
        cpu_t = 0.0
        idx = cnt = None
        worst = 0.0
        near_ties = 0
        gi, gc = torch.empty_like(sel_idx), torch.empty_like(sel_cnt)
        run_step()
        torch.cuda.synchronize()
        for l in range(n_cpu):
            x = W.make_layer(cfg, l, device="cpu")
            # the same seeds give different normals on CPU and GPU generators, so the GPU is re-run on
            # this CPU-generated layer for the sampled parity check
            xr = O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
            w0, c0 = time.perf_counter(), time.process_time()
            if cfg.is_anchor(l):
                s = O.block_scores(x["q"], xr)
                idx, cnt = O.select_blocks(s, x["seq_lens"], cfg.block_size, cfg.k_blocks, cfg.n_sink, cfg.n_local)
            out_ref, _ = O.verify_attn(x["q"], x["k_pool"], x["v_pool"], x["block_table"], x["seq_lens"],
                                       x["k_draft"], x["v_draft"], x["draft_mask"], idx, cnt, cfg.block_size)
            wall += time.perf_counter() - w0
            cpu_t += time.process_time() - c0
            xg = {k: (v.cuda() if isinstance(v, torch.Tensor) else v) for k, v in x.items()}
            if args.hnd and xg["block_table"] is not None:
                for key in ("k_pool", "v_pool"):
                    xg[key] = xg[key].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
            r = torch.empty_like(reps[0])
            o = torch.empty_like(outs[0])
            S.svf_block_reps(shape, xg["k_pool"], xg["block_table"], xg["seq_lens"], r)
            # anchor layers retrieve into gi / gc; the following layers reuse them (Eq. 9)
            S.svf_verify_step(shape, step_mode(cfg, l), xg["q"], r, xg["k_pool"], xg["v_pool"], xg["block_table"],
                              xg["seq_lens"], xg["k_draft"], xg["v_draft"], xg["draft_mask"], gi, gc, o, ws)
            torch.cuda.synchronize()
            if cfg.is_anchor(l) and not np.array_equal(gi.cpu().numpy(), idx):
                # blocks may differ only where the oracle's score is within 1e-3 (relative) of the
                # weakest block kept for its score; such near-ties are counted and reported
                gi_h, lens_h = gi.cpu().numpy(), x["seq_lens"].tolist()
                for b in range(cfg.B):
                    nb_b = -(-int(lens_h[b]) // cfg.block_size)
                    for h in range(cfg.Hkv):
                        c = int(cnt[b, h])
                        diff = set(gi_h[b, h, :c].tolist()) ^ set(idx[b, h, :c].tolist())
                        if not diff <= set(O.near_tie_blocks(s[b, h], nb_b, idx[b, h, :c], 1e-3, cfg.n_sink, cfg.n_local)):
                            raise SystemExit("bench: GPU block selection differs from the oracle on the sampled "
                                             f"layer {l} beyond near-ties (sequence {b}, KV head {h}: {sorted(diff)})")
                        near_ties += len(diff)
                # this layer and the reuse layers behind it are checked on the blocks the GPU kept
                idx, cnt = gi_h.copy(), gc.cpu().numpy().copy()
                out_ref, _ = O.verify_attn(x["q"], x["k_pool"], x["v_pool"], x["block_table"], x["seq_lens"],
                                           x["k_draft"], x["v_draft"], x["draft_mask"], idx, cnt, cfg.block_size)
            worst = max(worst, float(np.abs(o.double().cpu().numpy() - out_ref).max()))
            del xg, x
        tol = 2e-2 if cfg.dtype == "bf16" else 1e-4
        if worst > tol:
            raise SystemExit(f"bench: sampled parity check failed: max-abs {worst:.3e} > {tol}")
        cpu_us_step = wall / n_cpu * n_layers * 1e6
        cpu_baseline = {"value": round(cpu_us_step, 1), "unit": "us/step",
                        "cores": os.cpu_count(), "kind": "oracle",
                        "sample": f"fp64 numpy oracle (interpreted loops over sequences and KV heads around BLAS "
                                  f"calls, not a tuned CPU kernel): select+attention timed on layers 0..{n_cpu - 1} "
                                  f"of {n_layers} ({wall:.2f} s wall, {cpu_t / max(wall, 1e-9):.1f} threads busy on "
                                  f"average of the {os.cpu_count()} host cores), scaled to {n_layers} layers; "
                                  f"max-abs vs GPU {worst:.2e}; near-tie blocks excused {near_ties}"}

    value_us = ms_step * 1e3
    if cfg.dtype != "bf16" or cfg.d != 128:
        kernel_name = "verify_attn_valu_kernel"
    elif cfg.gamma * (cfg.Hq // cfg.Hkv) > 64:     # more than two groups of 32 query rows per KV head
        kernel_name = "verify_attn_mfma_rows_kernel (reuse layer, split merge inside)"
    else:
        kernel_name = "verify_attn_mfma_kernel (reuse layer)"
    line = {
        "metric": "verify-attn us/step (32k ctx, gamma=8, 2k budget)" if cfg.name == W.CONFIGS[3].name
                  else f"verify-attn us/step ({cfg.name})",
        "value": round(value_us, 2),
        "unit": "us/step",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 5),
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg.dtype,
        "data": "synthetic",
        "config": {"workload": cfg.name, "B": cfg.B, "Hq": cfg.Hq, "Hkv": cfg.Hkv, "d": cfg.d, "T": cfg.T,
                   "block_size": cfg.block_size, "gamma": cfg.gamma, "budget_tokens": cfg.k_blocks * cfg.block_size,
                   "page_size": cfg.page_size, "page_layout": "head-major" if args.hnd else "token-major",
                   "layers": n_layers, "anchor_layers": n_anchor,
                   "launch": "stream" if args.no_graph else "hipgraph"},
        "roofline": {"bound": "hbm", "kernel": kernel_name, "achieved": round(attn_gbps, 1),
                     "peak": HBM_PEAK_GBPS, "unit": "GB/s", "frac": round(attn_gbps / HBM_PEAK_GBPS, 4),
                     "traffic": measured_traffic(cfg.name) if n_layers == cfg.n_layers and not args.hnd and not args.tree else None,
                     "algorithmic_bytes_per_launch": bytes_["verify_attn"],
                     "avg_launch_us": round(attn_us, 3),
                     # against a plain device copy that moves the same bytes per launch, timed above
                     "stream_ceiling_GBps": round(copy_gbps, 1),
                     "frac_of_stream_ceiling": round(attn_gbps / copy_gbps, 4)},
        "cpu_baseline": cpu_baseline,
        "extra": {"step_GBps": round(step_bytes / (value_us * 1e-6) / 1e9, 1),
                  "step_us_median": step_stats["median"], "step_us_min": step_stats["min"],
                  "step_us_p90": step_stats["p90"],
                  "near_ties": near_ties,
                  # bounded waits between workgroups that ran out in all launches on the step's workspace so far
                  # (warm-up, timed and per-replay runs): the fallbacks give the same bits but cost microseconds
                  "wait_fallbacks": dict(zip(("exchange", "merge"), S.svf_diag_wait_fallbacks(shape, ws))),
                  "copy_same_bytes_us_per_launch": round(copy_us, 3),
                  "step_us_stream_launches": round(ms_step_eager * 1e3, 2),
                  "anchor_layer_us": round(anchor_us, 3),
                  "anchor_layer_GBps": round((bytes_["verify_attn"] + bytes_["score_select"]) / (anchor_us * 1e-6) / 1e9, 1),
                  "standalone_score_select_us": round(sel_us, 3),
                  "standalone_score_select_GBps": round(bytes_["score_select"] / (sel_us * 1e-6) / 1e9, 1),
                  "block_reps_us_per_layer": round(reps_ms * 1e3, 2),
                  "block_reps_GBps": round(bytes_["block_reps"] / (reps_ms * 1e-3) / 1e9, 1),
                  "setup_s": round(setup_s, 1)},
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
