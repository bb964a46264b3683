"""The verification step under HIP graph replay (the launch configuration the benchmark times): a
captured sequence of anchor and reuse layers must give, on every replay, the bits of the same calls
made eagerly - with other work and synchronisations between the replays (the anchor kernel's key
exchange advances its tags inside the graph, the workspaces reset themselves) - and those bits are
checked against the oracle."""
import dataclasses

import pytest
import torch

import paper_2512_21911_amd as S
import workloads as W
from svf_harness import DeviceRun, check_attn, oracle_attn, to_gpu

pytestmark = pytest.mark.gpu


def build_layers(cfg, n_layers):
    runs = []
    for l in range(n_layers):
        run = DeviceRun(cfg, to_gpu(W.make_layer(cfg, l)), poison=False)
        run.block_reps()
        if not cfg.is_anchor(l):                          # Eq. 9: the nearest preceding anchor's set, list and workspace
            a = runs[l - l % cfg.anchor_every]
            run.sel_idx, run.sel_cnt, run.ws = a.sel_idx, a.sel_cnt, a.ws
        runs.append(run)
    torch.cuda.synchronize()
    return runs


def step(cfg, runs):
    for l, run in enumerate(runs):
        run.verify_step(S.SVF_STEP_ANCHOR if cfg.is_anchor(l) else S.SVF_STEP_REUSE_GATHER)


def snapshot(runs):
    return [(r.out.clone(), r.lse.clone(), r.sel_idx.clone(), r.sel_cnt.clone()) for r in runs]


def poison_outputs(runs, cfg):
    for l, r in enumerate(runs):
        r.out.fill_(float("nan"))
        r.lse.fill_(float("nan"))
        if cfg.is_anchor(l):
            r.sel_idx.fill_(-7)
            r.sel_cnt.fill_(-7)


@pytest.mark.parametrize("T,n_layers,tree", [(4096, 4, 0), (32768, 2, 0), (4096, 4, 24)])
def test_step_graph_replays_match_eager_calls(T, n_layers, tree):
    cfg = W.shrink(W.CONFIGS[3], T) if T < W.CONFIGS[3].T else W.CONFIGS[3]
    if tree:        # a draft tree: the many-rows kernel
        cfg = dataclasses.replace(cfg, name=cfg.name + "_tree", gamma=tree, tree_depth=4)
    runs = build_layers(cfg, n_layers)
    step(cfg, runs)
    torch.cuda.synchronize()
    want = snapshot(runs)
    # the eager result against the oracle (reuse layers attend with the anchor's set, Eq. 9)
    for l, r in enumerate(runs):
        x = W.make_layer(cfg, l)
        out_ref, lse_ref = oracle_attn(cfg, x, r.sel_idx.cpu(), r.sel_cnt.cpu())
        check_attn(cfg, r.out, r.lse, out_ref, lse_ref)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        step(cfg, runs)                                   # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            step(cfg, runs)
    torch.cuda.synchronize()
    scratch = torch.zeros(1 << 20, device="cuda")
    for replay in range(4):
        poison_outputs(runs, cfg)
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for l, (r, (out, lse, idx, cnt)) in enumerate(zip(runs, want)):
            assert torch.equal(r.sel_idx, idx) and torch.equal(r.sel_cnt, cnt), f"replay {replay} layer {l}: selection"
            assert torch.equal(r.out.view(torch.int16), out.view(torch.int16)), f"replay {replay} layer {l}: output bits"
            assert torch.equal(r.lse.view(torch.int32), lse.view(torch.int32)), f"replay {replay} layer {l}: lse bits"
        # the program's own eager work between replays: an eager step and an unrelated kernel
        scratch.add_(1.0)
        if replay == 1:
            step(cfg, runs)
        torch.cuda.synchronize()
