"""The entry point that allocates nothing (workspace in a static device array) against
svf_verify_attn: the same bits, on two calls in a row, the second with a smaller input."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2512_21911_amd as S
import workloads as W
from svf_harness import DeviceRun, check_attn, oracle_attn, to_gpu

pytestmark = pytest.mark.gpu


def run_both(cfg):
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x))
    run.block_reps().score_select().verify_attn().sync()
    out0, lse0 = run.out.clone(), run.lse.clone()
    ref, lse_ref = oracle_attn(cfg, x, run.sel_idx.cpu(), run.sel_cnt.cpu())
    check_attn(cfg, out0, lse0, ref, lse_ref)
    run.out.fill_(float("nan"))
    run.lse.fill_(float("nan"))
    g = run.x
    before = torch.cuda.memory_allocated()
    S.svf_verify_attn_static_ws(run.shape, g["q"], g["k_pool"], g["v_pool"], g["block_table"], g["seq_lens"],
                                g["k_draft"], g["v_draft"], g["draft_mask"], run.sel_idx, run.sel_cnt, run.out, run.lse)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert torch.equal(run.out.view(torch.int16 if cfg.dtype == "bf16" else torch.int32),
                       out0.view(torch.int16 if cfg.dtype == "bf16" else torch.int32)), cfg.name
    assert torch.equal(run.lse.view(torch.int32), lse0.view(torch.int32)), cfg.name
    check_attn(cfg, run.out, run.lse, ref, lse_ref)
    return run


def test_static_workspace_entry_point_matches_on_two_calls_in_a_row():
    assert S.svf_static_workspace_bytes() == 16 << 20
    big = W.shrink(W.CONFIGS[3], 8192)                     # several splits per (sequence, KV head)
    small = W.shrink(W.CONFIGS[2], 2048)                   # a smaller input right behind it, another shape
    run_both(big)
    run_both(small)
    run_both(big)                                          # and back: the array is cleared per call
    run_both(W.CONFIGS[1])                                 # fp32: the vector-ALU kernels and their merge launch
    # a 24-node draft tree: the many-rows kernel, whose splits meet through the same words of the array
    run_both(dataclasses.replace(W.shrink(W.CONFIGS[3], 8192), name="cfg3_8k_tree24", gamma=24, tree_depth=4))
    run_both(small)


def test_static_workspace_entry_point_refuses_what_does_not_fit():
    cfg = W.shrink(W.CONFIGS[3], 4096)
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x))
    run.block_reps().score_select().sync()
    g = run.x
    huge = S.make_shape(B=cfg.B, gamma=64, Hq=cfg.Hq * 4, Hkv=cfg.Hkv, d=cfg.d, dtype="f32", block_size=cfg.block_size,
                        max_seq_len=cfg.T, k_blocks=cfg.k_blocks, k_pool=g["k_pool"], page_size=cfg.page_size,
                        max_pages_per_seq=g["block_table"].shape[1])
    assert S.svf_workspace_bytes(huge) > S.svf_static_workspace_bytes()
    with pytest.raises(S.SvfError) as e:
        S.svf_verify_attn_static_ws(huge, g["q"], g["k_pool"], g["v_pool"], g["block_table"], g["seq_lens"],
                                    g["k_draft"], g["v_draft"], g["draft_mask"], run.sel_idx, run.sel_cnt, run.out)
    assert e.value.code == -6
