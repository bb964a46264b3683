"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Selected block ids are bit-exact apart from counted near-ties (relative score gap 1e-3);
outputs within max-abs 2e-2 (bf16) / 1e-4 (fp32); representatives within 1e-5."""
import dataclasses

import numpy as np
import pytest
import torch

import paper_2512_21911_amd as S
import workloads as W
from oracle import svf_oracle as O
from svf_harness import (LSE_TOL, OUT_TOL, DeviceRun, check_attn, check_reps, check_selection, full_parity,
                         oracle_attn, shape_for, to_gpu)

pytestmark = pytest.mark.gpu


def report(name, r):
    print(f"[parity] {name}: max_abs_err={r['max_abs_err']:.3e} near_ties={r['near_ties']}", flush=True)


# ------------------------------------------------------------------ the five configurations

def test_cfg1_tiny_fp32():
    r = full_parity(W.CONFIGS[1])
    report("cfg1", r)
    x, run = r["x"], r["run"]
    idx = run.sel_idx.cpu().numpy()
    for h in range(2):
        assert set(x["planted"][0][h].tolist()) <= set(idx[0, h].tolist())
    assert r["near_ties"] == 0


def test_cfg2_llama8b_bf16():
    r = full_parity(W.CONFIGS[2])
    report("cfg2", r)
    idx = r["run"].sel_idx.cpu().numpy()
    for h in range(8):
        assert set(r["x"]["planted"][0][h].tolist()) <= set(idx[0, h].tolist())


@pytest.mark.parametrize("cfg_id,T", [(3, 4096), (4, 16384), (5, 8192)])
def test_shrunk_paged_configs(cfg_id, T):
    cfg = W.shrink(W.CONFIGS[cfg_id], T)
    r = full_parity(cfg)
    report(f"cfg{cfg_id}@T={T}", r)


@pytest.mark.parametrize("cfg_id", [3, 4, 5])
def test_full_size_configs(cfg_id):
    """One layer at the benchmark's full shape, in the launch configuration the bench times."""
    cfg = W.CONFIGS[cfg_id]
    r = full_parity(cfg)
    report(f"cfg{cfg_id} full", r)
    if cfg_id == 4:   # more planted blocks than budget: everything kept must be planted
        idx = r["run"].sel_idx.cpu().numpy()
        for h in range(cfg.Hkv):
            assert set(idx[0, h].tolist()) <= set(r["x"]["planted"][0][h].tolist())


def test_tree60_over_the_full_size_cache():
    """A 60-node draft tree (Sec. 4.1's EAGLE-3 runs) over cfg 3's cache: the many-rows kernel at the
    shape `bench.py --tree 60` times."""
    cfg = dataclasses.replace(W.CONFIGS[3], name="cfg3_tree60", gamma=60, tree_depth=6, n_layers=1)
    r = full_parity(cfg)
    report("cfg3 cache, 60-node tree", r)


def test_cfg3_reuse_layer_matches_anchor_blocks():
    """Eq. 9: the non-anchor layer attends with the anchor's block set."""
    cfg = W.shrink(W.CONFIGS[3], 4096)
    x0 = W.make_layer(cfg, 0)
    x1 = W.make_layer(cfg, 1)
    run0 = DeviceRun(cfg, to_gpu(x0))
    run0.block_reps().verify_step(True).sync()
    idx0, cnt0 = run0.sel_idx.clone(), run0.sel_cnt.clone()
    run1 = DeviceRun(cfg, to_gpu(x1))
    run1.sel_idx.copy_(idx0)
    run1.sel_cnt.copy_(cnt0)
    run1.verify_step(S.SVF_STEP_REUSE).sync()            # own workspace: nothing of the anchor call in it
    assert torch.equal(run1.sel_idx, idx0)
    ref, lse = oracle_attn(cfg, x1, idx0.cpu(), cnt0.cpu())
    check_attn(cfg, run1.out, run1.lse, ref, lse)
    # with the anchor call's workspace the gather list is reused on this layer's pools: same bits
    out_plain = run1.out.clone()
    run1.out.fill_(float("nan"))
    run1.ws = run0.ws
    run1.verify_step(S.SVF_STEP_REUSE_GATHER).sync()
    assert torch.equal(run1.out.view(torch.int16), out_plain.view(torch.int16))
    # and it is bit-identical to svf_verify_attn with the same indices
    out_step = run1.out.clone()
    run1.out.fill_(float("nan"))
    run1.verify_attn().sync()
    assert torch.equal(out_step.view(torch.int16), run1.out.view(torch.int16))


def test_cfg5_groups_of_four_reuse_schedule():
    """cfg 5's schedule at a shorter context: 8 layers, anchors every 4th, ragged lengths, B = 8,
    Hkv = 4.  One workspace and one sel_idx / sel_cnt serve the whole step, as in a model: an anchor
    layer retrieves, the three layers behind it attend through its gather list (Eq. 9).  Every layer
    is checked against the oracle with the oracle's blocks of the nearest preceding anchor."""
    cfg = W.shrink(W.CONFIGS[5], 8192, n_layers=8)
    assert cfg.anchor_every == 4 and cfg.min_len > 0
    xs = [W.make_layer(cfg, l) for l in range(cfg.n_layers)]
    lens = xs[0]["seq_lens"].tolist()
    assert len(set(lens)) > 1 and any(L % cfg.block_size for L in lens)
    run = DeviceRun(cfg, to_gpu(xs[0]))
    near = 0
    idx_ref = cnt_ref = None
    for l, x in enumerate(xs):
        run.x = to_gpu(x)
        run.out.fill_(float("nan"))
        run.lse.fill_(float("nan"))
        anchor = cfg.is_anchor(l)
        if anchor:
            run.block_reps()
            run.sel_idx.fill_(-7)
            run.sel_cnt.fill_(-7)
        run.verify_step(S.SVF_STEP_ANCHOR if anchor else S.SVF_STEP_REUSE_GATHER).sync()
        if anchor:
            scores_ref = O.block_scores(x["q"], check_reps(cfg, x, run.reps))
            idx_ref, cnt_ref, n = check_selection(cfg, x, scores_ref, run.sel_idx, run.sel_cnt)
            near += n
            kept = (run.sel_idx.cpu(), run.sel_cnt.cpu())     # the oracle's unless near-ties occurred
        else:
            assert torch.equal(run.sel_idx.cpu(), kept[0]) and torch.equal(run.sel_cnt.cpu(), kept[1])
        ref, lse = oracle_attn(cfg, x, kept[0], kept[1])
        err = check_attn(cfg, run.out, run.lse, ref, lse)
        print(f"[cfg5 schedule] layer {l} ({'anchor' if anchor else 'reuse'}): max_abs_err={err:.3e}", flush=True)
        # the same layer through svf_verify_attn (no gather list) gives the same bits
        out_step = run.out.clone()
        run.out.fill_(float("nan"))
        run.verify_attn().sync()
        assert torch.equal(out_step.view(torch.int16), run.out.view(torch.int16))
    print(f"[cfg5 schedule] near-ties excused: {near}", flush=True)


def test_row_without_a_visible_key_is_zero():
    """A sequence with no kept block and a draft mask that lacks a row's own bit: nothing to attend
    to.  Every kernel and every split count gives out = 0 and lse = -inf for that row (the oracle's
    reading), ordinary rows beside it."""
    for cfg in (small(B=1, gamma=4), small(B=1, gamma=4, k_blocks=16), small(B=1, gamma=4, dtype="f32", d=64)):
        x = W.make_layer(cfg)
        x["draft_mask"] = W.masks_to_tensor([0b0000, 0b0011, 0b0100, 0b1111])
        run = DeviceRun(cfg, to_gpu(x))
        run.sel_idx.fill_(-1)
        run.sel_cnt.fill_(0)
        run.verify_attn().sync()
        ref, lse = oracle_attn(cfg, x, run.sel_idx.cpu(), run.sel_cnt.cpu())
        out = run.out.double().cpu().numpy()
        assert (out[:, 0] == 0).all() and np.isneginf(run.lse.cpu().numpy()[:, 0]).all()
        assert np.isfinite(out).all()
        assert np.abs(out - ref).max() <= OUT_TOL[cfg.dtype]
        assert np.abs(run.lse.double().cpu().numpy()[:, 1:] - lse[:, 1:]).max() <= LSE_TOL[cfg.dtype]
        # and beside kept blocks (several splits): the masked row only sees the cache
    cfg = small(B=1, gamma=4, k_blocks=8)
    x = W.make_layer(cfg)
    x["draft_mask"] = W.masks_to_tensor([0b0000, 0b0011, 0b0100, 0b1111])
    r = full_parity(cfg, x=x)
    report("mask without own bit", r)


# ------------------------------------------------------------------ edge cases

def small(dtype="bf16", **kw):
    base = dict(name="edge", cfg_id=9, dtype=dtype, B=2, Hq=8, Hkv=2, d=128, T=1024, block_size=64, gamma=4,
                k_blocks=4, page_size=16, planted=2, shift=1.5)
    base.update(kw)
    return W.VerifyConfig(**base)


EDGE = {
    "ragged_lengths": small(min_len=100),
    "dense_budget": small(k_blocks=16),
    "budget_above_blocks": small(k_blocks=40, min_len=300),
    "gamma1_decode": small(gamma=1),
    "gamma64_chain": small(gamma=64, B=1),
    "tree16": small(gamma=16, tree_depth=4),
    "sink_local": small(n_sink=1, n_local=2, k_blocks=5, min_len=500),
    "block16_page64": small(block_size=16, page_size=64, k_blocks=12),
    "block48_contig": small(block_size=48, page_size=0, T=1000, min_len=700, k_blocks=5),
    "block128_page16": small(block_size=128, page_size=16, k_blocks=3),
    "d64_bf16": small(d=64),
    "f32_d128": small(dtype="f32"),
    "f32_d64_paged": small(dtype="f32", d=64, min_len=64),
    "gqa8": small(Hq=16, Hkv=2, gamma=6),
    "mha": small(Hq=4, Hkv=4, gamma=3),
    # two draft tiles (more than 32 drafts) in the one-row-group-per-workgroup kernel
    "mha_gamma40": small(Hq=2, Hkv=2, gamma=40),
    "mha_gamma33_tree": small(Hq=2, Hkv=2, gamma=33, tree_depth=5, B=3, min_len=300),
    "short_seq": small(T=40, page_size=8, block_size=16, k_blocks=2),
    # the anchor kernel's own retrieval: sixteen query heads per KV head (more than one batch of
    # head loads), a second selection key per thread (more than 512 blocks), a page table too long
    # to be staged in LDS, two row groups
    "gqa16": small(Hq=32, Hkv=2, gamma=2),
    "blocks_768": small(B=1, Hq=4, Hkv=1, T=49152, k_blocks=24, planted=5, min_len=40000),
    "long_page_table": small(B=1, Hq=4, Hkv=1, T=20480, page_size=4, k_blocks=8, planted=3),
    "two_row_groups": small(Hq=16, Hkv=2, gamma=7, n_sink=1, n_local=1),
    # a page-table row whose length is no multiple of four entries (staged entry by entry)
    "page_table_63_entries": small(T=1000, min_len=600, k_blocks=5),
    # more than two row groups of 32 query rows: one workgroup walks the tiles for up to eight row groups
    "rows_gamma24_tree": small(gamma=24, tree_depth=5),
    "rows_ring_of_stages": small(B=8, Hq=32, Hkv=8, gamma=24, T=4096, k_blocks=32, tree_depth=4, min_len=3000),
    "rows_single_split": small(B=32, Hq=32, Hkv=8, gamma=20, T=1024, k_blocks=4),
    "rows_gamma60_tree": small(gamma=60, tree_depth=6, T=4096, k_blocks=16, n_sink=1, n_local=1),
    "rows_two_sets_of_eight": small(B=1, Hq=16, Hkv=2, gamma=64, T=2048, k_blocks=8),
    # shapes that leave the fused path: more than 1024 blocks (two retrieval kernels + gather list),
    # more than 1024 kept blocks (no gather list)
    "blocks_2048": small(B=1, Hq=4, Hkv=1, T=32768, block_size=16, k_blocks=40, planted=6),
    "budget_1500_blocks": small(B=1, Hq=4, Hkv=1, T=8192, block_size=4, page_size=4, k_blocks=1500, planted=20),
}


@pytest.mark.parametrize("name", sorted(EDGE))
def test_edge_case(name):
    r = full_parity(EDGE[name])
    report(name, r)


def test_empty_sequence_in_a_batch():
    """A sequence with no prefix attends to its drafts only; its neighbours are unaffected."""
    cfg = small(B=3, min_len=100)
    x = W.make_layer(cfg)
    x["seq_lens"][1] = 0
    r = full_parity(cfg, x=x)
    assert r["run"].sel_cnt.cpu().tolist()[1] == [0, 0]
    report("empty sequence", r)


def test_hnd_strides_and_scale():
    """Head-major pages ([page][Hkv][slot][d]) through the stride fields, and an explicit softmax scale."""
    cfg = small(min_len=400)
    x = W.make_layer(cfg)
    xg = to_gpu(x)
    for key in ("k_pool", "v_pool"):
        hnd = xg[key].permute(0, 2, 1, 3).contiguous()          # storage [page][Hkv][slot][d]
        xg[key + "_store"] = hnd
        xg[key] = hnd.permute(0, 2, 1, 3)                        # logical view, strides carry the layout
    shape = shape_for(cfg, xg, sm_scale=0.05)
    assert shape.kv_stride_head == cfg.page_size * cfg.d and shape.kv_stride_tok == cfg.d
    run = DeviceRun(cfg, xg, shape)
    run.block_reps().score_select().verify_attn().sync()
    ref = check_reps(cfg, x, run.reps)
    check_selection(cfg, x, O.block_scores(x["q"], ref), run.sel_idx, run.sel_cnt)
    out_ref, lse_ref = oracle_attn(cfg, x, run.sel_idx.cpu(), run.sel_cnt.cpu(), sm_scale=0.05)
    check_attn(cfg, run.out, run.lse, out_ref, lse_ref)


def test_per_batch_masks_and_null_mask():
    cfg = small(gamma=5)
    x = W.make_layer(cfg)
    xg = to_gpu(x)
    masks = torch.tensor([[1, 3, 5, 9, 19], [1, 3, 7, 15, 31]], dtype=torch.int64)
    run = DeviceRun(cfg, xg, shape_for(cfg, xg, mask_per_batch=1))
    run.block_reps().score_select().verify_attn(mask=masks.cuda()).sync()
    ref, lse = oracle_attn(cfg, x, run.sel_idx.cpu(), run.sel_cnt.cpu(), mask=masks)
    check_attn(cfg, run.out, run.lse, ref, lse)
    run2 = DeviceRun(cfg, xg)
    run2.block_reps().score_select().verify_attn(mask=None).sync()     # NULL mask = linear causal
    ref2, lse2 = oracle_attn(cfg, x, run2.sel_idx.cpu(), run2.sel_cnt.cpu(), mask=None)
    check_attn(cfg, run2.out, run2.lse, ref2, lse2)


def test_incremental_block_reps():
    """Representatives of a block range only: other rows stay untouched."""
    cfg = small()
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x), poison=False)
    run.reps.fill_(123.0)
    run.block_reps(first_block=5, n_blocks=3).sync()
    ref = O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
    got = run.reps.cpu().double().numpy()
    assert np.abs(got[:, :, 5:8] - ref[:, :, 5:8]).max() < 1e-5
    assert (got[:, :, :5] == 123.0).all() and (got[:, :, 8:] == 123.0).all()


def test_exact_ties_lowest_index_wins():
    """All representatives equal => every score ties => blocks 0..k-1 (after forced ones)."""
    cfg = small(n_sink=0, n_local=1, k_blocks=4)
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x), poison=False)
    run.reps.fill_(0.25)
    run.score_select().sync()
    idx = run.sel_idx.cpu().numpy()
    assert (idx == np.array([0, 1, 2, 15])).all()
    run.reps.fill_(0.0)                      # +0 / -0 scores must tie as well
    run.score_select().sync()
    assert (run.sel_idx.cpu().numpy() == np.array([0, 1, 2, 15])).all()


@pytest.mark.parametrize("T,n_sink,n_local", [(32768, 0, 0), (65536, 0, 0), (65536, 1, 2), (40000, 2, 1)])
def test_ties_in_the_anchor_launch_lowest_index_wins(T, n_sink, n_local):
    """Sec. 3.1 top-N rule with equal scores (the lowest block index wins), through the retrieval
    that runs inside the anchor layer's attention launch: 512 and up to 1024 blocks (one and two
    keys per thread of the selecting workgroup), all scores equal and scores equal in runs.  The
    ids must be those of svf_score_select on the same representatives, and for all-equal scores
    the closed form: forced blocks, then the lowest indices."""
    cfg = W.CONFIGS[3].scaled(T=T, n_sink=n_sink, n_local=n_local)
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x), poison=False)
    nb = -(-T // cfg.block_size)
    k = run.shape.k_blocks
    # (a) every score ties
    run.reps.fill_(0.25)
    run.verify_step(S.SVF_STEP_ANCHOR).sync()
    forced = list(range(n_sink)) + list(range(nb - n_local, nb))
    free = [j for j in range(nb) if j not in forced][: k - len(forced)]
    want = np.array(sorted(forced + free), dtype=np.int32)
    got = run.sel_idx.cpu().numpy()
    assert (got == want[None, None, :]).all()
    assert (run.sel_cnt.cpu().numpy() == k).all()
    # (b) runs of equal scores: representative j = level(j) in every channel, so that the score is
    # level(j) x (sum of the mean query's channels); whatever that sum's sign, ties abound and the
    # threshold falls inside a run
    levels = torch.tensor([((j * 7) % 5) * 0.125 for j in range(cfg.nb_max)], device="cuda")
    run.reps.copy_(levels[None, None, :, None].expand_as(run.reps))
    run.verify_step(S.SVF_STEP_ANCHOR).sync()
    fused_idx, fused_cnt = run.sel_idx.clone(), run.sel_cnt.clone()
    run.score_select().sync()
    assert torch.equal(fused_idx, run.sel_idx) and torch.equal(fused_cnt, run.sel_cnt)
    sc = run.scores.cpu().double().numpy()
    idx, cnt = O.select_blocks(sc, x["seq_lens"], cfg.block_size, cfg.k_blocks, n_sink, n_local)
    assert (fused_idx.cpu().numpy() == idx).all() and (fused_cnt.cpu().numpy() == cnt).all()


# ------------------------------------------------------------------ properties that hold at any size

def test_constant_values_give_constant_output():
    cfg = W.shrink(W.CONFIGS[3], 4096)
    x = W.make_layer(cfg)
    x["v_pool"] = torch.full_like(x["v_pool"], 0.375)
    x["v_draft"] = torch.full_like(x["v_draft"], 0.375)
    run = DeviceRun(cfg, to_gpu(x))
    run.block_reps().score_select().verify_attn().sync()
    out = run.out.float().cpu()
    assert (out - 0.375).abs().max() <= 0.375 * 2 ** -8        # one bf16 ulp


def test_unselected_block_cannot_influence_output():
    cfg = W.shrink(W.CONFIGS[3], 4096)
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x))
    run.block_reps().score_select().verify_attn().sync()
    out0, idx0 = run.out.clone(), run.sel_idx.clone()
    # overwrite V of one unselected block per (b, h) with large noise
    idx = idx0.cpu().numpy()
    table = x["block_table"]
    g = torch.Generator().manual_seed(5)
    v2 = x["v_pool"].clone()
    for b in range(cfg.B):
        for h in range(cfg.Hkv):
            j = next(j for j in range(cfg.nb_max) if j not in set(idx[b, h].tolist()))
            for t in range(j * cfg.block_size, (j + 1) * cfg.block_size):
                pg = int(table[b, t // cfg.page_size])
                v2[pg, t % cfg.page_size, h] = (torch.randn(cfg.d, generator=g) * 100).to(v2.dtype)
    run.x["v_pool"] = v2.cuda()
    run.out.fill_(float("nan"))
    run.verify_attn().sync()
    assert torch.equal(run.sel_idx, idx0)
    assert torch.equal(run.out.view(torch.int16), out0.view(torch.int16))


def test_page_permutation_is_invisible():
    """Same logical cache in two physical page orders: identical representatives, ids and outputs."""
    cfg = W.shrink(W.CONFIGS[3], 4096)
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x))
    run.block_reps().score_select().verify_attn().sync()
    n_pages = x["k_pool"].shape[0]
    perm = torch.randperm(n_pages, generator=torch.Generator().manual_seed(3))
    y = dict(x)
    inv = torch.empty_like(perm)
    inv[perm] = torch.arange(n_pages)
    y["k_pool"] = x["k_pool"][perm]
    y["v_pool"] = x["v_pool"][perm]
    y["block_table"] = inv[x["block_table"].long()].to(torch.int32)
    run2 = DeviceRun(cfg, to_gpu(y))
    run2.block_reps().score_select().verify_attn().sync()
    assert torch.equal(run.reps.view(torch.int32), run2.reps.view(torch.int32))
    assert torch.equal(run.sel_idx, run2.sel_idx)
    assert torch.equal(run.out.view(torch.int16), run2.out.view(torch.int16))


def test_repeated_calls_are_bit_stable():
    cfg = W.CONFIGS[2]
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x))
    run.block_reps().score_select().verify_attn().sync()
    out0, idx0 = run.out.clone(), run.sel_idx.clone()
    for _ in range(5):
        run.out.fill_(float("nan"))
        run.verify_step(True).sync()
        assert torch.equal(run.sel_idx, idx0)
        assert torch.equal(run.out.view(torch.int16), out0.view(torch.int16))


def same_bits_whatever_the_wait(cfg):
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x))
    run.block_reps().score_select().verify_attn().sync()
    out0, lse0, idx0, cnt0 = run.out.clone(), run.lse.clone(), run.sel_idx.clone(), run.sel_cnt.clone()
    for polls in (0, 1, 2, 64, -1):
        S.svf_workspace_set_wait_polls(run.shape, run.ws, polls)
        before = S.svf_diag_wait_fallbacks(run.shape, run.ws)
        for rep in range(3):                       # the tag moves on from call to call
            for mode in (S.SVF_STEP_ANCHOR, S.SVF_STEP_REUSE_GATHER, S.SVF_STEP_REUSE):
                run.out.fill_(float("nan"))
                run.lse.fill_(float("nan"))
                if mode == S.SVF_STEP_ANCHOR:
                    run.sel_idx.fill_(-7)
                    run.sel_cnt.fill_(-7)
                run.verify_step(mode).sync()
                assert torch.equal(run.sel_idx, idx0) and torch.equal(run.sel_cnt, cnt0), f"polls={polls} mode={mode}"
                assert torch.equal(run.out.view(torch.int16), out0.view(torch.int16)), f"polls={polls} mode={mode}"
                assert torch.equal(run.lse.view(torch.int32), lse0.view(torch.int32)), f"polls={polls} mode={mode}"
        # the library counts the waits that ran out; without patience every wait between workgroups does
        after = S.svf_diag_wait_fallbacks(run.shape, run.ws)
        assert after[0] >= before[0] and after[1] >= before[1]
        if polls == 0:                             # (every shape tested this way has several splits)
            assert after[1] > before[1], "no merge fallback counted although nobody waits"
            print(f"\n[{cfg.name}] polls=0: exchange fallbacks +{after[0] - before[0]}, merge fallbacks +{after[1] - before[1]}")
        if polls in (64, -1):
            print(f"\n[{cfg.name}] polls={polls}: exchange fallbacks +{after[0] - before[0]}, merge fallbacks +{after[1] - before[1]}")
    # many calls in a row, no host synchronisation in between: tags keep moving, nothing stale is taken
    for polls in (-1, 1):
        S.svf_workspace_set_wait_polls(run.shape, run.ws, polls)
        outs = []
        for i in range(60):
            run.verify_step((S.SVF_STEP_ANCHOR, S.SVF_STEP_REUSE_GATHER, S.SVF_STEP_REUSE)[i % 3])
            outs.append(run.out.clone())
        torch.cuda.synchronize()
        assert torch.equal(run.sel_idx, idx0)
        assert all(torch.equal(o.view(torch.int16), out0.view(torch.int16)) for o in outs), f"polls={polls}"
    # clearing the workspace restores the default budget, a fresh call counter and empty statistics
    S.svf_workspace_init(run.ws)
    torch.cuda.synchronize()
    assert S.svf_diag_wait_fallbacks(run.shape, run.ws) == (0, 0)
    run.verify_step(S.SVF_STEP_ANCHOR).sync()
    assert torch.equal(run.out.view(torch.int16), out0.view(torch.int16))


@pytest.mark.parametrize("cfg_id,T", [(3, 8192), (5, 65536), (4, 131072), (3, 32768), (2, 8192)])
def test_same_bits_whatever_the_workgroups_wait_for_each_other(cfg_id, T):
    """The workgroups of a group wait for each other twice, with a bounded number of polls: for the
    block keys of the shared scoring (anchor layers), and for the split partials before each merges
    its slice of the rows.  A budget of zero or one poll sends some or all of them down the other
    paths (score everything oneself; leave the slice to the workgroup that arrives last): the same
    bits in every step mode, call after call (the tags move on)."""
    same_bits_whatever_the_wait(W.shrink(W.CONFIGS[cfg_id], T) if T < W.CONFIGS[cfg_id].T else W.CONFIGS[cfg_id])


# The kernel for many query rows merges up to 16 splits itself, by the same protocol: nine splits of
# three row groups; four splits of three row groups (a workgroup without a slice); four splits of
# eight row groups (two row groups per slice); eight splits of two sets of eight row groups; the
# 60-node tree over the full-size cache (eight splits of eight row groups).
ROWS_WAIT = {
    "nine_splits": EDGE["rows_gamma24_tree"],
    "more_splits_than_row_groups": EDGE["rows_ring_of_stages"],
    "two_row_groups_per_slice": small(B=8, Hq=32, Hkv=8, gamma=60, tree_depth=6, T=4096, k_blocks=32, min_len=3000),
    "two_sets_of_eight": small(B=8, Hq=16, Hkv=2, gamma=64, T=2048, k_blocks=8),
    "tree60_full_cache": dataclasses.replace(W.CONFIGS[3], name="cfg3_tree60", gamma=60, tree_depth=6, n_layers=1),
}


@pytest.mark.parametrize("name", sorted(ROWS_WAIT))
def test_many_rows_same_bits_whatever_the_workgroups_wait_for_each_other(name):
    same_bits_whatever_the_wait(ROWS_WAIT[name])


def test_budget_helper_matches_oracle():
    for L, L0, rho, bs in [(32768, 4096, 0.1, 64), (4096, 4096, 0.1, 64), (131072, 1024, 0.1, 128), (777, 100, 0.5, 7)]:
        assert S.svf_budget_blocks(L, L0, rho, bs) == O.budget_blocks(L, L0, rho, bs)


@pytest.mark.parametrize("cfg_id,T", [(3, 4096), (3, 32768), (5, 8192), (2, 8192)])
def test_selection_without_scores_takes_one_launch_and_the_same_blocks(cfg_id, T):
    """svf_score_select without the scores output runs the retrieving attention kernel's retrieval alone
    (one launch, key exchange between the workgroups of a pair): same blocks as the two-kernel path, call
    after call, also interleaved with anchor steps on the same workspace (they share the exchange tags)."""
    cfg = W.shrink(W.CONFIGS[cfg_id], T) if T < W.CONFIGS[cfg_id].T else W.CONFIGS[cfg_id]
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x), poison=False)
    run.block_reps().score_select(with_scores=True).sync()
    idx0, cnt0 = run.sel_idx.clone(), run.sel_cnt.clone()
    check_selection(cfg, x, O.block_scores(x["q"], O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"],
                                                                 cfg.block_size, cfg.nb_max)),
                    idx0, cnt0, cfg.n_sink, cfg.n_local)
    try:
        for polls in (64, 0, 1):
            S.svf_workspace_set_wait_polls(run.shape, run.ws, polls)
            for i in range(12):
                run.sel_idx.fill_(-7)
                run.sel_cnt.fill_(-7)
                run.score_select(with_scores=False)
                if i % 4 == 3:
                    run.verify_step(S.SVF_STEP_ANCHOR)
                run.sync()
                assert torch.equal(run.sel_idx, idx0) and torch.equal(run.sel_cnt, cnt0), f"polls={polls} call {i}"
    finally:
        S.svf_workspace_set_wait_polls(run.shape, run.ws, -1)
