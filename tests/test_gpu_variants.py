"""GPU parity of the retrieval variants (min/max block summaries, bf16 summaries, group maximum,
top-N over all KV heads of a sequence), through the C ABI, against the variants oracle on the same
seeded inputs.  Bars: min/max summaries bit-exact (they are keys of the cache); mean summaries
1e-5 in fp32 and one bf16 unit in the last place in bf16 (the device rounds its fp32 mean, the
oracle its fp64 mean); scores 1e-4 (2e-3 where bf16 mean summaries may differ by that unit);
kept blocks bit-exact apart from counted near-ties (relative score gap 1e-3); attention as in the
main parity tests."""
import numpy as np
import pytest
import torch

import paper_2512_21911_amd as S
import workloads as W
from oracle import svf_oracle as O
from oracle import svf_variants_oracle as V
from svf_harness import REPS_TOL, TIE_GAP, DeviceRun, check_attn, check_selection, oracle_attn, shape_for, to_gpu

pytestmark = pytest.mark.gpu

MEAN, MINMAX = S.SVF_SUMMARY_MEAN, S.SVF_SUMMARY_MINMAX
F32, BF16 = S.SVF_F32, S.SVF_BF16
GMEAN, GMAX = S.SVF_GROUP_MEAN, S.SVF_GROUP_MAX
PER_HEAD, GLOBAL = S.SVF_BUDGET_PER_HEAD, S.SVF_BUDGET_GLOBAL


def small(**kw):
    base = dict(name="variants_small", cfg_id=21, dtype="f32", B=3, Hq=8, Hkv=2, d=64, T=1500, block_size=16, gamma=4,
                k_blocks=9, page_size=8, planted=4, shift=1.5, min_len=300)
    base.update(kw)
    return W.VerifyConfig(**base)


def oracle_summaries(cfg, x, summary, sdtype):
    """The oracle's summaries, rounded to the storage type: (mean,) or (min, max)."""
    if summary == MEAN:
        reps = O.block_reps(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
        return (V.round_bf16(reps) if sdtype == BF16 else reps,)
    mn, mx = V.block_minmax(x["k_pool"], x["block_table"], x["seq_lens"], cfg.block_size, cfg.nb_max)
    return (V.round_bf16(mn), V.round_bf16(mx)) if sdtype == BF16 else (mn, mx)


def check_summaries(cfg, x, got, ref, summary, sdtype):
    got = got.double().cpu().numpy()
    lens = x["seq_lens"].tolist()
    off = 0
    for b, L in enumerate(lens):
        nb = -(-L // cfg.block_size)
        if nb == 0:
            continue
        if summary == MINMAX:
            np.testing.assert_array_equal(got[b, :, :nb, 0], ref[0][b, :, :nb])
            np.testing.assert_array_equal(got[b, :, :nb, 1], ref[1][b, :, :nb])
        elif sdtype == F32:
            err = np.abs(got[b, :, :nb] - ref[0][b, :, :nb]) / np.maximum(1.0, np.abs(ref[0][b, :, :nb]))
            assert err.max() <= REPS_TOL
        else:
            r = ref[0][b, :, :nb]
            ulp = 2.0 ** (np.floor(np.log2(np.maximum(np.abs(r), 1e-30))) - 7)
            d = np.abs(got[b, :, :nb] - r)
            assert (d <= ulp * 1.0001).all(), "bf16 mean summary off by more than one unit in the last place"
            off += int((d > 0).sum())
    return off


def check_global_selection(cfg, x, scores_ref, idx_gpu, cnt_gpu, n_total, stride):
    idx_ref, cnt_ref = V.select_global(scores_ref, x["seq_lens"], cfg.block_size, n_total, stride, cfg.n_sink, cfg.n_local)
    idx_g, cnt_g = idx_gpu.cpu().numpy(), cnt_gpu.cpu().numpy()
    near = 0
    for b, L in enumerate(x["seq_lens"].tolist()):
        nb = -(-L // cfg.block_size)
        assert cnt_g[b].sum() == min(n_total, cfg.Hkv * nb)
        for h in range(cfg.Hkv):
            g = idx_g[b, h, :cnt_g[b, h]]
            assert (np.diff(g) > 0).all() and (idx_g[b, h, cnt_g[b, h]:] == -1).all()
            assert cnt_g[b, h] == 0 or (g.min() >= 0 and g.max() < nb)
        kept_g = {(h, int(j)) for h in range(cfg.Hkv) for j in idx_g[b, h, :cnt_g[b, h]]}
        kept_r = {(h, int(j)) for h in range(cfg.Hkv) for j in idx_ref[b, h, :cnt_ref[b, h]]}
        if kept_g != kept_r:
            ties = set(V.near_tie_pairs(scores_ref[b], nb, idx_ref[b], cnt_ref[b], TIE_GAP, cfg.n_sink, cfg.n_local))
            diff = kept_g ^ kept_r
            assert diff <= ties, f"sequence {b}: {sorted(diff)} are not near-ties"
            near += len(diff)
    return near


def run_variant(cfg, summary, sdtype, group, budget, n_total=0, stride=None, x=None, attn=True):
    x = W.make_layer(cfg) if x is None else x
    k_row = cfg.k_blocks if stride is None else stride
    shape = shape_for(cfg, x, k_blocks=k_row)
    run = DeviceRun(cfg, to_gpu(x), shape=shape)
    rt = S.SvfRetrieval(summary, sdtype, group, budget, n_total)
    rows = 2 if summary == MINMAX else 1
    tdt = torch.bfloat16 if sdtype == BF16 else torch.float32
    summ = torch.full((cfg.B, cfg.Hkv, cfg.nb_max, rows, cfg.d), float("nan"), device="cuda", dtype=tdt)
    xg = run.x
    S.svf_block_summaries(shape, rt, xg["k_pool"], xg["block_table"], xg["seq_lens"], summ)
    S.svf_retrieve(shape, rt, xg["q"], summ, xg["seq_lens"], run.sel_idx, run.sel_cnt, run.ws, run.scores)
    if attn:
        run.verify_attn()
    run.sync()

    ref = oracle_summaries(cfg, x, summary, sdtype)
    off = check_summaries(cfg, x, summ if summary == MINMAX else summ[:, :, :, 0], ref, summary, sdtype)
    if summary == MEAN:
        s_head = V.head_scores(x["q"], reps=ref[0])
    else:
        s_head = V.head_scores(x["q"], mn=ref[0], mx=ref[1])
    scores_ref = V.group_scores(s_head, cfg.Hkv, V.GROUP_MAX if group == GMAX else V.GROUP_MEAN)
    got = run.scores.double().cpu().numpy()
    tol = 2e-3 if (summary == MEAN and sdtype == BF16) else 1e-4
    for b, L in enumerate(x["seq_lens"].tolist()):
        nb = -(-L // cfg.block_size)
        err = np.abs(got[b, :, :nb] - scores_ref[b, :, :nb]) / np.maximum(1.0, np.abs(scores_ref[b, :, :nb]))
        assert nb == 0 or err.max() <= tol, f"scores b={b}: {err.max():.3e}"
        assert (got[b, :, nb:] == 0).all()
    if budget == PER_HEAD:
        _, _, near = check_selection(cfg, x, scores_ref, run.sel_idx, run.sel_cnt, cfg.n_sink, cfg.n_local, k_row)
    else:
        near = check_global_selection(cfg, x, scores_ref, run.sel_idx, run.sel_cnt, n_total, k_row)
    err = None
    if attn:
        out_ref, lse_ref = oracle_attn(cfg, x, run.sel_idx.cpu(), run.sel_cnt.cpu())
        err = check_attn(cfg, run.out, run.lse, out_ref, lse_ref)
    print(f"[variants] {cfg.name} summary={summary} dtype={sdtype} group={group} budget={budget}: "
          f"near_ties={near} bf16_last_place={off} attn_err={err}", flush=True)
    return run, x, scores_ref


COMBOS = [(MINMAX, F32, GMEAN, PER_HEAD), (MINMAX, BF16, GMAX, PER_HEAD), (MEAN, BF16, GMEAN, PER_HEAD),
          (MEAN, F32, GMAX, PER_HEAD), (MEAN, F32, GMEAN, GLOBAL), (MINMAX, F32, GMAX, GLOBAL),
          (MEAN, BF16, GMAX, GLOBAL)]


@pytest.mark.parametrize("summary,sdtype,group,budget", COMBOS)
def test_small_fp32_paged_ragged(summary, sdtype, group, budget):
    cfg = small()
    n_total = 20 if budget == GLOBAL else 0
    run_variant(cfg, summary, sdtype, group, budget, n_total, stride=20 if budget == GLOBAL else None)


@pytest.mark.parametrize("summary,sdtype,group,budget", COMBOS)
def test_cfg3_shape_shrunk(summary, sdtype, group, budget):
    """bf16 cache, d = 128, pages of 16, four sequences: the benchmark's shape with a shorter prefix; the
    global budget is the per-head budget times the KV heads (Eq. 6)."""
    cfg = W.shrink(W.CONFIGS[3], 8192)
    n_total = cfg.k_blocks * cfg.Hkv if budget == GLOBAL else 0
    run_variant(cfg, summary, sdtype, group, budget, n_total, stride=min(cfg.nb_max, n_total) if budget == GLOBAL else None)


def test_defaults_are_the_main_path_bit_for_bit():
    cfg = small(dtype="bf16", d=128, Hq=8, Hkv=2)
    x = W.make_layer(cfg)
    run = DeviceRun(cfg, to_gpu(x))
    run.block_reps().score_select().sync()
    rt = S.SvfRetrieval(MEAN, F32, GMEAN, PER_HEAD, 0)
    summ = torch.full_like(run.reps, float("nan"))
    idx, cnt, sc = torch.full_like(run.sel_idx, -7), torch.full_like(run.sel_cnt, -7), torch.full_like(run.scores, 7.0)
    S.svf_block_summaries(run.shape, rt, run.x["k_pool"], run.x["block_table"], run.x["seq_lens"], summ)
    S.svf_retrieve(run.shape, rt, run.x["q"], summ, run.x["seq_lens"], idx, cnt, run.ws, sc)
    torch.cuda.synchronize()
    lens = x["seq_lens"].tolist()
    for b, L in enumerate(lens):
        nb = -(-L // cfg.block_size)
        assert torch.equal(summ[b, :, :nb].view(torch.int32), run.reps[b, :, :nb].view(torch.int32))
    assert torch.equal(idx, run.sel_idx) and torch.equal(cnt, run.sel_cnt)
    assert torch.equal(sc.view(torch.int32), run.scores.view(torch.int32))


def test_global_with_one_kv_head_is_the_per_head_rule():
    cfg = small(Hq=4, Hkv=1, k_blocks=7)
    x = W.make_layer(cfg)
    run_g, _, _ = run_variant(cfg, MEAN, F32, GMEAN, GLOBAL, 7, stride=7, x=x, attn=False)
    run_p = DeviceRun(cfg, to_gpu(x))
    run_p.block_reps().score_select().sync()
    assert torch.equal(run_g.sel_idx, run_p.sel_idx) and torch.equal(run_g.sel_cnt, run_p.sel_cnt)


def test_group_of_one_and_of_sixteen():
    """One query head per KV head (mean and maximum coincide) and sixteen (two rounds of staged heads)."""
    cfg1 = small(Hq=2, Hkv=2)
    x = W.make_layer(cfg1)
    a, _, _ = run_variant(cfg1, MINMAX, F32, GMEAN, PER_HEAD, x=x, attn=False)
    b, _, _ = run_variant(cfg1, MINMAX, F32, GMAX, PER_HEAD, x=x, attn=False)
    assert torch.equal(a.scores.view(torch.int32), b.scores.view(torch.int32))
    cfg16 = small(Hq=32, Hkv=2, d=128, dtype="bf16", block_size=32, page_size=16, T=2048, k_blocks=8)
    run_variant(cfg16, MINMAX, BF16, GMEAN, PER_HEAD)
    run_variant(cfg16, MEAN, F32, GMAX, GLOBAL, 16, stride=16)


def test_sink_local_and_budget_beyond_all_pairs():
    cfg = small(n_sink=1, n_local=2, k_blocks=9)
    run_variant(cfg, MINMAX, F32, GMAX, GLOBAL, 24, stride=24)
    # budget larger than the pairs there are: every block of every head is kept
    cfg2 = small(T=400, min_len=100, k_blocks=25)
    run, x, _ = run_variant(cfg2, MEAN, F32, GMEAN, GLOBAL, 10 ** 6, stride=25)
    for b, L in enumerate(x["seq_lens"].tolist()):
        assert (run.sel_cnt[b].cpu().numpy() == -(-L // cfg2.block_size)).all()


def test_many_blocks_and_an_empty_sequence():
    """More blocks per head than the selecting workgroup has threads (several sweeps), and a sequence
    without any prefix in the batch."""
    cfg = small(T=20000, block_size=8, page_size=8, min_len=17000, k_blocks=40, B=2, planted=6)
    run_variant(cfg, MEAN, F32, GMAX, GLOBAL, 64, stride=64, attn=False)
    cfg2 = small()
    x = W.make_layer(cfg2)
    x["seq_lens"][1] = 0
    run, _, _ = run_variant(cfg2, MINMAX, BF16, GMEAN, GLOBAL, 20, stride=20, x=x)
    assert (run.sel_cnt[1] == 0).all() and (run.sel_idx[1] == -1).all()
